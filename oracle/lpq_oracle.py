"""ctypes front end of the CPU oracle in lpq_oracle.c.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  The GPU library and its Python binding never import
this module, and this module imports nothing of theirs.  All arrays are numpy,
host memory.  `build()` compiles the C file with gcc next to it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lpq_oracle.c")
_LIB = os.path.join(_HERE, "liblpq_oracle.so")

MINMAX, ABSMAX, GAUSS = 0, 1, 2
PER_FEATURE, GLOBAL, SHARED_WIDTH = 0, 1, 2
L2SQ, IP = 0, 1

_CALIB = {"minmax": MINMAX, "absmax": ABSMAX, "gauss": GAUSS, "quantile": 3}
_SCOPE = {"per_feature": PER_FEATURE, "global": GLOBAL, "shared_width": SHARED_WIDTH}
_METRIC = {"l2sq": L2SQ, "ip": IP}


def build(force: bool = False) -> str:
    """Compile lpq_oracle.c into liblpq_oracle.so (plain gcc -O2, no intrinsics)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = C.CDLL(build())
        f32p, i8p, i32p = C.POINTER(C.c_float), C.POINTER(C.c_int8), C.POINTER(C.c_int32)
        lib.lpqo_derive_m.argtypes = [f32p, f32p, C.c_int, C.c_int, f32p]
        lib.lpqo_derive_m.restype = None
        lib.lpqo_calibrate.argtypes = [f32p, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_int,
                                       C.c_int, C.c_double, f32p, f32p, f32p, f32p]
        lib.lpqo_calibrate.restype = C.c_int
        lib.lpqo_encode.argtypes = [f32p, C.c_int64, C.c_int64, C.c_int, C.c_int, f32p, f32p,
                                    f32p, f32p, i8p, C.c_int64, i32p]
        lib.lpqo_encode.restype = None
        lib.lpqo_dist_l2sq.argtypes = [i8p, i8p, C.c_int]
        lib.lpqo_dist_l2sq.restype = C.c_int32
        lib.lpqo_dist_ip.argtypes = [i8p, i8p, C.c_int]
        lib.lpqo_dist_ip.restype = C.c_int32
        lib.lpqo_search_i8.argtypes = [i8p, C.c_int64, C.c_int64, i8p, C.c_int64, C.c_int64,
                                       C.c_int, C.c_int, C.c_int, i32p, i32p, C.c_int]
        lib.lpqo_search_i8.restype = C.c_int
        lib.lpqo_search_f32.argtypes = [f32p, C.c_int64, C.c_int64, f32p, C.c_int64, C.c_int64,
                                        C.c_int, C.c_int, C.c_int, i32p, f32p, C.c_int]
        lib.lpqo_search_f32.restype = C.c_int
        lib.lpqo_recall.argtypes = [i32p, i32p, C.c_int64, C.c_int]
        lib.lpqo_recall.restype = C.c_double
        lib.lpqo_max_threads.argtypes = []
        lib.lpqo_max_threads.restype = C.c_int
        _lib = lib
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(C.POINTER(ct))


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _mat(a, dtype):
    a = np.asarray(a)
    if a.dtype != dtype or a.ndim != 2 or a.strides[1] != a.itemsize or a.strides[0] % a.itemsize:
        a = np.ascontiguousarray(a, dtype=dtype)
    return a, a.strides[0] // a.itemsize


class Quantizer:
    """The constants (k, S_b, S_e) of Equation 1 per feature, and the derived m."""

    def __init__(self, d: int, bits: int = 8):
        assert d >= 1 and 1 <= bits <= 8
        self.d, self.bits = d, bits
        self.k = np.zeros(d, np.float32)
        self.sb = np.zeros(d, np.float32)
        self.se = np.zeros(d, np.float32)
        self.m = np.zeros(d, np.float32)

    def set_params(self, k, sb, se):
        self.k, self.sb, self.se = _f32(k).copy(), _f32(sb).copy(), _f32(se).copy()
        assert self.k.shape == self.sb.shape == self.se.shape == (self.d,)
        _load().lpqo_derive_m(_p(self.sb, C.c_float), _p(self.se, C.c_float), self.d, self.bits,
                              _p(self.m, C.c_float))
        return self

    def calibrate(self, x, mode="minmax", scope="per_feature", sigma_mult=1.0):
        x, ld = _mat(x, np.float32)
        assert x.shape[1] == self.d and x.shape[0] >= 1
        rc = _load().lpqo_calibrate(_p(x, C.c_float), x.shape[0], ld, self.d, self.bits,
                                    _CALIB[mode], _SCOPE[scope], float(sigma_mult),
                                    _p(self.k, C.c_float), _p(self.sb, C.c_float),
                                    _p(self.se, C.c_float), _p(self.m, C.c_float))
        if rc:
            raise ValueError("non-finite value in calibration data")
        return self

    def encode(self, x, with_norms=False):
        x, ld = _mat(x, np.float32)
        n = x.shape[0]
        assert x.shape[1] == self.d
        codes = np.zeros((n, self.d), np.int8)
        norms = np.zeros(n, np.int32)
        _load().lpqo_encode(_p(x, C.c_float), n, ld, self.d, self.bits, _p(self.k, C.c_float),
                            _p(self.sb, C.c_float), _p(self.se, C.c_float),
                            _p(self.m, C.c_float), _p(codes, C.c_int8), self.d,
                            _p(norms, C.c_int32))
        return (codes, norms) if with_norms else codes


def dist(a, b, metric="l2sq") -> int:
    a = np.ascontiguousarray(a, np.int8)
    b = np.ascontiguousarray(b, np.int8)
    assert a.shape == b.shape and a.ndim == 1
    f = _load().lpqo_dist_l2sq if _METRIC[metric] == L2SQ else _load().lpqo_dist_ip
    return int(f(_p(a, C.c_int8), _p(b, C.c_int8), a.shape[0]))


def max_threads() -> int:
    return int(_load().lpqo_max_threads())


def search_i8(codes, qcodes, k, metric="l2sq", threads=1):
    """ids int32 [nq,k], dists int32 [nq,k]; rows best first, ties to the lower id."""
    codes, ldc = _mat(codes, np.int8)
    qcodes, ldq = _mat(qcodes, np.int8)
    n, d = codes.shape
    nq = qcodes.shape[0]
    assert qcodes.shape[1] == d and 1 <= k <= n
    ids = np.zeros((nq, k), np.int32)
    dists = np.zeros((nq, k), np.int32)
    rc = _load().lpqo_search_i8(_p(codes, C.c_int8), n, ldc, _p(qcodes, C.c_int8), nq, ldq, d, k,
                                _METRIC[metric], _p(ids, C.c_int32), _p(dists, C.c_int32),
                                int(threads))
    if rc:
        raise MemoryError("oracle search")
    return ids, dists


def search_f32(x, q, k, metric="l2sq", threads=1):
    """Exact search on the fp32 vectors (binary64 sums): ids int32, dists fp32."""
    x, ldx = _mat(x, np.float32)
    q, ldq = _mat(q, np.float32)
    n, d = x.shape
    nq = q.shape[0]
    assert q.shape[1] == d and 1 <= k <= n
    ids = np.zeros((nq, k), np.int32)
    dists = np.zeros((nq, k), np.float32)
    rc = _load().lpqo_search_f32(_p(x, C.c_float), n, ldx, _p(q, C.c_float), nq, ldq, d, k,
                                 _METRIC[metric], _p(ids, C.c_int32), _p(dists, C.c_float),
                                 int(threads))
    if rc:
        raise MemoryError("oracle search")
    return ids, dists


def gather_dist(codes, qcodes, ids, metric="l2sq"):
    """int32 [nq, m]: integer distance between query i and item ids[i, j] (negative id: +-INT32 extreme)."""
    codes, ldc = _mat(codes, np.int8)
    qcodes, ldq = _mat(qcodes, np.int8)
    ids = np.ascontiguousarray(ids, np.int32)
    nq, m = ids.shape
    assert qcodes.shape[0] == nq and qcodes.shape[1] == codes.shape[1]
    assert ids.max(initial=-1) < codes.shape[0]
    out = np.zeros((nq, m), np.int32)
    lib = _load()
    lib.lpqo_gather_dist.restype = None
    lib.lpqo_gather_dist(_p(codes, C.c_int8), C.c_int64(ldc), _p(qcodes, C.c_int8), C.c_int64(nq), C.c_int64(ldq),
                         C.c_int(codes.shape[1]), _p(ids, C.c_int32), C.c_int(m), C.c_int(_METRIC[metric]),
                         _p(out, C.c_int32))
    return out


def rerank_f32(x, q, cand_ids, k, metric="l2sq"):
    """Exact re-rank of candidate lists [nq, kc] on the fp32 vectors: (ids int32, dists fp32) [nq, k]."""
    x, ldx = _mat(x, np.float32)
    q, ldq = _mat(q, np.float32)
    cand = np.ascontiguousarray(cand_ids, np.int32)
    nq, kc = cand.shape
    assert q.shape[0] == nq and q.shape[1] == x.shape[1] and k >= 1
    assert cand.max(initial=-1) < x.shape[0]
    ids = np.zeros((nq, k), np.int32)
    dists = np.zeros((nq, k), np.float32)
    lib = _load()
    lib.lpqo_rerank_f32.restype = C.c_int
    rc = lib.lpqo_rerank_f32(_p(x, C.c_float), C.c_int64(ldx), _p(q, C.c_float), C.c_int64(nq), C.c_int64(ldq),
                             C.c_int(x.shape[1]), _p(cand, C.c_int32), C.c_int(kc), C.c_int(k),
                             C.c_int(_METRIC[metric]), _p(ids, C.c_int32), _p(dists, C.c_float))
    if rc:
        raise MemoryError("oracle rerank")
    return ids, dists


def recall(approx_ids, exact_ids) -> float:
    a = np.ascontiguousarray(approx_ids, np.int32)
    e = np.ascontiguousarray(exact_ids, np.int32)
    assert a.shape == e.shape and a.ndim == 2
    return float(_load().lpqo_recall(_p(a, C.c_int32), _p(e, C.c_int32), a.shape[0], a.shape[1]))


def nibble_codes(codes):
    """Codes as a 4-bit two's-complement field can hold them: values above 7 become 7, values
    below -8 become -8 (Equation 1 at B = 4 reaches +8, one more than a nibble's range; the top
    code is stored as the largest value that fits, as +128 is stored as 127 at B = 8)."""
    c = np.asarray(codes, np.int8).astype(np.int32)
    return np.minimum(np.maximum(c, -8), 7).astype(np.int8)


def pack_nibbles(codes, d_pad):
    """Rows of nibble codes as bytes, written out from the storage definition: byte j of a row
    holds feature 2j in bits 0-3 and feature 2j + 1 in bits 4-7, each as code + 8; features
    beyond the row's d count as code 0 up to d_pad features.  Plain loops."""
    c = nibble_codes(codes)
    n, d = c.shape
    assert d_pad % 2 == 0 and d_pad >= d
    out = np.zeros((n, d_pad // 2), np.uint8)
    for r in range(n):
        for j in range(d_pad // 2):
            lo = int(c[r, 2 * j]) if 2 * j < d else 0
            hi = int(c[r, 2 * j + 1]) if 2 * j + 1 < d else 0
            out[r, j] = (lo + 8) | ((hi + 8) << 4)
    return out
