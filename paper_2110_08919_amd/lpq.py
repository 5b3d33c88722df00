"""Thin ctypes binding of liblpq.so with the names of include/lpq.h.

Argument marshalling only: every step of the search path runs in the HIP library.
torch is used for device memory (tensors are the caller-owned buffers the C ABI asks
for) and for the stream the work is enqueued on.  There is no CPU fallback: if the
library cannot be loaded, importing the symbols raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("LPQ_LIBRARY") or os.path.join(_HERE, "liblpq.so")   # LPQ_LIBRARY: another build of the same ABI

OK, EINVAL, ERANGE, ENOMEM, EDEVICE, ENONFINITE, ESTATE = range(7)
CALIB_MINMAX, CALIB_ABSMAX, CALIB_GAUSS, CALIB_QUANTILE = 0, 1, 2, 3
SCOPE_PER_FEATURE, SCOPE_GLOBAL, SCOPE_SHARED_WIDTH = 0, 1, 2
METRIC_L2SQ, METRIC_IP = 0, 1
TUNE_PATH, TUNE_SPLITS, TUNE_SEED_ROWS, TUNE_DRY_RUN, TUNE_WORK_ORDER, TUNE_WAVE_QUERIES, TUNE_REGION_CAP = 0, 1, 2, 3, 4, 5, 6

CALIB = {"minmax": CALIB_MINMAX, "absmax": CALIB_ABSMAX, "gauss": CALIB_GAUSS, "quantile": CALIB_QUANTILE}
SCOPE = {"per_feature": SCOPE_PER_FEATURE, "global": SCOPE_GLOBAL, "shared_width": SCOPE_SHARED_WIDTH}
METRIC = {"l2sq": METRIC_L2SQ, "ip": METRIC_IP}

_ERR_NAMES = {1: "LPQ_EINVAL", 2: "LPQ_ERANGE", 3: "LPQ_ENOMEM", 4: "LPQ_EDEVICE",
              5: "LPQ_ENONFINITE", 6: "LPQ_ESTATE"}


class LpqError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{_ERR_NAMES.get(code, code)}: {msg}")
        self.code = code


_lib = None


def lib() -> C.CDLL:
    """The loaded library (raises OSError if liblpq.so has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise OSError(f"{LIB_PATH} is missing: run `python -m paper_2110_08919_amd.build`")
        L = C.CDLL(LIB_PATH)
        vp, i64, i32, f32 = C.c_void_p, C.c_int64, C.c_int, C.c_float
        sig = {
            "lpq_quantizer_create": (i32, [C.POINTER(vp), i32, i32]),
            "lpq_quantizer_destroy": (None, [vp]),
            "lpq_quantizer_calibrate": (i32, [vp, vp, i64, i64, i32, i32, f32, vp]),
            "lpq_quantizer_set_params": (i32, [vp, vp, vp, vp]),
            "lpq_quantizer_get_params": (i32, [vp, vp, vp, vp, vp]),
            "lpq_encode": (i32, [vp, vp, i64, i64, vp, i64, vp, vp]),
            "lpq_index_create": (i32, [C.POINTER(vp), vp, i64]),
            "lpq_index_create_packed": (i32, [C.POINTER(vp), vp, i64]),
            "lpq_index_destroy": (None, [vp]),
            "lpq_index_add_f32": (i32, [vp, vp, i64, i64, vp]),
            "lpq_index_add_i8": (i32, [vp, vp, i64, i64, vp]),
            "lpq_index_size": (i64, [vp]),
            "lpq_index_data": (i32, [vp, C.POINTER(vp), C.POINTER(i64), C.POINTER(vp)]),
            "lpq_search_workspace_bytes": (C.c_size_t, [vp, i64, i32, i32]),
            "lpq_search": (i32, [vp, vp, i64, i64, i32, i32, vp, vp, vp, C.c_size_t, vp]),
            "lpq_search_static": (i32, [vp, vp, i64, i64, i32, i32, vp, vp, vp]),
            "lpq_search_i8": (i32, [vp, vp, i64, i64, i32, i32, vp, vp, vp, C.c_size_t, vp]),
            "lpq_search_f32_workspace_bytes": (C.c_size_t, [i64, i64, i32, i32]),
            "lpq_search_f32": (i32, [vp, i64, i64, vp, i64, i64, i32, i32, i32, vp, vp, vp, C.c_size_t, vp]),
            "lpq_gather_dist_i8": (i32, [vp, vp, i64, i64, vp, i32, i32, vp, vp]),
            "lpq_rerank_f32": (i32, [vp, i64, i64, vp, i64, i64, i32, vp, i32, i32, i32, vp, vp, vp]),
            "lpq_search_overflow_stats": (i32, [vp, i64, i32, i32, vp, C.POINTER(i64), C.POINTER(i64)]),
            "lpq_search_overflow_left": (i32, [vp, i64, i32, i32, vp, C.POINTER(i64)]),
            "lpq_set_tuning": (i32, [i32, i64]),
            "lpq_profile_enable": (i32, [i32]),
            "lpq_profile_read": (i32, [C.POINTER(i64), C.POINTER(C.c_double)]),
            "lpq_profile_read_kind": (i32, [i32, C.POINTER(i64), C.POINTER(C.c_double)]),
            "lpq_search_plan_info": (i32, [i32, i32, i32, i64, i64, i32, C.POINTER(i64), i32]),
            "lpq_probe_mfma_i8": (i32, [vp, C.c_size_t, i32, C.POINTER(C.c_double), vp]),
            "lpq_probe_scan_core": (i32, [vp, C.c_size_t, i32, C.POINTER(C.c_double), vp]),
            "lpq_probe_stream": (i32, [vp, C.c_size_t, i32, i32, C.POINTER(C.c_double), vp]),
            "lpq_last_error": (C.c_char_p, []),
        }
        for name, (res, args) in sig.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def _check(rc: int):
    if rc != 0:
        raise LpqError(rc, lib().lpq_last_error().decode())


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t):
    return None if t is None else t.data_ptr()


def _dev_matrix(t: torch.Tensor, dtype):
    assert t.is_cuda and t.dtype == dtype and t.dim() == 2 and t.stride(1) == 1, "need a row-major device matrix"
    ld = t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1])   # a 1-row stride is arbitrary
    return t.data_ptr(), t.shape[0], ld


def set_tuning(key: int, value: int):
    _check(lib().lpq_set_tuning(key, value))


def profile_enable(on: bool):
    _check(lib().lpq_profile_enable(1 if on else 0))


PROFILE_SCAN, PROFILE_SEED = 0, 1


def profile_read(kind=None):
    """(launches, total ms) of all bracketed launches, or of one kind (PROFILE_SCAN / PROFILE_SEED)."""
    n, ms = C.c_int64(0), C.c_double(0.0)
    if kind is None:
        _check(lib().lpq_profile_read(C.byref(n), C.byref(ms)))
    else:
        _check(lib().lpq_profile_read_kind(kind, C.byref(n), C.byref(ms)))
    return n.value, ms.value


PLAN_INFO_COUNT = 35


def search_plan_info(d: int, bits: int, packed: bool, n_items: int, nq: int, k: int):
    """lpq_search_plan_info: the plan of a search as a list of PLAN_INFO_COUNT integers (no device needed)."""
    out = (C.c_int64 * PLAN_INFO_COUNT)()
    _check(lib().lpq_search_plan_info(d, bits, 1 if packed else 0, n_items, nq, k, out, PLAN_INFO_COUNT))
    return list(out)


def probe_mfma_i8(operands: torch.Tensor = None, iters: int = 50000) -> float:
    """Sustained 1e12 op/s of a register-resident int8 matrix-instruction loop whose operand
    registers are filled from `operands` (a contiguous device tensor; None = zeros)."""
    out = C.c_double(0.0)
    nbytes = 0 if operands is None else operands.numel() * operands.element_size()
    _check(lib().lpq_probe_mfma_i8(_ptr(operands), nbytes, iters, C.byref(out), _stream()))
    return out.value


def probe_scan_core(operands: torch.Tensor = None, stages: int = 12000) -> float:
    """Sustained 1e12 op/s of the batched scan's inner loop alone (no copies, barrier or candidates),
    its LDS ring and query registers filled from `operands` (None = zeros)."""
    out = C.c_double(0.0)
    nbytes = 0 if operands is None else operands.numel() * operands.element_size()
    _check(lib().lpq_probe_scan_core(_ptr(operands), nbytes, stages, C.byref(out), _stream()))
    return out.value


def probe_stream(src: torch.Tensor, mode: int = 0, reps: int = 10) -> float:
    """Sustained 1e9 B/s of reading `src` (contiguous device tensor): mode 0 asynchronous
    global->LDS copies, mode 1 register loads."""
    out = C.c_double(0.0)
    _check(lib().lpq_probe_stream(src.data_ptr(), src.numel() * src.element_size(), mode, reps, C.byref(out), _stream()))
    return out.value


class Quantizer:
    """lpq_quantizer_* : the constants of Equation 1 on the device."""

    def __init__(self, d: int, bits: int = 8):
        h = C.c_void_p()
        _check(lib().lpq_quantizer_create(C.byref(h), d, bits))
        self._h, self.d, self.bits = h, d, bits

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.lpq_quantizer_destroy(self._h)
            self._h = None

    def calibrate(self, x: torch.Tensor, mode="minmax", scope="per_feature", sigma_mult=1.0):
        p, n, ld = _dev_matrix(x, torch.float32)
        assert x.shape[1] == self.d
        _check(lib().lpq_quantizer_calibrate(self._h, p, n, ld, CALIB[mode], SCOPE[scope], sigma_mult, _stream()))
        return self

    def set_params(self, k, s_b, s_e):
        arrs = [torch.as_tensor(a, dtype=torch.float32).contiguous().cpu() for a in (k, s_b, s_e)]
        assert all(a.numel() == self.d for a in arrs)
        _check(lib().lpq_quantizer_set_params(self._h, *[a.data_ptr() for a in arrs]))
        return self

    def get_params(self):
        out = [torch.empty(self.d, dtype=torch.float32) for _ in range(4)]
        _check(lib().lpq_quantizer_get_params(self._h, *[a.data_ptr() for a in out]))
        return tuple(a.numpy() for a in out)  # k, S_b, S_e, m

    def encode(self, x: torch.Tensor, with_norms=False, ld_codes=None):
        p, n, ld = _dev_matrix(x, torch.float32)
        ldc = ld_codes or self.d
        codes = torch.zeros((n, ldc), dtype=torch.int8, device=x.device)
        norms = torch.empty(n, dtype=torch.int32, device=x.device) if with_norms else None
        _check(lib().lpq_encode(self._h, p, n, ld, codes.data_ptr(), ldc, _ptr(norms), _stream()))
        codes = codes[:, :self.d]
        return (codes, norms) if with_norms else codes


class Index:
    """lpq_index_* and lpq_search*: the flat int8 corpus and exhaustive top-k search."""

    def __init__(self, quantizer: Quantizer, capacity: int, packed: bool = False):
        h = C.c_void_p()
        create = lib().lpq_index_create_packed if packed else lib().lpq_index_create
        _check(create(C.byref(h), quantizer._h, capacity))
        self._h, self.d, self.capacity, self.packed = h, quantizer.d, capacity, packed
        self._ws = None

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.lpq_index_destroy(self._h)
            self._h = None

    def add_f32(self, x: torch.Tensor):
        p, n, ld = _dev_matrix(x, torch.float32)
        assert x.shape[1] == self.d
        _check(lib().lpq_index_add_f32(self._h, p, n, ld, _stream()))
        return self

    def add_i8(self, codes: torch.Tensor):
        p, n, ld = _dev_matrix(codes, torch.int8)
        assert codes.shape[1] == self.d
        _check(lib().lpq_index_add_i8(self._h, p, n, ld, _stream()))
        return self

    @property
    def size(self) -> int:
        return lib().lpq_index_size(self._h)

    def data(self):
        """(codes_ptr, ld_codes, norms_ptr): raw device pointers into the index storage."""
        cp, ld, npn = C.c_void_p(), C.c_int64(), C.c_void_p()
        _check(lib().lpq_index_data(self._h, C.byref(cp), C.byref(ld), C.byref(npn)))
        return cp.value, ld.value, npn.value

    def storage(self):
        """Host copies (numpy) of the stored rows, uint8 [size, ld_codes] as they lie in device memory
        (int8 codes, or two nibbles per byte for a packed index), and of the norms int32 [size]."""
        import numpy as np
        cp, ld, npn = self.data()
        torch.cuda.synchronize()
        n = self.size
        rows = torch.empty((n, ld), dtype=torch.uint8, device="cuda")
        norms = torch.empty((n,), dtype=torch.int32, device="cuda")
        hip = C.CDLL("libamdhip64.so")
        hip.hipMemcpy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int]
        for dst, src, nb in ((rows, cp, n * ld), (norms, npn, n * 4)):
            rc = hip.hipMemcpy(dst.data_ptr(), src, nb, 3)   # device to device
            if rc:
                raise LpqError(-1, f"hipMemcpy failed with {rc}")
        return np.asarray(rows.cpu()), np.asarray(norms.cpu())

    def workspace_bytes(self, nq: int, k: int, metric="l2sq") -> int:
        return lib().lpq_search_workspace_bytes(self._h, nq, k, METRIC[metric])

    def _workspace(self, nbytes: int, device) -> torch.Tensor:
        if self._ws is None or self._ws.numel() < nbytes or self._ws.device != device:
            self._ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
        return self._ws

    def gather_dist(self, qcodes: torch.Tensor, ids: torch.Tensor, metric="l2sq"):
        """int32 [nq, m]: integer distance between query i (int8 codes) and item ids[i, j]."""
        qp, nq, ld = _dev_matrix(qcodes, torch.int8)
        ip, ni, ldi = _dev_matrix(ids, torch.int32)
        assert ni == nq and ldi == ids.shape[1]
        out = torch.empty(ids.shape, dtype=torch.int32, device=ids.device)
        _check(lib().lpq_gather_dist_i8(self._h, qp, nq, ld, ip, ids.shape[1], METRIC[metric], out.data_ptr(),
                                        _stream()))
        return out

    def overflow_stats(self, nq: int, k: int, metric, workspace: torch.Tensor = None):
        """(queries searched again exactly, largest region fill) of the last search in `workspace`
        (default: the index's own workspace, used when search() was given none)."""
        workspace = self._ws if workspace is None else workspace
        a, b = C.c_int64(0), C.c_int64(0)
        _check(lib().lpq_search_overflow_stats(self._h, nq, k, METRIC[metric], workspace.data_ptr(), C.byref(a), C.byref(b)))
        return a.value, b.value

    def overflow_left(self, nq: int, k: int, metric, workspace: torch.Tensor = None):
        """Queries that overflowed again in the second round of the collecting scan of the last search
        (they went through the generic kernel); 0 when there was no second round."""
        workspace = self._ws if workspace is None else workspace
        a = C.c_int64(0)
        _check(lib().lpq_search_overflow_left(self._h, nq, k, METRIC[metric], workspace.data_ptr(), C.byref(a)))
        return a.value

    def search(self, q: torch.Tensor, k: int, metric="l2sq", out=None, workspace=None):
        """q fp32 [nq, d] or int8 codes [nq, d] on the device -> (ids int32, dists int32) [nq, k]."""
        is_codes = q.dtype == torch.int8
        p, nq, ld = _dev_matrix(q, torch.int8 if is_codes else torch.float32)
        ids, dists = out if out is not None else (
            torch.empty((nq, k), dtype=torch.int32, device=q.device),
            torch.empty((nq, k), dtype=torch.int32, device=q.device))
        need = self.workspace_bytes(nq, k, metric)
        ws = workspace if workspace is not None else self._workspace(need, q.device)
        fn = lib().lpq_search_i8 if is_codes else lib().lpq_search
        _check(fn(self._h, p, nq, ld, k, METRIC[metric], ids.data_ptr(), dists.data_ptr(),
                  ws.data_ptr(), ws.numel(), _stream()))
        return ids, dists

    def search_static(self, q: torch.Tensor, k: int, metric="l2sq", out=None):
        """lpq_search_static: fp32 queries, the library's built-in workspace, no allocation inside the call
        (pass `out` to keep this wrapper from allocating the result tensors either)."""
        p, nq, ld = _dev_matrix(q, torch.float32)
        ids, dists = out if out is not None else (
            torch.empty((nq, k), dtype=torch.int32, device=q.device),
            torch.empty((nq, k), dtype=torch.int32, device=q.device))
        _check(lib().lpq_search_static(self._h, p, nq, ld, k, METRIC[metric], ids.data_ptr(), dists.data_ptr(), _stream()))
        return ids, dists


STATIC_WORKSPACE_BYTES = 64 << 20


def rerank_f32(x: torch.Tensor, q: torch.Tensor, cand_ids: torch.Tensor, k: int, metric="l2sq"):
    """Exact re-rank of candidate lists int32 [nq, kc] on the fp32 vectors: (ids int32, dists fp32) [nq, k]."""
    xp, n, ldx = _dev_matrix(x, torch.float32)
    qp, nq, ldq = _dev_matrix(q, torch.float32)
    cp, nc, ldc = _dev_matrix(cand_ids, torch.int32)
    assert nc == nq and ldc == cand_ids.shape[1] and q.shape[1] == x.shape[1]
    ids = torch.empty((nq, k), dtype=torch.int32, device=x.device)
    dists = torch.empty((nq, k), dtype=torch.float32, device=x.device)
    _check(lib().lpq_rerank_f32(xp, n, ldx, qp, nq, ldq, x.shape[1], cp, cand_ids.shape[1], k, METRIC[metric],
                                ids.data_ptr(), dists.data_ptr(), _stream()))
    return ids, dists


def search_f32(x: torch.Tensor, q: torch.Tensor, k: int, metric="l2sq"):
    """Exact fp32 search: (ids int32, dists fp32) [nq, k]."""
    xp, n, ldx = _dev_matrix(x, torch.float32)
    qp, nq, ldq = _dev_matrix(q, torch.float32)
    d = x.shape[1]
    assert q.shape[1] == d
    ids = torch.empty((nq, k), dtype=torch.int32, device=x.device)
    dists = torch.empty((nq, k), dtype=torch.float32, device=x.device)
    need = lib().lpq_search_f32_workspace_bytes(n, nq, d, k)
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
    _check(lib().lpq_search_f32(xp, n, ldx, qp, nq, ldq, d, k, METRIC[metric], ids.data_ptr(),
                                dists.data_ptr(), ws.data_ptr(), ws.numel(), _stream()))
    return ids, dists
