"""Seeded synthetic inputs shaped like the paper's workloads.

This module only makes *inputs* (corpora and query sets).  It holds none of the
method's arithmetic (no quantizer, no distance, no top-k): the CPU oracle and the
HIP library are both fed from here and share nothing else.

Every value is a pure function of ``(seed, stream, row, col)`` through a 64-bit
counter hash, so any row range of any configuration can be regenerated on its own
(chunk-wise on the GPU for the large corpora, row-wise on the CPU for spot checks).
The hash uses wrapping int64 arithmetic only and therefore gives identical bits on
CPU and GPU tensors.  The recipes with exact post-processing (``bimodal``,
``skewed_int``) are bit-identical across devices; the Gaussian recipes go through
``log/cos/sqrt`` and are generated once on one device and then shared as arrays.

What each recipe stands in for (the paper's datasets are not available):

* ``bimodal``     product embeddings whose values lie strictly inside (-0.125, 0.125),
                  half of the mass in the band +-(0.08, 0.125), same law in every
                  dimension (Section 1, Figure 1 description).
* ``skewed_int``  a 128-d descriptor benchmark with non-negative integer features in
                  [0, 255], ~30 % zeros, skewed with a heavy right tail (the L2 row
                  of Table 2).
* ``aniso_unit``  100-d word-embedding-like unit vectors with a 1/i eigen-spectrum,
                  searched by inner product = angular (the angular row of Table 2).
* ``scaled_unit`` 96-d unit vectors whose per-dimension spread differs by 10x.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np
import torch

STREAM_CORPUS = 0
STREAM_QUERIES = 1
STREAM_PARAMS = 2

_MASK64 = (1 << 64) - 1


def _s64(v: int) -> int:
    """Python int -> the int64 holding the same 64 bits."""
    v &= _MASK64
    return v - (1 << 64) if v >= (1 << 63) else v


_GOLDEN = _s64(0x9E3779B97F4A7C15)
_MUL1 = _s64(0xBF58476D1CE4E5B9)
_MUL2 = _s64(0x94D049BB133111EB)


def _lsr(z: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift of an int64 tensor."""
    return (z >> s) & ((1 << (64 - s)) - 1)


def _mix64(z: torch.Tensor) -> torch.Tensor:
    """A 64-bit finalizer (xor-shift-multiply rounds) on wrapping int64 tensors."""
    z = z + _GOLDEN
    z = (z ^ _lsr(z, 30)) * _MUL1
    z = (z ^ _lsr(z, 27)) * _MUL2
    return z ^ _lsr(z, 31)


def _mix64_int(z: int) -> int:
    z = (z + 0x9E3779B97F4A7C15) & _MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
    return z ^ (z >> 31)


def hash_bits(seed: int, stream: int, row0: int, rows: int, d: int,
              device="cpu") -> torch.Tensor:
    """int64 tensor [rows, d] of hashed bits for rows row0 .. row0+rows-1."""
    key = _s64(_mix64_int(_mix64_int(seed) ^ ((stream + 1) * 0xD1B54A32D192ED03 & _MASK64)))
    r = torch.arange(row0, row0 + rows, dtype=torch.int64, device=device).unsqueeze(1)
    c = torch.arange(d, dtype=torch.int64, device=device).unsqueeze(0)
    ctr = r * d + c
    return _mix64(_mix64(ctr ^ key) + key)


def _u24(h: torch.Tensor, shift: int) -> torch.Tensor:
    """24 bits of h starting at bit `shift`, as an int64 in [0, 2^24)."""
    return _lsr(h, shift) & 0xFFFFFF


def _unit_f32(h: torch.Tensor, shift: int) -> torch.Tensor:
    """Uniform fp32 in [0, 1): 24 hashed bits times 2^-24 (exact)."""
    return _u24(h, shift).to(torch.float32) * (1.0 / 16777216.0)


# ----------------------------------------------------------------------------- recipes
_JUST_BELOW_EIGHTH = float(np.nextafter(np.float32(0.125), np.float32(0.0)))


def _bimodal(h: torch.Tensor) -> torch.Tensor:
    sign = 1.0 - 2.0 * ((h >> 63) & 1).to(torch.float32)
    outer = ((h >> 62) & 1).to(torch.bool)
    u = _unit_f32(h, 8)
    mag = torch.where(outer, u * 0.045 + 0.08, u * 0.08)
    mag = torch.clamp(mag, max=_JUST_BELOW_EIGHTH)
    return sign * mag


def _skewed_tables(seed: int, d: int) -> np.ndarray:
    """Per-dimension inverse-CDF thresholds over 24-bit uniforms: [d, 255] int32.

    P(0) = 0.3; otherwise 1 + floor(Exp(scale_j)), capped at 255.  The scales are
    spread (log-uniformly in [10, 60]) so that narrow dimensions never reach 255
    and the overall mean is about 20.
    """
    h = hash_bits(seed, STREAM_PARAMS, 0, 1, d)[0]
    u = (_u24(h, 8).numpy().astype(np.float64) + 0.5) / 16777216.0
    scale = 10.0 * np.exp(u * math.log(60.0 / 10.0))
    v = np.arange(0, 255, dtype=np.float64)[None, :]          # value v: cdf(v)
    cdf = 0.3 + 0.7 * (1.0 - np.exp(-v / scale[:, None]))
    thr = np.floor(cdf * 16777216.0).astype(np.int64)
    return np.minimum(thr, 16777216).astype(np.int32)


def _skewed_int(h: torch.Tensor, tables: torch.Tensor) -> torch.Tensor:
    u = _u24(h, 20).to(torch.int32)                            # [rows, d]
    v = torch.searchsorted(tables, u.t().contiguous(), right=True)   # [d, rows]
    return v.t().to(torch.float32).contiguous()


def _normal(h: torch.Tensor) -> torch.Tensor:
    """Box-Muller from two 24-bit uniforms of one hash word."""
    u1 = (_u24(h, 40).to(torch.float32) + 1.0) * (1.0 / 16777216.0)   # (0, 1]
    u2 = _unit_f32(h, 8)
    return torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)


def _unit_rows(x: torch.Tensor) -> torch.Tensor:
    return x / torch.linalg.vector_norm(x, dim=1, keepdim=True).clamp_min(1e-30)


def _orthogonal(seed: int, d: int) -> np.ndarray:
    h = hash_bits(seed, STREAM_PARAMS, 1, d, d)
    g = _normal(h).numpy().astype(np.float64)
    q, r = np.linalg.qr(g)
    return (q * np.sign(np.diag(r))[None, :]).astype(np.float32)


# ----------------------------------------------------------------------------- configs
@dataclass(frozen=True)
class Workload:
    """One synthetic workload: shapes, recipe, metric and calibration to use."""
    name: str
    recipe: str
    n: int
    d: int
    nq: int
    metric: str            # "l2sq" | "ip"
    ks: tuple
    calib: str             # "minmax" | "absmax" | "gauss"
    scope: str             # "per_feature" | "global"
    seed: int = 0
    _cache: dict = field(default_factory=dict, compare=False, repr=False)

    def scaled(self, n: int | None = None, nq: int | None = None) -> "Workload":
        """Same recipe and seed at a smaller size (prefixes of the same rows)."""
        return Workload(self.name, self.recipe, n or self.n, self.d, nq or self.nq,
                        self.metric, self.ks, self.calib, self.scope, self.seed)

    # -- generation ----------------------------------------------------------
    def _params(self, device):
        key = str(device)
        if key not in self._cache:
            p = {}
            if self.recipe == "skewed_int":
                p["tables"] = torch.from_numpy(_skewed_tables(self.seed, self.d)).to(device)
            elif self.recipe == "aniso_unit":
                p["scale"] = (torch.arange(1, self.d + 1, dtype=torch.float32) ** -0.5).to(device)
                p["rot"] = torch.from_numpy(_orthogonal(self.seed, self.d)).to(device)
            elif self.recipe == "scaled_unit":
                h = hash_bits(self.seed, STREAM_PARAMS, 0, 1, self.d)[0]
                p["std"] = (0.02 + 0.18 * _unit_f32(h, 8)).to(device)
            self._cache[key] = p
        return self._cache[key]

    def rows(self, stream: int, row0: int, rows: int, device="cpu") -> torch.Tensor:
        """fp32 [rows, d]: rows row0.. of the corpus (stream 0) or query set (stream 1)."""
        h = hash_bits(self.seed, stream, row0, rows, self.d, device)
        p = self._params(device)
        if self.recipe == "bimodal":
            return _bimodal(h)
        if self.recipe == "skewed_int":
            return _skewed_int(h, p["tables"])
        if self.recipe == "aniso_unit":
            z = _normal(h) * p["scale"]
            return _unit_rows(z @ p["rot"])
        if self.recipe == "scaled_unit":
            return _unit_rows(_normal(h) * p["std"])
        raise ValueError(self.recipe)

    def corpus(self, device="cpu", chunk: int = 1 << 20, out: torch.Tensor | None = None):
        """The whole corpus as one fp32 tensor [n, d], generated chunk by chunk."""
        if out is None:
            out = torch.empty((self.n, self.d), dtype=torch.float32, device=device)
        for r0 in range(0, self.n, chunk):
            r1 = min(self.n, r0 + chunk)
            out[r0:r1] = self.rows(STREAM_CORPUS, r0, r1 - r0, device)
        return out

    def corpus_chunks(self, device="cpu", chunk: int = 1 << 20):
        for r0 in range(0, self.n, chunk):
            r1 = min(self.n, r0 + chunk)
            yield r0, self.rows(STREAM_CORPUS, r0, r1 - r0, device)

    def queries(self, device="cpu") -> torch.Tensor:
        return self.rows(STREAM_QUERIES, 0, self.nq, device)


# The five workloads of the benchmark description, in its order.
TINY = Workload("tiny_bimodal_10k_x128", "bimodal", 10_000, 128, 100, "l2sq", (10,),
                "minmax", "per_feature", seed=0)
SKEWED_1M = Workload("skewed_int_1m_x128", "skewed_int", 1_000_000, 128, 10_000, "l2sq",
                     (10, 100), "minmax", "global", seed=0)
ANISO_1M2 = Workload("aniso_unit_1m2_x100", "aniso_unit", 1_200_000, 100, 10_000, "ip",
                     (10,), "absmax", "global", seed=0)
SCALED_10M = Workload("scaled_unit_10m_x96", "scaled_unit", 10_000_000, 96, 10_000, "l2sq",
                      (10,), "absmax", "global", seed=0)
PRODUCT_100M = Workload("bimodal_100m_x256", "bimodal", 100_000_000, 256, 10_000, "ip",
                        (100,), "absmax", "per_feature", seed=0)

WORKLOADS = (TINY, SKEWED_1M, ANISO_1M2, SCALED_10M, PRODUCT_100M)
