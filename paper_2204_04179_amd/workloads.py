"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws random inputs (item-ID histories, item content
features, encoder weights, upstream gradients).  It holds none of the
method's arithmetic and imports neither the HIP binding nor the CPU oracle,
so both sides can be fed the very same buffers.

The paper evaluates on Knowledge-Tracing datasets and a news-recommendation
dataset (Section 5.1, Table 3); none of them is available here.  The presets
below take only their shape statistics: item vocabularies of order 1e4 (KT)
and 1e5 (news), an encoder width of 768 (the 6-layer distilled BERT of
Appendix D), and heavy repetition of popular items, which is what makes the
boost ratio R of Section 4.4 larger than one.

Recipe
------
* ids: bounded Zipf over ranks 1..N-1, P(rank r) proportional to r**(-s),
  drawn by inverse CDF on the cumulative sum.  Ranks map to item IDs through a
  seeded random permutation of 1..N-1, so popular items are not neighbouring
  feature rows.  ID 0 is padding only.
* X ~ N(0,1); W ~ N(0, 1/d_in) (standard deviation d_in**-0.5); dH ~ N(0,1),
  including at padded positions (the method has to ignore those).
* bf16 tensors are float32 draws rounded to nearest-even and returned as
  uint16 bit patterns.
* Multi-step: step k of a window uses the stream (seed, tag, k); the rank->id
  permutation, X and W are fixed for the whole window.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional

import numpy as np

F32 = "f32"
BF16 = "bf16"


@dataclass(frozen=True)
class Workload:
    name: str
    B: int            # histories per batch
    L: int            # item IDs per history (news: 50 clicked + 5 candidates)
    N: int            # vocabulary; valid ids are 0..N-1, 0 = padding
    s: float          # Zipf exponent
    d_in: int         # content-feature width
    d: int            # representation width
    xw_dtype: str     # dtype of X and W
    K: int            # accumulation period (1 = Single-step)
    padding: Optional[str]  # None | "last3" | "uniform20"
    seed: int = 0

    @property
    def M(self) -> int:
        return self.B * self.L


WORKLOADS = {
    "tiny": Workload("tiny", 4, 16, 100, 1.1, 64, 32, F32, 1, "last3"),
    "kt": Workload("kt", 64, 100, 13_000, 1.0, 768, 256, BF16, 1, "uniform20"),
    "news": Workload("news", 128, 55, 100_000, 1.2, 768, 400, BF16, 1, None),
    "kt_multi": Workload("kt_multi", 256, 200, 20_000, 0.9, 768, 256, BF16, 8, None),
    "stress": Workload("stress", 1024, 200, 1_000_000, 1.05, 1024, 1024, BF16, 4, None),
}


def get(name: str, **overrides) -> Workload:
    w = WORKLOADS[name]
    return replace(w, **overrides) if overrides else w


_TAG_PERM, _TAG_IDS, _TAG_LEN, _TAG_X, _TAG_W, _TAG_DH = range(6)


def _rng(w: Workload, tag: int, step: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([w.seed, tag, step])))


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bits."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns to float32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def rank_to_id(w: Workload) -> np.ndarray:
    """perm[r-1] = item ID of popularity rank r (r = 1..N-1)."""
    return (_rng(w, _TAG_PERM).permutation(w.N - 1) + 1).astype(np.int32)


def ids(w: Workload, step: int = 0) -> np.ndarray:
    """int32 [B, L] item-ID histories of step `step`; 0 = padding."""
    ranks = np.arange(1, w.N, dtype=np.float64)
    cdf = np.cumsum(ranks ** (-w.s))
    cdf /= cdf[-1]
    u = _rng(w, _TAG_IDS, step).random((w.B, w.L))
    r = np.minimum(np.searchsorted(cdf, u, side="left"), w.N - 2)
    out = rank_to_id(w)[r].astype(np.int32)
    if w.padding == "last3":
        out[:, w.L - 3:] = 0
    elif w.padding == "uniform20":
        lo = min(20, w.L)
        lens = _rng(w, _TAG_LEN, step).integers(lo, w.L + 1, size=w.B)
        out[np.arange(w.L)[None, :] >= lens[:, None]] = 0
    elif w.padding is not None:
        raise ValueError(w.padding)
    return out


def _normal(rng: np.random.Generator, shape, scale: float, dtype: str) -> np.ndarray:
    rows = shape[0]
    out = np.empty(shape, dtype=np.float32 if dtype == F32 else np.uint16)
    chunk = max(1, (1 << 24) // max(1, int(np.prod(shape[1:]))))
    for r0 in range(0, rows, chunk):
        r1 = min(rows, r0 + chunk)
        a = rng.standard_normal((r1 - r0,) + tuple(shape[1:]), dtype=np.float32)
        if scale != 1.0:
            a *= np.float32(scale)
        out[r0:r1] = a if dtype == F32 else f32_to_bf16_bits(a)
    return out


def features(w: Workload) -> np.ndarray:
    """X [N, d_in]: float32, or uint16 bf16 bit patterns.  Row index = item ID."""
    return _normal(_rng(w, _TAG_X), (w.N, w.d_in), 1.0, w.xw_dtype)


def weights(w: Workload) -> np.ndarray:
    """W [d_in, d] with variance 1/d_in: float32, or uint16 bf16 bit patterns."""
    return _normal(_rng(w, _TAG_W), (w.d_in, w.d), w.d_in ** -0.5, w.xw_dtype)


def upstream_grad(w: Workload, step: int = 0) -> np.ndarray:
    """dL/dH [B*L, d] float32 ~ N(0,1); non-zero at padded positions on purpose."""
    return _normal(_rng(w, _TAG_DH, step), (w.M, w.d), 1.0, F32)
