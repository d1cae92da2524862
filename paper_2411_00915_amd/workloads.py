"""Seeded synthetic workloads for the heterogeneous-LoRA batching operator.

This module only *draws inputs*: segment tables, rank/scale tables and the
random matrices x, W, A_a, B_a.  It holds none of the operator's arithmetic,
so both the CPU oracle's tests and the HIP path's tests/bench may use it.

Every array is produced in the mathematical orientation of the operator
(ATMM, paper section 4.3; LoRA definition, section 2):

    x   [T, K]      token activations
    W   [K, N]      base weight
    A_a [K, r_a]    adapter "down" factor  (Delta W_a = A_a @ B_a)
    B_a [r_a, N]    adapter "up" factor

For the bf16 configurations the float32 arrays hold values that are exactly
representable in bfloat16 (rounded to nearest-even here), so that the oracle
(which widens them to float64) and the GPU (which narrows them to bf16 without
loss) consume identical numbers.

The shapes follow the paper's 7B/13B-class LMM layers (hidden 4096 and 5120,
adapter rank 64, requests of 128-1024 tokens; paper section 3.2, section 6.1
and its model table); value distributions are zero-mean normals whose
variances keep x.A and (x.A).B at unit scale.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

BASE_SEED = 24110915 * 10


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round a float32 array to the nearest bfloat16 value (ties to even),
    returned as float32.  Finite inputs only."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of a float32 array that already holds bf16 values."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    assert not np.any(u & np.uint32(0xFFFF)), "values are not bf16-representable"
    return (u >> np.uint32(16)).astype(np.uint16)


@dataclass
class Workload:
    name: str
    dtype: str                       # "f32" or "bf16"
    T: int
    K: int
    N: int
    seg_indptr: np.ndarray           # int32 [S+1]
    seg_adapter: np.ndarray          # int32 [S], -1 = no adapter
    adapter_rank: np.ndarray         # int32 [n_a]
    adapter_scale: np.ndarray        # float32 [n_a]
    x: np.ndarray                    # float32 [T, K]
    W: Optional[np.ndarray]          # float32 [K, N] or None when not drawn
    A: List[np.ndarray] = field(default_factory=list)   # float32 [K, r_a]
    B: List[np.ndarray] = field(default_factory=list)   # float32 [r_a, N]

    @property
    def num_segments(self) -> int:
        return int(self.seg_adapter.shape[0])

    @property
    def num_adapters(self) -> int:
        return int(self.adapter_rank.shape[0])

    def token_adapter(self) -> np.ndarray:
        """Adapter id of every token, by expanding the segment table."""
        lens = np.diff(self.seg_indptr)
        return np.repeat(self.seg_adapter, lens).astype(np.int32)


def _normal(rng: np.random.Generator, shape, var: float, dtype: str) -> np.ndarray:
    a = rng.standard_normal(size=shape, dtype=np.float32) * np.float32(np.sqrt(var))
    return round_to_bf16(a) if dtype == "bf16" else a


_TABLES_ONLY = False


class tables_only:
    """Context manager: the generators inside it return the segment, rank and scale tables of a configuration
    without drawing its matrices (x, W, A, B stay None / empty).  The tables come before the matrices in the draw
    order, so they are the same either way.  For benchmarks, which fill device buffers of the right sizes with
    random values instead of uploading gigabytes of host draws."""

    def __enter__(self):
        global _TABLES_ONLY
        self._before, _TABLES_ONLY = _TABLES_ONLY, True
        return self

    def __exit__(self, *exc):
        global _TABLES_ONLY
        _TABLES_ONLY = self._before
        return False


def _draw_matrices(rng, dtype, T, K, N, ranks, with_w, used=None):
    """Draw order is fixed: x, W, A_0..A_{n-1}, B_0..B_{n-1}."""
    if _TABLES_ONLY:
        return None, None, [], []
    x = _normal(rng, (T, K), 1.0, dtype)
    W = _normal(rng, (K, N), 1.0 / K, dtype) if with_w else None
    A = [_normal(rng, (K, int(r)), 1.0 / K, dtype) for r in ranks]
    B = [_normal(rng, (int(r), N), 1.0 / max(int(r), 1), dtype) for r in ranks]
    return x, W, A, B


def _segments_from_lengths(lengths, adapters):
    indptr = np.zeros(len(lengths) + 1, dtype=np.int32)
    indptr[1:] = np.cumsum(np.asarray(lengths, dtype=np.int64))
    return indptr, np.asarray(adapters, dtype=np.int32)


def _lengths_until(total: int, draw) -> List[int]:
    """Draw request lengths until their sum reaches `total`; cut the last."""
    out, acc = [], 0
    while acc < total:
        ln = int(draw())
        ln = min(ln, total - acc)
        out.append(ln)
        acc += ln
    return out


def cfg1(seed: int = BASE_SEED + 1, with_w: bool = True) -> Workload:
    """Tiny fp32 plumbing case: 64 tokens, 256->256, 4 segments of 16, rank 8."""
    rng = np.random.default_rng(seed)
    T, K, N, n_a = 64, 256, 256, 4
    ranks = np.full(n_a, 8, dtype=np.int32)
    indptr, seg_ad = _segments_from_lengths([16] * 4, [0, 1, 2, 3])
    x, W, A, B = _draw_matrices(rng, "f32", T, K, N, ranks, with_w)
    return Workload("cfg1_tiny_f32", "f32", T, K, N, indptr, seg_ad, ranks,
                    np.full(n_a, 1.0, dtype=np.float32), x, W, A, B)


def cfg2(seed: int = BASE_SEED + 2, with_w: bool = True) -> Workload:
    """Decode-shaped batch: 256 single-token requests, 4096->4096, 64 adapters
    of rank uniform on {8,16,32,64}, adapter ids uniform and unsorted."""
    rng = np.random.default_rng(seed)
    T, K, N, n_a = 256, 4096, 4096, 64
    ranks = rng.choice(np.array([8, 16, 32, 64]), size=n_a).astype(np.int32)
    ids = rng.integers(0, n_a, size=T)
    indptr, seg_ad = _segments_from_lengths([1] * T, ids)
    x, W, A, B = _draw_matrices(rng, "bf16", T, K, N, ranks, with_w)
    return Workload("cfg2_decode", "bf16", T, K, N, indptr, seg_ad, ranks,
                    np.full(n_a, 2.0, dtype=np.float32), x, W, A, B)


def cfg3(projection: int = 0, seed: int = BASE_SEED + 3, with_w: bool = True) -> Workload:
    """Vision-prefill batch: 4 requests of 1024 tokens, 4096->4096, rank 64.
    `projection` in 0..3 (q, k, v, o) re-draws the matrices, same segments."""
    rng = np.random.default_rng(seed + 1000 * projection)
    T, K, N, n_a = 4096, 4096, 4096, 4
    ranks = np.full(n_a, 64, dtype=np.int32)
    indptr, seg_ad = _segments_from_lengths([1024] * 4, [0, 1, 2, 3])
    x, W, A, B = _draw_matrices(rng, "bf16", T, K, N, ranks, with_w)
    return Workload(f"cfg3_prefill_p{projection}", "bf16", T, K, N, indptr, seg_ad, ranks,
                    np.full(n_a, 2.0, dtype=np.float32), x, W, A, B)


def _zipf_probs(n: int, s: float) -> np.ndarray:
    p = 1.0 / np.arange(1, n + 1, dtype=np.float64) ** s
    return p / p.sum()


def _cfg4_common(rng, decode_tokens: int):
    T, K, N, n_a = 8192, 4096, 11008, 128
    ranks = rng.choice(np.array([8, 16, 32, 64, 128]), size=n_a).astype(np.int32)
    probs = _zipf_probs(n_a, 1.1)
    sigma = 1.0
    mu = np.log(64.0) - 0.5 * sigma * sigma      # mean of the lognormal variable is 64

    def draw_len():
        return int(np.clip(np.rint(rng.lognormal(mu, sigma)), 1, 2048))

    lengths = _lengths_until(T - decode_tokens, draw_len) + [1] * decode_tokens
    ids = rng.choice(n_a, size=len(lengths), p=probs)
    order = np.argsort(ids, kind="stable")       # requests sorted by adapter
    lengths = [lengths[i] for i in order]
    ids = ids[order]
    indptr, seg_ad = _segments_from_lengths(lengths, ids)
    return T, K, N, n_a, ranks, indptr, seg_ad


def cfg4(seed: int = BASE_SEED + 4, with_w: bool = True, decode_tokens: int = 0,
         name: str = "cfg4_mixed") -> Workload:
    """Mixed serving batch: 8192 tokens, 4096->11008, 128 adapters with ranks
    from {8,...,128}, Zipf(1.1) popularity, lognormal request lengths (mean 64,
    sigma 1, clipped to [1, 2048]), requests sorted by adapter."""
    rng = np.random.default_rng(seed)
    T, K, N, n_a, ranks, indptr, seg_ad = _cfg4_common(rng, decode_tokens)
    x, W, A, B = _draw_matrices(rng, "bf16", T, K, N, ranks, with_w)
    return Workload(name, "bf16", T, K, N, indptr, seg_ad, ranks,
                    np.full(n_a, 2.0, dtype=np.float32), x, W, A, B)


def cfg4d(seed: int = BASE_SEED + 6, with_w: bool = True) -> Workload:
    """Companion of cfg4 in which 1024 of the 8192 tokens are single-token
    decode requests, so decode and prefill segments really mix."""
    return cfg4(seed=seed, with_w=with_w, decode_tokens=1024, name="cfg4d_mixed_decode")


def cfg5(shape: str = "attn", seed: int = BASE_SEED + 5, with_w: bool = True) -> Workload:
    """Large fused-layer case: 16384 tokens, 5120->5120 ("attn") or
    5120->13824 ("mlp"), 256 adapters of rank in {16,32,64,128}, uniform
    popularity, geometric(1/32) segment lengths in arrival order."""
    rng = np.random.default_rng(seed + (0 if shape == "attn" else 1000))
    T, K, n_a = 16384, 5120, 256
    N = 5120 if shape == "attn" else 13824
    ranks = rng.choice(np.array([16, 32, 64, 128]), size=n_a).astype(np.int32)
    lengths = _lengths_until(T, lambda: rng.geometric(1.0 / 32.0))
    ids = rng.integers(0, n_a, size=len(lengths))
    indptr, seg_ad = _segments_from_lengths(lengths, ids)
    x, W, A, B = _draw_matrices(rng, "bf16", T, K, N, ranks, with_w)
    return Workload(f"cfg5_large_{shape}", "bf16", T, K, N, indptr, seg_ad, ranks,
                    np.full(n_a, 2.0, dtype=np.float32), x, W, A, B)


def random_case(seed: int, T: int, K: int, N: int, n_a: int, ranks, dtype: str = "bf16",
                max_seg: int = 8, frac_none: float = 0.0, scales=None,
                with_w: bool = True, empty_segments: bool = False) -> Workload:
    """Small randomised case for parity/edge tests: ragged segments, optional
    tokens without an adapter, optional empty segments, per-adapter scales."""
    rng = np.random.default_rng(seed)
    ranks_arr = rng.choice(np.asarray(ranks), size=n_a).astype(np.int32)
    lengths = _lengths_until(T, lambda: rng.integers(1, max_seg + 1)) if T > 0 else []
    if empty_segments and lengths:
        for pos in sorted(rng.integers(0, len(lengths) + 1, size=3), reverse=True):
            lengths.insert(int(pos), 0)
    ids = rng.integers(0, max(n_a, 1), size=len(lengths))
    if frac_none > 0:
        ids = np.where(rng.random(len(lengths)) < frac_none, -1, ids)
    indptr, seg_ad = _segments_from_lengths(lengths, ids)
    x, W, A, B = _draw_matrices(rng, dtype, T, K, N, ranks_arr, with_w)
    if scales is None:
        sc = np.full(n_a, 2.0, dtype=np.float32)
    else:
        sc = rng.choice(np.asarray(scales, dtype=np.float32), size=n_a).astype(np.float32)
    return Workload(f"rand_{seed}", dtype, T, K, N, indptr, seg_ad, ranks_arr, sc, x, W, A, B)


CONFIGS = {
    "cfg1": cfg1,
    "cfg2": cfg2,
    "cfg3": cfg3,
    "cfg4": cfg4,
    "cfg4d": cfg4d,
    "cfg5": cfg5,
}
