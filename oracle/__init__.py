"""TEST INFRASTRUCTURE -- NOT PART OF THE PRODUCT PATH.

Python face of the float64 CPU oracle (oracle/lora_oracle.c) for the
heterogeneous-LoRA batching operator, plus an even plainer pure-Python
version for tiny inputs (oracle/tiny.py) and an independent derivation of the
planner's index tables (oracle/plan_ref.py).

Only tests/, the smoke check and the benchmark's cpu_baseline leg may import
this package.  It imports nothing from the HIP package.

Operands are in the mathematical orientation of the operator
(paper section 2 and section 4.3):  x [T,K], W [K,N], A_a [K,r_a],
B_a [r_a,N];  y[t] = x[t] W + s_a (x[t] A_a) B_a.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liblora_oracle.so")
_lib = None

_c_i32p = ctypes.POINTER(ctypes.c_int32)
_c_f64p = ctypes.POINTER(ctypes.c_double)
_c_f64pp = ctypes.POINTER(_c_f64p)


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from . import build as _build
        _build.build(force=True)
    lib = ctypes.CDLL(_LIB_PATH)
    lib.oracle_num_threads.restype = ctypes.c_int
    lib.oracle_token_adapter.restype = ctypes.c_int
    lib.oracle_token_adapter.argtypes = [ctypes.c_int32, ctypes.c_int32, _c_i32p, _c_i32p, _c_i32p]
    lib.oracle_shrink.restype = None
    lib.oracle_shrink.argtypes = [ctypes.c_int32, ctypes.c_int32, _c_i32p, _c_i32p, _c_f64p,
                                  _c_f64p, _c_f64pp, ctypes.c_int, _c_f64p, ctypes.c_int32,
                                  _c_i32p, ctypes.c_int32]
    lib.oracle_expand.restype = None
    lib.oracle_expand.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, _c_i32p, _c_i32p,
                                  _c_f64p, _c_f64p, _c_f64pp, _c_f64pp, _c_f64p, _c_f64p,
                                  _c_i32p, ctypes.c_int32]
    lib.oracle_expand_fast.restype = None
    lib.oracle_expand_fast.argtypes = lib.oracle_expand.argtypes + [ctypes.c_int32]
    lib.oracle_base.restype = None
    lib.oracle_base.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, _c_f64p, _c_f64p,
                                _c_f64p, _c_i32p, ctypes.c_int32]
    lib.oracle_forward.restype = None
    lib.oracle_forward.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, _c_i32p, _c_i32p,
                                   _c_f64p, _c_f64p, _c_f64p, _c_f64pp, _c_f64pp, _c_f64p,
                                   _c_i32p, ctypes.c_int32, ctypes.c_int32]
    _lib = lib
    return lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _p64(a: Optional[np.ndarray]):
    return a.ctypes.data_as(_c_f64p) if a is not None else None


def _p32(a: Optional[np.ndarray]):
    return a.ctypes.data_as(_c_i32p) if a is not None else None


def _ptr_table(mats: Sequence[np.ndarray]):
    """float64 copies of the matrices and a C array of pointers to them."""
    keep = [_f64(m) for m in mats]
    arr = (_c_f64p * max(len(keep), 1))()
    for i, m in enumerate(keep):
        arr[i] = m.ctypes.data_as(_c_f64p)
    return keep, arr


class Adapters:
    """float64 adapter set held for repeated oracle calls (converted once)."""

    def __init__(self, rank, scale, A: Sequence[np.ndarray], B: Sequence[np.ndarray]):
        self.rank = _i32(rank)
        self.scale = _f64(scale)
        assert len(A) == len(B) == self.rank.shape[0]
        for a, (Aa, Ba) in enumerate(zip(A, B)):
            assert Aa.shape[1] == self.rank[a] and Ba.shape[0] == self.rank[a], "rank table mismatch"
        self._A, self.A_ptrs = _ptr_table(A)
        self._B, self.B_ptrs = _ptr_table(B)
        self.max_rank = int(self.rank.max()) if self.rank.size else 0


def token_adapter(T: int, seg_indptr, seg_adapter) -> np.ndarray:
    """Adapter id per token from the segment table (linear scan per token)."""
    indptr, seg_ad = _i32(seg_indptr), _i32(seg_adapter)
    S = seg_ad.shape[0]
    assert indptr.shape[0] == S + 1
    out = np.empty(max(T, 1), dtype=np.int32)
    rc = _load().oracle_token_adapter(T, S, _p32(indptr), _p32(seg_ad), _p32(out))
    if rc != 0:
        raise ValueError("segment table does not tile [0, T)")
    return out[:T]


def _rows(rows):
    if rows is None:
        return None, 0
    r = _i32(rows)
    return r, int(r.shape[0])


def shrink(x, tok_adapter, ad: Adapters, apply_scale: bool = True, rows=None,
           R: Optional[int] = None) -> np.ndarray:
    """v[t, j] = sum_k x[t,k] A_a[k,j] (times s_a if apply_scale); [M, R] float64."""
    x = _f64(x)
    T, K = x.shape
    tok = _i32(tok_adapter)
    rws, n_rows = _rows(rows)
    M = n_rows if rws is not None else T
    R = ad.max_rank if R is None else R
    v = np.empty((M, max(R, 1)), dtype=np.float64)
    _load().oracle_shrink(T, K, _p32(tok), _p32(ad.rank), _p64(ad.scale), _p64(x), ad.A_ptrs,
                          1 if apply_scale else 0, _p64(v), max(R, 1), _p32(rws), n_rows)
    return v[:, :R]


def expand(x, tok_adapter, ad: Adapters, N: int, y_in=None, rows=None, literal: bool = False) -> np.ndarray:
    """y_in + s_a (x A_a) B_a per token; [M, N] float64.  `literal` runs the
    triple loop exactly as the formula is written (slow; small inputs)."""
    x = _f64(x)
    T, K = x.shape
    tok = _i32(tok_adapter)
    rws, n_rows = _rows(rows)
    M = n_rows if rws is not None else T
    yin = _f64(y_in) if y_in is not None else None
    if yin is not None:
        assert yin.shape == (M, N)
    y = np.empty((M, N), dtype=np.float64)
    lib = _load()
    if literal:
        lib.oracle_expand(T, K, N, _p32(tok), _p32(ad.rank), _p64(ad.scale), _p64(x), ad.A_ptrs,
                          ad.B_ptrs, _p64(yin), _p64(y), _p32(rws), n_rows)
    else:
        lib.oracle_expand_fast(T, K, N, _p32(tok), _p32(ad.rank), _p64(ad.scale), _p64(x), ad.A_ptrs,
                               ad.B_ptrs, _p64(yin), _p64(y), _p32(rws), n_rows, ad.max_rank)
    return y


def base(x, W, rows=None) -> np.ndarray:
    """x W; [M, N] float64."""
    x, W = _f64(x), _f64(W)
    T, K = x.shape
    assert W.shape[0] == K
    N = W.shape[1]
    rws, n_rows = _rows(rows)
    M = n_rows if rws is not None else T
    y = np.empty((M, N), dtype=np.float64)
    _load().oracle_base(T, K, N, _p64(x), _p64(W), _p64(y), _p32(rws), n_rows)
    return y


def forward(x, W, tok_adapter, ad: Adapters, rows=None) -> np.ndarray:
    """x W + s_a (x A_a) B_a per token; [M, N] float64."""
    x, W = _f64(x), _f64(W)
    T, K = x.shape
    assert W.shape[0] == K
    N = W.shape[1]
    tok = _i32(tok_adapter)
    rws, n_rows = _rows(rows)
    M = n_rows if rws is not None else T
    y = np.empty((M, N), dtype=np.float64)
    _load().oracle_forward(T, K, N, _p32(tok), _p32(ad.rank), _p64(ad.scale), _p64(x), _p64(W),
                           ad.A_ptrs, ad.B_ptrs, _p64(y), _p32(rws), n_rows, ad.max_rank)
    return y


def merge(W, A, B, scale: float, sign: int = 1) -> np.ndarray:
    """Mode switch (paper section 4.4.2, "swift inference mode switch"): the adapter folded into the
    base weight, W + sign * s * (A B) with sign = +1 to merge and -1 to unmerge; [K, N] float64.
    Written as the definition of the product, one rank-1 term at a time."""
    W, A, B = _f64(W), _f64(A), _f64(B)
    K, N = W.shape
    r = A.shape[1]
    assert A.shape == (K, r) and B.shape == (r, N) and sign in (1, -1)
    out = W.copy()
    for j in range(r):
        out += (sign * float(scale)) * np.outer(A[:, j], B[j, :])
    return out


def error_metrics(y, y_ref, threshold: float = 1e-2):
    """(normwise relative error, max elementwise relative error over
    |y_ref| > threshold).  Both sides are widened to float64 first."""
    y = np.asarray(y, dtype=np.float64)
    y_ref = np.asarray(y_ref, dtype=np.float64)
    diff = y - y_ref
    denom = float(np.linalg.norm(y_ref))
    normwise = float(np.linalg.norm(diff)) / denom if denom > 0 else float(np.linalg.norm(diff))
    mask = np.abs(y_ref) > threshold
    elem = float(np.max(np.abs(diff[mask]) / np.abs(y_ref[mask]))) if mask.any() else 0.0
    return normwise, elem
