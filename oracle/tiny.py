"""TEST INFRASTRUCTURE -- NOT PART OF THE PRODUCT PATH.

The operator written out with Python scalars, one token / one output element
at a time, for tiny inputs only (paper section 2: an adapter's update is the
product of its two low-rank factors and its result is added onto the base
output; section 4.3: each request of the batch uses its own adapter).
Used to cross-check the C oracle; it shares nothing with it.
"""
from __future__ import annotations

from typing import List, Sequence


def token_adapter(T: int, seg_indptr: Sequence[int], seg_adapter: Sequence[int]) -> List[int]:
    out = [None] * T
    for s, a in enumerate(seg_adapter):
        for t in range(int(seg_indptr[s]), int(seg_indptr[s + 1])):
            assert out[t] is None, "segments overlap"
            out[t] = int(a)
    assert all(o is not None for o in out), "segments leave a gap"
    return out


def forward(x, W, tok_adapter, rank, scale, A, B):
    """y[t][n] = sum_k x[t][k] W[k][n] + s_a sum_j (sum_k x[t][k] A_a[k][j]) B_a[j][n]."""
    T, K, N = len(x), len(W), len(W[0])
    y = [[0.0] * N for _ in range(T)]
    for t in range(T):
        a = tok_adapter[t]
        for n in range(N):
            acc = 0.0
            for k in range(K):
                acc += float(x[t][k]) * float(W[k][n])
            if a >= 0 and rank[a] > 0:
                delta = 0.0
                for j in range(int(rank[a])):
                    vj = 0.0
                    for k in range(K):
                        vj += float(x[t][k]) * float(A[a][k][j])
                    delta += vj * float(B[a][j][n])
                acc += float(scale[a]) * delta
            y[t][n] = acc
    return y
