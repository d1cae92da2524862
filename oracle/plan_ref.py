"""TEST INFRASTRUCTURE -- NOT PART OF THE PRODUCT PATH.

Independent derivation of the integer tables a batch plan must contain, and a
checker for tile lists.  The paper's counterpart is the request-to-adapter
mapping of the batch (section 5, implementation of ATMM) and the lookup that
picks a tile configuration per input shape (section 4.3.1); the tables below
are what is *unique* about a correct plan:

  token_adapter[t]   adapter of token t (-1: none; rank-0 adapters count as none)
  perm               tokens that have an adapter, stably sorted by adapter id
  group_adapter      the distinct adapters in use, ascending
  group_offset       exclusive prefix sums of the group sizes (length G+1)

Tile lists are the planner's free choice; `check_cover` verifies they tile the
work exactly once and never mix adapters.

`gemm_tables` derives the tables of the fused forward (unmerged inference in one
product, section 4.4): the row order and the adapter stages of every 256-row tile.
"""
from __future__ import annotations

import numpy as np


def tables(T, seg_indptr, seg_adapter, adapter_rank):
    seg_indptr = np.asarray(seg_indptr, dtype=np.int64)
    seg_adapter = np.asarray(seg_adapter, dtype=np.int64)
    adapter_rank = np.asarray(adapter_rank, dtype=np.int64)
    lens = np.diff(seg_indptr)
    tok = np.repeat(seg_adapter, lens)
    assert tok.shape[0] == T
    if adapter_rank.size:
        inactive = (tok >= 0) & (adapter_rank[np.clip(tok, 0, adapter_rank.size - 1)] == 0)
        tok = np.where(inactive, -1, tok)
    active = np.nonzero(tok >= 0)[0]
    order = np.argsort(tok[active], kind="stable")
    perm = active[order]
    counts = np.bincount(tok[active], minlength=adapter_rank.size) if active.size else np.zeros(adapter_rank.size, dtype=np.int64)
    group_adapter = np.nonzero(counts)[0]
    group_offset = np.concatenate([[0], np.cumsum(counts[group_adapter])])
    return (tok.astype(np.int32), perm.astype(np.int32), group_adapter.astype(np.int32),
            group_offset.astype(np.int32))


def check_cover(tiles_rows_cols, tok_adapter, perm, extent, adapter_rank=None, rank_axis=False):
    """Paint every tile onto a [T_active x extent] canvas and require each cell
    of an active token to be covered exactly once.

    tiles_rows_cols: iterable of (adapter, row0, nrows, c0, cn) with rows
    indexing `perm` and columns indexing [0, extent) -- or, when rank_axis is
    set, [0, rank(adapter)).
    """
    n_act = len(perm)
    canvas = np.zeros((n_act, extent), dtype=np.int32)
    for (a, row0, nrows, c0, cn) in tiles_rows_cols:
        assert 0 <= row0 and nrows > 0 and row0 + nrows <= n_act, "tile rows out of range"
        assert 0 <= c0 and cn > 0, "tile columns out of range"
        lim = int(adapter_rank[a]) if rank_axis else extent
        assert c0 + cn <= lim, "tile columns beyond extent"
        toks = perm[row0:row0 + nrows]
        assert np.all(tok_adapter[toks] == a), "tile mixes adapters"
        canvas[row0:row0 + nrows, c0:c0 + cn] += 1
    for p in range(n_act):
        lim = int(adapter_rank[tok_adapter[perm[p]]]) if rank_axis else extent
        assert np.all(canvas[p, :lim] == 1), f"row {p}: cells not covered exactly once"
        assert np.all(canvas[p, lim:] == 0)
    return True


def gemm_tables(T, tok_adapter, perm, adapter_rank, rows_per_tile=256, stage_cols=32, weight_cols=64):
    """Row order and per-tile adapter stages of the fused forward.

    Rows: the tokens with an adapter in `perm` order, then the tokens without one in index order.  The whole blocks
    of `rows_per_tile` rows are then put in decreasing order of their number of (adapter, block of `weight_cols`
    columns) pairs, ties in their original order; a last partial block stays last.  A tile's stages: for each
    adapter in the order its rows appear, one entry adapter | block << 24 per block of `stage_cols` columns of the
    adapter's 2 r columns."""
    tok = np.asarray(tok_adapter, dtype=np.int64)
    rank = np.asarray(adapter_rank, dtype=np.int64)
    rows = [int(t) for t in perm] + [t for t in range(T) if tok[t] < 0]
    assert len(rows) == T

    def adapters_of(block):
        seen = []
        for t in block:
            a = int(tok[t])
            if a >= 0 and (not seen or seen[-1] != a):
                seen.append(a)
        return seen

    def blocks_of(a, cols):
        return -(-2 * int(rank[a]) // cols)

    full = T // rows_per_tile
    blocks = [rows[b * rows_per_tile:(b + 1) * rows_per_tile] for b in range(full)]
    weight = [sum(blocks_of(a, weight_cols) for a in adapters_of(blk)) for blk in blocks]
    idx = sorted(range(full), key=lambda b: -weight[b])          # sorted() is stable
    order = [t for b in idx for t in blocks[b]] + rows[full * rows_per_tile:]
    offset, stages = [0], []
    for t0 in range(0, T, rows_per_tile):
        for a in adapters_of(order[t0:t0 + rows_per_tile]):
            stages.extend(a | (jb << 24) for jb in range(blocks_of(a, stage_cols)))
        offset.append(len(stages))
    return np.asarray(order, np.int32), np.asarray(offset, np.int32), np.asarray(stages, np.int32)
