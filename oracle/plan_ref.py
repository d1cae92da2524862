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

`check_gemm_tables` does the same for the tables of the fused forward (unmerged
inference in one product, section 4.4): a row order that is a permutation, and per
tile of rows exactly one stage per adapter present and block of its columns.
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


def check_cover(tiles_rows_cols, tok_adapter, perm, extent, adapter_rank=None, rank_axis=False, rows=None):
    """Paint every tile onto a [T_active x extent] canvas and require each cell
    of an active token to be covered exactly once.

    tiles_rows_cols: iterable of (adapter, row0, nrows, c0, cn) with rows
    indexing `perm` and columns indexing [0, extent) -- or, when rank_axis is
    set, [0, rank(adapter)).  rows: optional boolean mask over perm; rows outside it must not be covered at all.
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
        if rows is not None and not rows[p]:
            assert np.all(canvas[p] == 0), f"row {p}: covered although its group has no such part"
            continue
        assert np.all(canvas[p, :lim] == 1), f"row {p}: cells not covered exactly once"
        assert np.all(canvas[p, lim:] == 0)
    return True


def mixture_tables(T, seg_indptr, seg_adapter, adapter_rank, merged):
    """Mixture mode (section 4.4.1): adapter `merged` is folded into the base weight.  Requests of that adapter then
    need no branch; every other request -- with an adapter of its own or with none -- needs the merged update taken
    off again.  Returns (seg_adapter of the tokens' own branches: the merged adapter's segments carry none,
    removal: boolean [T], True where the removal applies)."""
    seg_adapter = np.asarray(seg_adapter, dtype=np.int64)
    lens = np.diff(np.asarray(seg_indptr, dtype=np.int64))
    own = np.where(seg_adapter == merged, -1, seg_adapter)
    removal = np.repeat(seg_adapter != merged, lens)
    assert removal.shape[0] == T
    return own.astype(np.int32), removal


def check_gemm_tables(T, tok_adapter, adapter_rank, order, stage_offset, stages, rows_per_tile=256, stage_cols=64,
                      merged=-1, removal=None):
    """Validity of the fused forward's tables (they are the planner's free choice; only this is fixed).

    The fused forward adds s_a (x A_a) B_a to the base product as extra contraction length: for every adapter a the
    columns of [v_hi | v_lo] (2 r_a of them) are cut into blocks of `stage_cols`, and a tile of rows must run one
    stage per (adapter present in the tile, block) -- each exactly once, or the delta of some token is dropped or
    counted twice -- and none for adapters it does not hold.  `order` must visit every token exactly once.

    Mixture mode (`merged` >= 0, `removal` a boolean mask over tokens): a tile that holds a token of the mask must
    also run the merged adapter's blocks once more, marked by bit 23 of the stage (they apply to the masked rows,
    whatever adapter these have); a tile without such a token must not."""
    tok = np.asarray(tok_adapter, dtype=np.int64)
    rank = np.asarray(adapter_rank, dtype=np.int64)
    order = np.asarray(order, dtype=np.int64)
    stage_offset = np.asarray(stage_offset, dtype=np.int64)
    stages = np.asarray(stages, dtype=np.int64)
    assert np.array_equal(np.sort(order), np.arange(T)), "row order is not a permutation of the tokens"
    n_tiles = -(-T // rows_per_tile)
    assert stage_offset.shape[0] == n_tiles + 1 and stage_offset[0] == 0 and stage_offset[-1] == stages.shape[0]
    assert np.all(np.diff(stage_offset) >= 0)
    for tile in range(n_tiles):
        rows = order[tile * rows_per_tile:(tile + 1) * rows_per_tile]
        present = {int(a) for a in tok[rows] if a >= 0}
        want = sorted((a, jb) for a in present for jb in range(-(-2 * int(rank[a]) // stage_cols)))
        mine = stages[stage_offset[tile]:stage_offset[tile + 1]]
        got = sorted((int(s) & 0xffffff, int(s) >> 24) for s in mine if not int(s) & (1 << 23))
        assert got == want, f"tile {tile}: adapter stages do not cover its adapters' columns exactly once"
        marked = sorted((int(s) & 0x7fffff, int(s) >> 24) for s in mine if int(s) & (1 << 23))
        if merged >= 0 and np.any(np.asarray(removal)[rows]):
            assert marked == [(merged, jb) for jb in range(-(-2 * int(rank[merged]) // stage_cols))], \
                f"tile {tile}: the merged adapter's removal does not cover its columns exactly once"
        else:
            assert not marked, f"tile {tile}: removal stages although no row needs them"
    return True
