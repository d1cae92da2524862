"""Host-side tests of the C-ABI library: planner tables bit-exact against an
independent derivation, tile lists cover the work exactly once, error paths,
exported symbols.  No GPU needed (lora_plan_create is pure host code)."""
import ctypes
import os
import re

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from oracle import plan_ref
from paper_2411_00915_amd import binding as B
from paper_2411_00915_amd import device, workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _export(w, variant=B.LORA_VARIANT_AUTO):
    p = device.make_plan(w, variant)
    v = B.lora_plan_export(p)
    q = B.lora_plan_query(p)
    p.destroy()
    return v, q


def _check_tables(w, v):
    tok, perm, ga, go = plan_ref.tables(w.T, w.seg_indptr, w.seg_adapter, w.adapter_rank)
    assert v["num_tokens"] == w.T
    assert np.array_equal(v["token_adapter"], tok)
    assert np.array_equal(v["perm"], perm)
    assert np.array_equal(v["group_adapter"], ga)
    assert np.array_equal(v["group_offset"], go)
    return tok, perm


def _check_gemm_tables(w, v, tok, perm):
    """the fused forward's row order and adapter stages: a permutation, and every tile's stages cover the columns of
    exactly the adapters its rows carry, once each (the order of rows and stages is the planner's choice)"""
    if v["kernel_family"] != B.LORA_VARIANT_TILED:
        return
    if w.T == 0:
        assert v["gemm_order"].shape[0] == 0 and v["gemm_stage"].shape[0] == 0
        return
    assert v["gemm_order"].shape[0] == w.T
    plan_ref.check_gemm_tables(w.T, tok, w.adapter_rank, v["gemm_order"], v["gemm_stage_offset"], v["gemm_stage"],
                               stage_cols=64)


def _check_tiles(w, v, tok, perm):
    both = v["kernel_family"] == B.LORA_VARIANT_TILED
    assert both or v["expand_tiles"].shape[0] == 0
    if v["shrink_kernel_family"] != B.LORA_VARIANT_TILED:          # (it is TILED whenever kernel_family is)
        assert not both and v["shrink_tiles"].shape[0] == 0
        return
    max_r = int(w.adapter_rank.max()) if w.num_adapters else 0
    P = v["v_parts"]
    assert P in (1, 2, 4)
    et_ = [(t[0], t[1], t[2], t[3], t[4]) for t in v["expand_tiles"]]
    if len(perm):
        for part in range(P):          # every K part covers the (token, rank) plane exactly once
            st_ = [(t[0], t[1], t[2], t[3], t[4]) for t in v["shrink_tiles"] if (t[5] >> 8) & 15 == part]
            plan_ref.check_cover(st_, tok, perm, max(max_r, 1), adapter_rank=w.adapter_rank, rank_axis=True)
        assert all((t[5] >> 12) & 15 == P and (t[5] >> 8) & 15 < P for t in v["shrink_tiles"])
        if both:
            plan_ref.check_cover(et_, tok, perm, w.N)
    else:
        assert v["shrink_tiles"].shape[0] == 0 and not et_
    for t in v["shrink_tiles"]:
        tb, jb = t[5] & 15, (t[5] >> 4) & 15
        assert t[2] <= 16 * tb and t[4] <= 16 * jb and tb in (1, 2, 4, 8) and 1 <= jb <= 8
        assert t[3] % 16 == 0
    for t in v["expand_tiles"]:
        tb = t[5] & 15
        assert t[2] <= 16 * tb and tb in (1, 2, 4, 8) and t[3] % 64 == 0


def _check_mixture(w, m, variant=B.LORA_VARIANT_AUTO):
    """Mixture mode: the plan must be the plan of the tokens' own branches (merged adapter's segments without
    adapter) plus a second batch, over exactly the tokens that are not the merged adapter's, all on that adapter."""
    p = device.make_plan(w, variant, merged_adapter=m)
    v = B.lora_plan_export(p)
    R, v_bytes, ws_bytes = B.lora_plan_query(p)
    p.destroy()
    if m < 0 or m >= w.num_adapters or w.adapter_rank[m] == 0:
        assert v["merged_adapter"] == -1 and v["num_unmerge"] == 0 and v["unmerge_v_offset"] == 0
        tok, perm = _check_tables(w, v)
        _check_tiles(w, v, tok, perm)
        return v
    own_seg, removal = plan_ref.mixture_tables(w.T, w.seg_indptr, w.seg_adapter, w.adapter_rank, m)
    own = wl.Workload(w.name, w.dtype, w.T, w.K, w.N, w.seg_indptr, own_seg, w.adapter_rank, w.adapter_scale, w.x, None)
    tok, perm = _check_tables(own, v)
    _check_tiles(own, v, tok, perm)
    assert v["merged_adapter"] == m
    assert np.array_equal(v["unmerge_perm"], np.nonzero(removal)[0])
    # the removal's tiles: every (token, rank index of m) and every (token, feature) exactly once
    rem_tok = np.where(removal, m, -1)
    rperm = v["unmerge_perm"]
    P2 = v["unmerge_v_parts"]
    if len(rperm) and v["unmerge_shrink_tiles"].shape[0]:
        for part in range(P2):
            st_ = [(t[0], t[1], t[2], t[3], t[4]) for t in v["unmerge_shrink_tiles"] if (t[5] >> 8) & 15 == part]
            plan_ref.check_cover(st_, rem_tok, rperm, int(w.adapter_rank[m]), adapter_rank=w.adapter_rank, rank_axis=True)
        plan_ref.check_cover([(t[0], t[1], t[2], t[3], t[4]) for t in v["unmerge_expand_tiles"]], rem_tok, rperm, w.N)
    # v: own parts, then (256-byte aligned) the removal's
    own_bytes = v["v_parts"] * w.T * R * 4
    assert v["unmerge_v_offset"] == (own_bytes + 255) // 256 * 256
    assert v_bytes == v["unmerge_v_offset"] + P2 * w.T * v["unmerge_v_row_stride"] * 4
    assert ws_bytes >= v_bytes + 2 * w.T * (R + v["unmerge_v_row_stride"]) * 2 and ws_bytes % 256 == 0
    if v["gemm_order"].shape[0]:
        plan_ref.check_gemm_tables(w.T, tok, w.adapter_rank, v["gemm_order"], v["gemm_stage_offset"], v["gemm_stage"],
                                   stage_cols=64, merged=m, removal=removal)
    return v


@pytest.mark.parametrize("name,m", [("cfg2", 5), ("cfg3", 1), ("cfg4", 0), ("cfg4", 77), ("cfg1", 2)])
def test_mixture_mode_tables(name, m):
    w = wl.CONFIGS[name](with_w=False)
    v = _check_mixture(w, m)
    assert v["num_unmerge"] == w.T - int(np.sum(plan_ref.tables(w.T, w.seg_indptr, w.seg_adapter, w.adapter_rank)[0] == m))
    if name == "cfg3":
        # 3 of the 4 requests need the removal; the tiles of the merged adapter's 1024 tokens carry no stage at all
        assert v["num_unmerge"] == 3072 and v["num_active"] == 3072
        off = v["gemm_stage_offset"]
        assert sum(1 for t in range(len(off) - 1) if off[t] == off[t + 1]) == 4


@settings(max_examples=100, deadline=None)
@given(st.lists(st.tuples(st.integers(0, 40), st.integers(-1, 5)), min_size=0, max_size=20),
       st.lists(st.sampled_from([0, 8, 16, 32, 64, 128]), min_size=6, max_size=6),
       st.integers(0, 5), st.sampled_from([64, 1000]))
def test_random_mixture_tables(segs, ranks, m, N):
    lengths = [s[0] for s in segs]
    T = sum(lengths)
    indptr = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32) if segs else np.zeros(1, np.int32)
    w = wl.Workload("h", "bf16", T, 64, N, indptr, np.asarray([s[1] for s in segs], np.int32), np.asarray(ranks, np.int32),
                    np.ones(6, np.float32), np.zeros((T, 64), np.float32), None)
    _check_mixture(w, m, B.LORA_VARIANT_TILED)


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3", "cfg4", "cfg4d", "cfg5"])
def test_config_tables_bit_exact(name):
    w = wl.CONFIGS[name](with_w=False) if name != "cfg5" else wl.cfg5("attn", with_w=False)
    # matrices are not needed here; the tables only depend on the integer structure
    v, q = _export(w)
    tok, perm = _check_tables(w, v)
    _check_tiles(w, v, tok, perm)
    _check_gemm_tables(w, v, tok, perm)
    R = max(8, (int(w.adapter_rank.max()) + 7) // 8 * 8)
    assert q[0] == R and q[1] == v["v_parts"] * w.T * R * 4 and q[2] >= q[1] and q[2] % 256 == 0
    expect = B.LORA_VARIANT_GENERAL if w.dtype == "f32" else B.LORA_VARIANT_TILED
    assert v["kernel_family"] == expect


@settings(max_examples=150, deadline=None)
@given(st.lists(st.tuples(st.integers(0, 40), st.integers(-1, 5)), min_size=0, max_size=20),
       st.lists(st.sampled_from([0, 8, 16, 24, 32, 64, 128]), min_size=6, max_size=6) |
       st.lists(st.sampled_from([0, 3, 8, 20, 100, 129, 256]), min_size=6, max_size=6),     # also ranks only the shrink tiles
       st.sampled_from([64, 200, 1000]))
def test_random_tables_and_tiles(segs, ranks, N):
    lengths = [s[0] for s in segs]
    ads = [s[1] for s in segs]
    T = sum(lengths)
    indptr = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32) if segs else np.zeros(1, np.int32)
    w = wl.Workload("h", "bf16", T, 64, N, indptr, np.asarray(ads, np.int32), np.asarray(ranks, np.int32),
                    np.ones(6, np.float32), np.zeros((T, 64), np.float32), None)
    v, _ = _export(w, B.LORA_VARIANT_TILED)
    tok, perm = _check_tables(w, v)
    _check_tiles(w, v, tok, perm)
    _check_gemm_tables(w, v, tok, perm)


def test_plan_is_deterministic():
    w = wl.cfg4(with_w=False)
    a, _ = _export(w)
    b, _ = _export(w)
    for k in a:
        assert np.array_equal(a[k], b[k]), k


def test_unaligned_layouts_take_general_kernels():
    base = dict(seed=1, T=10, N=32, n_a=2, with_w=False)
    G, T_ = B.LORA_VARIANT_GENERAL, B.LORA_VARIANT_TILED
    fam = lambda v: (v["kernel_family"], v["shrink_kernel_family"])
    w = wl.random_case(K=36, ranks=(8,), **base)           # K not a multiple of 8: nothing is tiled
    assert fam(_export(w)[0]) == (G, G)
    # ranks that only the expand cannot take: the shrink alone keeps the MFMA kernels (tiles for it, none for the expand)
    for ranks in ((5,), (256,), (3, 12, 100, 174)):
        w = wl.random_case(K=64, ranks=ranks, **base)
        for variant in (B.LORA_VARIANT_AUTO, T_):
            v = _export(w, variant)[0]
            assert fam(v) == (G, T_) and v["shrink_tiles"].shape[0] > 0 and v["expand_tiles"].shape[0] == 0
            tok, perm = _check_tables(w, v)
            _check_tiles(w, v, tok, perm)
        assert fam(_export(w, G)[0]) == (G, G)
    wf = wl.random_case(K=64, ranks=(5,), dtype="f32", **base)
    assert fam(_export(wf)[0]) == (G, G)                    # fp32: general throughout
    w = wl.random_case(K=64, ranks=(8,), **base)
    assert fam(_export(w, G)[0]) == (G, G)
    assert fam(_export(w)[0]) == (T_, T_)


def _desc(T=4, indptr=(0, 2, 4), seg_ad=(0, 1), ranks=(8, 16), scales=(1.0, 2.0), k=64, n=64,
          dtype=B.LORA_BF16, variant=0, keep=None):
    keep = keep if keep is not None else []
    i = np.asarray(indptr, np.int32); a = np.asarray(seg_ad, np.int32)
    r = np.asarray(ranks, np.int32); s = np.asarray(scales, np.float32)
    keep.extend([i, a, r, s])
    P = ctypes.POINTER(ctypes.c_int32); F = ctypes.POINTER(ctypes.c_float)
    return B.BatchDesc(T, len(seg_ad), i.ctypes.data_as(P), a.ctypes.data_as(P), len(ranks),
                       r.ctypes.data_as(P), s.ctypes.data_as(F), k, n, dtype, variant), keep


def test_error_paths():
    ok, keep = _desc()
    st_, h = B.lora_plan_create_raw(ok)
    assert st_ == B.LORA_OK and h
    B._lib.lora_plan_destroy(h)
    bad = [
        _desc(indptr=(1, 2, 4)),            # does not start at 0
        _desc(indptr=(0, 3, 2)),            # decreasing / wrong end
        _desc(indptr=(0, 2, 3)),            # does not end at T
        _desc(seg_ad=(0, 2)),               # adapter id out of range
        _desc(seg_ad=(0, -2)),
        _desc(ranks=(8, 257)),              # rank beyond LORA_MAX_RANK
        _desc(ranks=(8, -1)),
        _desc(scales=(1.0, float("nan"))),
        _desc(scales=(float("inf"), 1.0)),
        _desc(k=0), _desc(n=0), _desc(dtype=7), _desc(variant=9), _desc(T=-1),
    ]
    for d, keep in bad:
        st_, h = B.lora_plan_create_raw(d)
        assert st_ == B.LORA_ERR_INVALID_ARG and not h
    assert B.lora_plan_create_raw(None)[0] == B.LORA_ERR_INVALID_ARG
    for bad_m in (3, -1):                            # two adapters: 0 (none), 1 and 2 are the valid values
        d, keep = _desc()
        d.merged_adapter_plus1 = bad_m
        assert B.lora_plan_create_raw(d)[0] == B.LORA_ERR_INVALID_ARG
    d, keep = _desc()
    d.seg_indptr = None
    assert B.lora_plan_create_raw(d)[0] == B.LORA_ERR_INVALID_ARG
    assert B._lib.lora_plan_query(None, None, None, None) == B.LORA_ERR_INVALID_ARG
    B._lib.lora_plan_destroy(None)           # allowed
    assert B.lora_status_str(B.LORA_ERR_WORKSPACE).startswith("workspace")
    # empty batch and empty segments are valid
    st_, h = B.lora_plan_create_raw(_desc(T=0, indptr=(0,), seg_ad=())[0])
    assert st_ == B.LORA_OK
    B._lib.lora_plan_destroy(h)
    st_, h = B.lora_plan_create_raw(_desc(T=4, indptr=(0, 0, 4, 4), seg_ad=(0, 1, 0))[0])
    assert st_ == B.LORA_OK
    B._lib.lora_plan_destroy(h)


def test_compute_calls_reject_bad_arguments_without_a_gpu():
    w = wl.random_case(2, 12, 64, 64, 2, (8,), with_w=False)
    p = device.make_plan(w)
    L = B._lib
    assert L.lora_shrink(p.handle, None, 64, None, None, None) == B.LORA_ERR_INVALID_ARG
    assert L.lora_shrink(None, 256, 64, 256, 256, None) == B.LORA_ERR_INVALID_ARG
    assert L.lora_shrink(p.handle, 256, 32, 256, 256, None) == B.LORA_ERR_INVALID_ARG       # ldx < K
    assert L.lora_expand(p.handle, 256, 256, 256, 64, ctypes.c_float(0.5), None) == B.LORA_ERR_INVALID_ARG   # beta
    assert L.lora_expand(p.handle, 256, 256, 256, 32, ctypes.c_float(1.0), None) == B.LORA_ERR_INVALID_ARG   # ldy < N
    assert L.lora_base_gemm(4, 0, 4, B.LORA_BF16, 256, 8, 256, 8, 256, 8, None) == B.LORA_ERR_INVALID_ARG
    assert L.lora_fused_forward(p.handle, 256, 64, 256, 64, 256, 256, 256, 64, 256, 16, None) == B.LORA_ERR_WORKSPACE
    p.destroy()
    # lora_merge(L, n, k, rank, scale, dtype, variant, Wt_ptrs, ldw, At_ptrs, Bt_ptrs, stream)
    f = ctypes.c_float
    assert L.lora_merge(2, 64, 64, 8, f(1.0), B.LORA_BF16, B.LORA_VARIANT_AUTO, None, 64, 256, 256, None) == B.LORA_ERR_INVALID_ARG
    assert L.lora_merge(2, 64, 64, 8, f(1.0), B.LORA_BF16, B.LORA_VARIANT_AUTO, 256, 32, 256, 256, None) == B.LORA_ERR_INVALID_ARG   # ldw < k
    assert L.lora_merge(2, 64, 64, 8, f(float("nan")), B.LORA_BF16, B.LORA_VARIANT_AUTO, 256, 64, 256, 256, None) == B.LORA_ERR_INVALID_ARG
    assert L.lora_merge(2, 64, 64, 300, f(1.0), B.LORA_BF16, B.LORA_VARIANT_AUTO, 256, 64, 256, 256, None) == B.LORA_ERR_INVALID_ARG  # rank
    assert L.lora_merge(2, 64, 60, 8, f(1.0), B.LORA_BF16, B.LORA_VARIANT_TILED, 256, 64, 256, 256, None) == B.LORA_ERR_UNSUPPORTED   # k % 8
    assert L.lora_merge(2, 64, 64, 8, f(1.0), B.LORA_F32, B.LORA_VARIANT_TILED, 256, 64, 256, 256, None) == B.LORA_ERR_UNSUPPORTED
    assert L.lora_merge(0, 64, 64, 8, f(1.0), B.LORA_BF16, B.LORA_VARIANT_AUTO, None, 64, None, None, None) == B.LORA_OK             # no layers
    assert L.lora_merge(2, 64, 64, 0, f(1.0), B.LORA_BF16, B.LORA_VARIANT_AUTO, None, 64, None, None, None) == B.LORA_OK             # rank 0


def test_tuning_roundtrip_changes_tiles():
    before = B.lora_tuning_get()
    try:
        B.lora_tuning_table_set([dict(tokens=0, k=1, n=1, max_rank=8, group_class=0, tunables={})])   # no entry applies
        w = wl.cfg3(with_w=False)
        a = _export(w)[0]
        B.lora_tuning_set(shrink_tb2_min_rows=1 << 20, shrink_tb4_min_rows=1 << 20, expand_tb2_min_rows=1 << 20,
                          shrink_small_waves=4, shrink_target_wgs=1,
                          shrink_small_jb=2, shrink_stream_min_tokens=1 << 30)
        b = _export(w)[0]
        assert b["shrink_waves"] == 4
        assert b["shrink_tiles"].shape[0] // b["v_parts"] > a["shrink_tiles"].shape[0] // a["v_parts"]
        assert b["expand_tiles"].shape[0] > a["expand_tiles"].shape[0]
        tok, perm = _check_tables(w, b)
        _check_tiles(w, b, tok, perm)
    finally:
        B.lora_tuning_set(**before)
        B.lora_tuning_table_set([])
    assert B.lora_tuning_get() == before


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "lora_abi.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(lora_[a-z_]+)\s*\(", hdr))
    assert {"lora_plan_create", "lora_shrink", "lora_expand", "lora_fused_forward"} <= names
    for n in sorted(names):
        assert hasattr(B._lib, n), f"{n} is declared in lora_abi.h but not exported"
    assert names == set(B.EXPORTED)


def test_trace_set_checks_its_arguments_without_a_gpu():
    import ctypes
    buf = (ctypes.c_int64 * 16)()
    base = ctypes.addressof(buf)
    assert B._lib.lora_trace_set(ctypes.c_void_p(base + 4), 64) == B.LORA_ERR_INVALID_ARG      # not 8-byte aligned
    assert B._lib.lora_trace_set(ctypes.c_void_p(base), 0) == B.LORA_ERR_INVALID_ARG           # no room at all
    assert B._lib.lora_trace_set(None, 0) == B.LORA_OK                                         # off (the default)


def test_shape_table_is_consulted_inside_plan_create():
    """The shape-keyed table (paper section 4.3.2): lora_plan_create looks the batch's class up -- tokens with an
    adapter (smallest entry at or above, else the largest), K, N, rank class, group class -- and plans with the
    entry on top of the process defaults; values in the descriptor override both; every plan keeps its snapshot."""
    defaults = B.lora_tuning_get()
    shipped = B.lora_tuning_table_get()
    assert all(set(e["tunables"]) <= set(B.TUNING_FIELDS) for e in shipped)
    w = wl.cfg2(with_w=False)                                   # 256 tokens, 4096 -> 4096, ranks up to 64, decode-shaped
    try:
        B.lora_tuning_table_set([
            dict(tokens=128, k=4096, n=4096, max_rank=64, group_class=0, tunables={"expand_wave_bytes": 4096}),
            dict(tokens=512, k=4096, n=4096, max_rank=64, group_class=0, tunables={"expand_wave_bytes": 32768, "fused_delay": 7}),
            dict(tokens=1024, k=4096, n=4096, max_rank=64, group_class=0, tunables={"expand_wave_bytes": 65536}),
            dict(tokens=512, k=4096, n=4096, max_rank=64, group_class=1, tunables={"expand_wave_bytes": 8192}),
            dict(tokens=512, k=4096, n=4096, max_rank=32, group_class=0, tunables={"expand_wave_bytes": 8192}),
            dict(tokens=512, k=4096, n=11008, max_rank=64, group_class=0, tunables={"expand_wave_bytes": 8192}),
        ])
        assert len(B.lora_tuning_table_get()) == 6
        p = device.make_plan(w)
        v = B.lora_plan_export(p)
        assert v["tuning_source"] == 1
        assert v["tuning"]["expand_wave_bytes"] == 32768 and v["tuning"]["fused_delay"] == 7      # the 512-token entry
        assert v["tuning"]["shrink_target_wgs"] == defaults["shrink_target_wgs"]                   # not in the entry
        n_tab = v["expand_tiles"].shape[0]
        # the descriptor's own values win over the entry
        q = device.make_plan(w, tuning={"expand_wave_bytes": 8192})
        vq = B.lora_plan_export(q)
        assert vq["tuning_source"] == 3 and vq["tuning"]["expand_wave_bytes"] == 8192 and vq["tuning"]["fused_delay"] == 7
        assert vq["expand_tiles"].shape[0] > n_tab                                                 # smaller tiles, more of them
        tok, perm = _check_tables(w, vq)
        _check_tiles(w, vq, tok, perm)
        # beyond the largest bucket: the largest entry; a shape class without entry: defaults
        big = wl.random_case(5, 1500, 4096, 4096, 600, (8, 64), max_seg=1, with_w=False)
        assert B.lora_plan_export(device.make_plan(big))["tuning"]["expand_wave_bytes"] == 65536
        other = wl.random_case(6, 100, 512, 512, 30, (8, 64), max_seg=1, with_w=False)
        vo = B.lora_plan_export(device.make_plan(other))
        assert vo["tuning_source"] == 0 and vo["tuning"] == defaults
        # group classes: 0 every adapter group below 64 tokens, 2 groups of 512 tokens or more on average, 1 between;
        # an entry without values is a match that keeps the defaults (and is not reported as a source)
        B.lora_tuning_table_set([
            dict(tokens=4096, k=4096, n=4096, max_rank=64, group_class=1, tunables={"expand_stream_stages": 8}),
            dict(tokens=4096, k=4096, n=4096, max_rank=64, group_class=2, tunables={"expand_stream_stages": 32}),
            dict(tokens=2048, k=4096, n=4096, max_rank=64, group_class=2, tunables={}),
        ])
        long_requests = wl.cfg3(with_w=False)                                       # 4 adapters x 1024 tokens
        assert B.lora_plan_export(device.make_plan(long_requests))["tuning"]["expand_stream_stages"] == 32
        mixed = wl.random_case(7, 4096, 4096, 4096, 40, (64,), max_seg=200, with_w=False)   # about 100 tokens per adapter
        assert B.lora_plan_export(device.make_plan(mixed))["tuning"]["expand_stream_stages"] == 8
        half = wl.random_case(8, 2048, 4096, 4096, 2, (64,), max_seg=2048, with_w=False)
        half = wl.Workload("h", "bf16", 2048, 4096, 4096, np.array([0, 1024, 2048], np.int32), np.array([0, 1], np.int32),
                           half.adapter_rank, half.adapter_scale, half.x, None)
        vh = B.lora_plan_export(device.make_plan(half))
        assert vh["tuning_source"] == 0 and vh["tuning"] == defaults                 # the row of zeros, not the 4096-token entry
        # replacing the table does not touch plans already made
        B.lora_tuning_table_set([])
        assert B.lora_plan_export(p)["tuning"]["expand_wave_bytes"] == 32768
        assert B.lora_tuning_table_get() == shipped
        with pytest.raises(B.LoraError):
            B.lora_tuning_table_set([dict(tokens=64, k=64, n=64, max_rank=48, group_class=0, tunables={})])   # not a rank class
        with pytest.raises(KeyError):
            B.lora_tuning_table_set([dict(tokens=64, k=64, n=64, max_rank=64, group_class=0, tunables={"no_such_tunable": 1})])
    finally:
        B.lora_tuning_table_set([])
    assert B.lora_tuning_get() == defaults


def test_build_refuses_scratch_in_kernels_that_count_their_loads():
    """build.py's guard: a kernel that waits with hand-written s_waitcnt vmcnt(n) must not spill (scratch accesses
    use the same counter); the compiler's resource report is parsed and a nonzero scratch size fails the build."""
    from paper_2411_00915_amd import build as b
    R = b.REMARK
    head = f"k.hip:1:1: remark: Function Name: _ZN12_GLOBAL__N_116gemm_ring_kernelILb1EEEv {R}"
    other = f"k.hip:9:1: remark: Function Name: _ZN12_GLOBAL__N_117gemm_tiled_kernelILi4ELb0ELb0EEEv {R}"
    ok = [head, f"k.hip:1:1: remark:     ScratchSize [bytes/lane]: 0 {R}", f"k.hip:1:1: remark:     VGPRs Spill: 0 {R}",
          other, f"k.hip:9:1: remark:     ScratchSize [bytes/lane]: 64 {R}"]
    b._check_no_scratch("k.hip", ok, ("gemm_ring_kernel",))          # other kernels may use scratch
    for bad in ("ScratchSize [bytes/lane]: 8", "VGPRs Spill: 3"):
        with pytest.raises(RuntimeError):
            b._check_no_scratch("k.hip", [head, f"k.hip:1:1: remark:     {bad} {R}"], ("gemm_ring_kernel",))
    with pytest.raises(RuntimeError):                                  # no report at all: cannot vouch for it
        b._check_no_scratch("k.hip", [other], ("gemm_ring_kernel",))
    assert b._without_remarks(ok + ["  459 | {", "      | ^", "2 remarks generated when compiling for gfx950.", "real warning"]) == ["real warning"]


def test_streaming_tiles_for_small_batches_with_long_groups():
    """Below shrink_stream_min_tokens the planner still picks the streaming tiles (up to 128 tokens of one adapter
    over all its rank rows) when the batch cannot run as the single decode launch and holds a group of 64 tokens
    or 128 tokens in all; batches of short groups keep the 16-token tiles; 2^30 switches streaming off."""
    def shrink_rows(T, n_a, r, **tune):
        before = B.lora_tuning_get()
        try:
            if tune:
                B.lora_tuning_set(**tune)
            seg = np.linspace(0, T, n_a + 1).astype(np.int32)
            w = wl.Workload("s", "bf16", T, 4096, 4096, seg, np.arange(n_a, dtype=np.int32), np.full(n_a, r, np.int32),
                            np.ones(n_a, np.float32), np.zeros((T, 4096), np.float32), None)
            v, _ = _export(w, B.LORA_VARIANT_TILED)
            tok, perm = _check_tables(w, v)
            _check_tiles(w, v, tok, perm)
            return int(v["shrink_tiles"][:, 2].max()), int(v["shrink_tiles"][:, 4].max())     # tokens, rank rows of the largest tile
        finally:
            B.lora_tuning_set(**before)
    # (a streaming tile spans all rank rows of its adapter; the other family's tiles at most 64)
    assert shrink_rows(256, 1, 128) == (64, 128)                # one group of 256 tokens: streaming, 64-token tiles (few workgroups)
    assert shrink_rows(64, 1, 128) == (64, 128)                 # one group of 64 tokens
    assert shrink_rows(256, 16, 128) == (16, 128)               # 16 tokens per group, rank 128, 256 tokens in all: streaming
    assert shrink_rows(256, 16, 64)[0] == 16 and shrink_rows(256, 16, 64)[1] <= 32   # short groups, ranks <= 64: 16-token tiles of the decode launch
    assert shrink_rows(48, 4, 128)[1] <= 64                     # 48 tokens in groups of 12: too small for the streaming kernels
    assert shrink_rows(256, 1, 128, shrink_stream_min_tokens=1 << 30)[1] <= 64       # streaming switched off
