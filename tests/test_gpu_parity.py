"""GPU parity: the HIP path (through the C ABI) against the float64 CPU oracle,
element by element on the same seeded inputs.

Tolerances (bf16 inputs, fp32 accumulation, one rounding of y to bf16):
normwise relative error <= 2e-3 and max elementwise relative error <= 1e-2 over
|y_ref| > 1e-2.  v is fp32 and is held to 1e-5 / 1e-3; the fp32 plumbing
configuration to 1e-5 / 1e-4.  Per-call contracts: lora_expand is compared with
y_in (as stored) + s (x A) B; the fused call with x W + s (x A) B end to end.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
from paper_2411_00915_amd import binding as B
from paper_2411_00915_amd import device, workloads as wl

pytestmark = pytest.mark.gpu

BF16_TOL = (2e-3, 1e-2)
F32_TOL = (1e-5, 1e-4)
# v: fp32 sums of K <= 5120 exact products of O(1/sqrt(K)) size; the absolute error is a few 1e-6, which on
# entries just above the 1e-2 threshold is a relative error of a few 1e-4
V_TOL = (1e-5, 1e-3)
DEV = "cuda:0"


def _tol(w):
    return F32_TOL if w.dtype == "f32" else BF16_TOL


def _assert_close(got, ref, tol, what):
    nrm, elem = oracle.error_metrics(got, ref)
    print(f"    {what}: normwise {nrm:.3e} elementwise {elem:.3e}", flush=True)
    assert nrm <= tol[0], f"{what}: normwise {nrm:.3e} > {tol[0]}"
    assert elem <= tol[1], f"{what}: elementwise {elem:.3e} > {tol[1]}"


def _to_np(t):
    return t.detach().to(torch.float32).cpu().numpy()


def _y_in(w, seed=99):
    rng = np.random.default_rng(seed)
    y = rng.standard_normal((w.T, w.N), dtype=np.float32)
    return wl.round_to_bf16(y) if w.dtype == "bf16" else y


def run_delta_case(w, variant=B.LORA_VARIANT_AUTO, ld_pad=0, check_beta0=True, rows=None):
    """shrink + expand through the ABI vs the oracle.  `rows` limits the oracle
    comparison of y to a sample of tokens (v is always checked in full)."""
    print(f"  case {w.name} T={w.T} K={w.K} N={w.N} variant={variant} ld_pad={ld_pad}", flush=True)
    dl = device.to_device(w, DEV, with_w=False)
    tdt = device.torch_dtype(w)
    plan = device.make_plan(w, variant)
    view = B.lora_plan_export(plan)
    R, v_bytes, _ = B.lora_plan_query(plan)
    tok = oracle.token_adapter(w.T, w.seg_indptr, w.seg_adapter)
    ad = oracle.Adapters(w.adapter_rank, w.adapter_scale, w.A, w.B)
    ldx, ldy = w.K + ld_pad, w.N + ld_pad
    x = torch.zeros((w.T, ldx), dtype=tdt, device=DEV)
    x[:, :w.K] = dl.x
    CANARY = -12345.0
    P = view["v_parts"]
    assert v_bytes == P * w.T * R * 4
    v = torch.full((P, max(w.T, 1), R), CANARY, dtype=torch.float32, device=DEV)
    y0 = _y_in(w)
    y = torch.full((max(w.T, 1), ldy), 7.0, dtype=tdt, device=DEV)
    y[:w.T, :w.N] = torch.from_numpy(y0).to(DEV, tdt)

    B.lora_shrink(plan, x, ldx, dl.At_ptrs, v)
    B.lora_expand(plan, v, dl.Bt_ptrs, y, ldy, 1.0)
    torch.cuda.synchronize()

    v_parts = _to_np(v)[:, :w.T]
    assert all(np.array_equal(v_parts[p] == CANARY, v_parts[0] == CANARY) for p in range(P))
    v_np = np.where(v_parts[0] == CANARY, CANARY, v_parts.astype(np.float64).sum(axis=0)).astype(np.float32)
    v_ref = oracle.shrink(w.x, tok, ad, apply_scale=True, R=R)
    ranks_tok = np.where(tok >= 0, w.adapter_rank[np.clip(tok, 0, None)], 0) if w.num_adapters else np.zeros(w.T, int)
    valid = np.arange(R)[None, :] < ranks_tok[:, None]
    assert np.all(v_np[~valid] == CANARY), "v written outside [0, r_a) or for a token without adapter"
    if valid.any():
        _assert_close(np.where(valid, v_np, 0.0), v_ref, V_TOL if w.dtype == "bf16" else F32_TOL, "v")

    y_np = _to_np(y)[:w.T]
    assert np.all(y_np[:, w.N:] == 7.0), "y written beyond column N"
    no_ad = ranks_tok == 0
    assert np.array_equal(y_np[no_ad, :w.N], y0[no_ad]), "rows without adapter must stay bit-identical"
    sel = np.arange(w.T) if rows is None else np.asarray(rows)
    if w.T:
        y_ref = oracle.expand(w.x, tok, ad, w.N, y_in=y0[sel].astype(np.float64), rows=sel)
        _assert_close(y_np[sel, :w.N], y_ref, _tol(w), "expand beta=1")

    if check_beta0 and w.T:
        y2 = torch.full((w.T, ldy), 3.0, dtype=tdt, device=DEV)
        B.lora_expand(plan, v, dl.Bt_ptrs, y2, ldy, 0.0)
        torch.cuda.synchronize()
        y2_np = _to_np(y2)
        assert np.all(y2_np[no_ad] == 3.0) and np.all(y2_np[:, w.N:] == 3.0)
        d_ref = oracle.expand(w.x, tok, ad, w.N, rows=sel)
        act = ~no_ad[sel]
        if act.any():
            _assert_close(y2_np[sel, :w.N][act], d_ref[act], _tol(w), "expand beta=0")
        # run-to-run determinism (no atomics anywhere in the path)
        v_b = torch.full_like(v, CANARY)
        y_b = torch.full((w.T, ldy), 3.0, dtype=tdt, device=DEV)
        B.lora_shrink(plan, x, ldx, dl.At_ptrs, v_b)
        B.lora_expand(plan, v_b, dl.Bt_ptrs, y_b, ldy, 0.0)
        torch.cuda.synchronize()
        assert torch.equal(v_b, v) and torch.equal(y_b, y2), "two runs differ bitwise"
    torch.cuda.synchronize()
    plan.destroy()
    return view


def _forward_rows(w, view, n_sample, seed):
    """Rows of the oracle comparison for the big configurations: one seeded row out of every 16 consecutive rows of
    the order the fused GEMM walks (so every 16-row MFMA block of every wavefront of every 256-row tile is hit), the
    first and last token of every segment (at most n_sample of them) and n_sample seeded rows on top."""
    rng = np.random.default_rng(seed)
    order = view["gemm_order"] if view["gemm_order"].shape[0] == w.T else np.arange(w.T)
    nblk = (w.T + 15) // 16
    pick = np.minimum(np.arange(nblk) * 16 + rng.integers(0, 16, nblk), w.T - 1)
    edge = np.unique(np.concatenate([w.seg_indptr[:-1], w.seg_indptr[1:] - 1]))
    edge = edge[(edge >= 0) & (edge < w.T)]
    if edge.size > n_sample:
        edge = rng.choice(edge, n_sample, replace=False)
    rest = rng.choice(w.T, min(n_sample, w.T), replace=False)
    return np.unique(np.concatenate([order[pick], edge, rest])).astype(np.int64)


def run_forward_case(w, n_sample=None, seed=5, variant=B.LORA_VARIANT_AUTO):
    """base GEMM alone and the fused forward vs the oracle (on a row sample for the big configurations, see
    _forward_rows), then the fused forward on ALL rows against base GEMM + lora_delta of the same library."""
    dl = device.to_device(w, DEV, with_w=True)
    tdt = device.torch_dtype(w)
    plan = device.make_plan(w, variant)
    view = B.lora_plan_export(plan)
    R, v_bytes, ws_bytes = B.lora_plan_query(plan)
    tok = oracle.token_adapter(w.T, w.seg_indptr, w.seg_adapter)
    ad = oracle.Adapters(w.adapter_rank, w.adapter_scale, w.A, w.B)
    rows = np.arange(w.T) if (n_sample is None or n_sample >= w.T) else _forward_rows(w, view, n_sample, seed)
    print(f"  forward {w.name} T={w.T} K={w.K} N={w.N} oracle rows={rows.size}", flush=True)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=DEV)
    y = torch.full((w.T, w.N), 9.0, dtype=tdt, device=DEV)
    B.lora_base_gemm(w.T, w.K, w.N, dl.dtype, dl.x, w.K, dl.Wt, w.K, y, w.N)
    torch.cuda.synchronize()
    base_ref = oracle.base(w.x, w.W, rows=rows)
    _assert_close(_to_np(y)[rows], base_ref, _tol(w), "base gemm")
    y_base = y.clone()

    y.fill_(9.0)
    B.lora_fused_forward(plan, dl.x, w.K, dl.Wt, w.K, dl.At_ptrs, dl.Bt_ptrs, y, w.N, ws, ws.numel())
    torch.cuda.synchronize()
    y_ref = oracle.forward(w.x, w.W, tok, ad, rows=rows)
    _assert_close(_to_np(y)[rows], y_ref, _tol(w), "fused forward")

    # Every row, GPU against GPU: y_fused = rnd(xW + d), y_base = rnd(xW), y_delta = rnd(d) with one rounding each
    # (bf16: relative 2^-8; fp32: 2^-24) on top of fp32 accumulation noise, so element by element
    # |y_fused - (y_base + y_delta)| <= u (|y_fused| + |y_base| + |y_delta|) + accumulation slack.
    # A wrong row, a dropped or doubled adapter stage or a stale operand is an O(1) error.
    if w.T:
        v = torch.zeros(max(v_bytes // 4, 4), dtype=torch.float32, device=DEV)
        y_delta = torch.zeros((w.T, w.N), dtype=tdt, device=DEV)
        B.lora_delta(plan, dl.x, w.K, dl.At_ptrs, dl.Bt_ptrs, v, y_delta, w.N, 0.0)
        torch.cuda.synchronize()
        u = 2.0 ** -8 if w.dtype == "bf16" else 2.0 ** -24
        slack = 1e-4 if w.dtype == "bf16" else 1e-5
        yf, yb, yd = y.float(), y_base.float(), y_delta.float()
        excess = (yf - (yb + yd)).abs() - (1.01 * u * (yf.abs() + yb.abs() + yd.abs()) + slack)
        worst = float(excess.max())
        ranks_tok = np.where(tok >= 0, w.adapter_rank[np.clip(tok, 0, None)], 0) if w.num_adapters else np.zeros(w.T, int)
        none = torch.from_numpy(ranks_tok == 0).to(DEV)
        same = float((y[none] == y_base[none]).float().mean()) if bool(none.any()) else 1.0
        nrm = float(torch.linalg.norm(yf - (yb + yd)) / torch.linalg.norm(yb + yd).clamp_min(1e-30))
        print(f"    fused vs base gemm + lora_delta, all {w.T} rows: normwise {nrm:.3e}, worst excess over the "
              f"rounding bound {worst:.3e}; rows without adapter bit-identical to the base GEMM: {same:.4f}", flush=True)
        assert worst <= 0.0, "fused forward differs from base GEMM + delta by more than the three roundings allow"
        if bool(none.any()):      # no delta: the same product, at most the last bit apart (summation order)
            assert bool(((y[none].float() - y_base[none].float()).abs() <= 2 * u * y_base[none].float().abs() + slack).all())
    plan.destroy()


# ---------------------------------------------------------------- configurations
def test_cfg1_tiny_fp32():
    w = wl.cfg1()
    run_delta_case(w)
    run_forward_case(w)


def test_cfg2_decode():
    w = wl.cfg2()
    view = run_delta_case(w)
    assert view["kernel_family"] == B.LORA_VARIANT_TILED
    run_delta_case(w, B.LORA_VARIANT_GENERAL, check_beta0=False)
    run_forward_case(w)


@pytest.mark.parametrize("projection", [0, 1, 2, 3])
def test_cfg3_prefill(projection):
    w = wl.cfg3(projection)
    run_delta_case(w, check_beta0=(projection == 0))
    run_forward_case(w, n_sample=128)


def test_cfg4_mixed():
    w = wl.cfg4()
    run_delta_case(w, rows=np.arange(0, w.T, 4))
    run_forward_case(w, n_sample=192)


def test_cfg4d_mixed_with_decode_requests():
    w = wl.cfg4d()
    run_delta_case(w, rows=np.arange(0, w.T, 4), check_beta0=False)
    run_forward_case(w, n_sample=192)


@pytest.mark.parametrize("shape", ["attn", "mlp"])
def test_cfg5_large(shape):
    w = wl.cfg5(shape)
    run_delta_case(w, rows=np.arange(0, w.T, 8), check_beta0=False)
    run_forward_case(w, n_sample=128)


@pytest.mark.parametrize("T,K,N", [(3585, 128, 3600), (3600, 160, 3585), (3585, 200, 3600)])
def test_large_tile_gemm_ragged_shapes(T, K, N):
    """The 256 x 256 tile kernels on ragged T and N with few stages: the shortest ring (four stages of 32 k), an odd
    number of stages, and a K that is no multiple of 32 (staged through registers, with a K tail); base GEMM and
    fused forward, with mixed ranks, tokens without adapter and several adapters per tile."""
    w = wl.random_case(700 + K, T, K, N, 40, (8, 16, 24, 32, 64, 128), max_seg=90, frac_none=0.15, scales=(0.5, 2.0))
    run_forward_case(w, n_sample=160)


@pytest.mark.parametrize("K", [256, 200])
def test_large_tile_gemm_with_hundreds_of_adapters_per_tile(K):
    """Single-token segments of 400 adapters: a 256-row tile carries about 250 adapters.  K = 256: the ring kernel,
    whose wavefronts then walk about 60 adapters each for their 64 rows.  K = 200 (no multiple of 32): the
    register-staged kernel with far more adapter stages than it caches per tile (256), so that it reads the stages
    beyond its list from memory."""
    w = wl.random_case(811, 3840, K, 3328, 400, (32, 64), max_seg=1, frac_none=0.05)
    run_forward_case(w, n_sample=160)


@pytest.mark.parametrize("shape", ["decode", "prefill"])
def test_hip_graph_replays_match_the_eager_calls(shape):
    """lora_delta and lora_fused_forward captured into a HIP graph: every replay, with eager calls of the same plan
    and synchronisations in between, gives bit for bit what the eager calls give (the single-launch decode kernel
    keeps hand-off counters across launches; the streaming and GEMM kernels set function attributes on first use)."""
    if shape == "decode":      # one launch for shrink + expand
        w = wl.random_case(901, 180, 512, 768, 24, (8, 16, 32, 64), max_seg=3, frac_none=0.1)
    else:                      # streaming shrink / expand, ring GEMM with adapter stages
        w = wl.random_case(902, 3600, 1024, 3600, 12, (16, 32, 64, 128), max_seg=300, frac_none=0.1)
    dl = device.to_device(w, DEV, with_w=True)
    tdt = device.torch_dtype(w)
    plan = device.make_plan(w)
    R, v_bytes, ws_bytes = B.lora_plan_query(plan)
    B.lora_plan_upload(plan)
    y0 = torch.from_numpy(_y_in(w)).to(DEV, tdt)

    def buffers():
        return (torch.zeros(max(v_bytes // 4, 1), dtype=torch.float32, device=DEV), y0.clone(),
                torch.empty(w.T, w.N, dtype=tdt, device=DEV), torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=DEV))

    def run(v, y, yf, ws, stream=None):
        B.lora_delta(plan, dl.x, w.K, dl.At_ptrs, dl.Bt_ptrs, v, y, w.N, 1.0, stream)
        B.lora_fused_forward(plan, dl.x, w.K, dl.Wt, w.K, dl.At_ptrs, dl.Bt_ptrs, yf, w.N, ws, ws.numel(), stream)

    v_e, y_e, yf_e, ws_e = buffers()
    run(v_e, y_e, yf_e, ws_e)                                  # eager: also the first use of every kernel
    torch.cuda.synchronize()

    v_g, y_g, yf_g, ws_g = buffers()
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            run(v_g, y_g, yf_g, ws_g, side)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for replay in range(4):
        y_g.copy_(y0)                                          # lora_delta accumulates onto y
        yf_g.fill_(3.0)
        v_g.fill_(-7.0)
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y_g, y_e), f"lora_delta: replay {replay} differs from the eager call"
        assert torch.equal(yf_g, yf_e), f"lora_fused_forward: replay {replay} differs from the eager call"
        v2, y2, yf2, ws2 = buffers()                           # eager work of the same plan between the replays
        run(v2, y2, yf2, ws2)
        torch.cuda.synchronize()
        assert torch.equal(y2, y_e) and torch.equal(yf2, yf_e)
    plan.destroy()


# ---------------------------------------------------------------- edge cases
@pytest.mark.parametrize("variant", [B.LORA_VARIANT_TILED, B.LORA_VARIANT_GENERAL])
def test_ragged_small_cases(variant):
    # several tiles and ragged tails: K not a multiple of 32, N not of 64 / 16,
    # tokens without adapter, empty segments, heterogeneous scales, all ranks
    for seed, (T, K, N) in enumerate([(37, 72, 200), (150, 328, 1000), (9, 64, 24), (300, 520, 72)]):
        w = wl.random_case(100 + seed, T, K, N, 7, (8, 16, 24, 32, 40, 64, 128), max_seg=40,
                           frac_none=0.25, scales=(0.5, 1.0, 2.0, -1.5, 3.25), empty_segments=True)
        run_delta_case(w, variant)
        run_delta_case(w, variant, ld_pad=8, check_beta0=False)
        run_forward_case(w, variant=variant)


def test_fused_forward_with_a_single_k_stage():
    # K of at most 64 is one stage of the register-staged GEMM: the first stage fetched ahead is then already an
    # adapter stage, whose descriptors every thread reads from LDS (a missing barrier there once let a workgroup read
    # them before they were written; found by a random sweep).  Several row tiles, many adapters per tile, plain and
    # mixture mode, different batches back to back.
    for seed, (T, K, N, n_a, ranks) in enumerate([(700, 64, 200, 9, (64,)), (300, 40, 328, 30, (8, 16, 32)),
                                                  (520, 64, 136, 5, (128,)), (130, 32, 72, 12, (8, 64))]):
        w = wl.random_case(600 + seed, T, K, N, n_a, ranks, max_seg=3, frac_none=0.1, scales=(1.0, 2.0, -0.5))
        run_forward_case(w, n_sample=min(T, 160), variant=B.LORA_VARIANT_TILED)
        run_mixture_case(w, seed % n_a, n_sample=min(T, 96))


def test_seeded_sweep_of_random_batches():
    # Many small batches drawn from a seeded generator -- token counts from one to a few thousand, K from one GEMM
    # stage to 4096, ragged N, one to 150 adapters, aligned and odd rank sets, segment lengths from decode to
    # prefill -- through lora_delta (both kernel families decide for themselves), the single launch with and without
    # its fallback, the fused forward and mixture mode.  (A sweep like this found the missing barrier that
    # test_fused_forward_with_a_single_k_stage pins.)
    rng = np.random.default_rng(20241128)
    rank_sets = [(8, 16, 32, 64), (8, 64), (16, 128), (8, 16, 24, 40, 128), (64,), (128,), (3, 12, 100), (8, 20, 256), (4, 8)]
    for i in range(36):
        T = int(rng.choice([1, 7, 33, 100, 256, 300, 700, 1500, 2600]))
        K = int(rng.choice([64, 328, 1024, 2048, 4096]))
        N = int(rng.choice([64, 200, 1000, 2048, 4096]))
        n_a = int(rng.choice([1, 3, 9, 40, 150]))
        ranks = rank_sets[int(rng.integers(len(rank_sets)))]
        max_seg = int(rng.choice([1, 2, 12, 64, 300, 1024]))
        frac_none, empty = float(rng.choice([0.0, 0.2])), bool(rng.integers(2))
        m = int(rng.integers(n_a))
        if T * N < 400:
            continue                                # the normwise bound is a statement about many roundings
        w = wl.random_case(7000 + i, T, K, N, n_a, ranks, max_seg=max_seg, frac_none=frac_none,
                           scales=(0.5, 2.0, -1.5), empty_segments=empty)
        print(f"[{i}] T={T} K={K} N={N} adapters={n_a} ranks={ranks} max_seg={max_seg}", flush=True)
        run_delta_case(w, check_beta0=bool(i % 2))
        if i % 3 == 0:
            run_forward_case(w, n_sample=min(T, 96))
        if i % 4 == 1:
            _delta_case(w)
            _delta_case(w, fallback=True)
        # (mixture's identity check against unmerged inference assumes an update that does not dwarf W)
        if i % 5 == 0 and K >= 1024 and max(ranks) <= 64 and all(r % 8 == 0 for r in ranks):
            run_mixture_case(w, m, n_sample=min(T, 64))


def test_large_token_counts():
    # four times the tokens of the largest benchmark configuration (64-bit row offsets, tile lists of tens of
    # thousands of entries, thousands of adapter groups); the oracle checks v in full and y on sampled rows
    rng = np.random.default_rng(9)
    for seed, (T, K, N, n_a, ranks, max_seg) in enumerate([(65536, 1024, 2048, 512, (8, 16, 32, 64, 128), 64),
                                                           (50000, 2048, 1024, 2000, (8, 16), 1)]):
        w = wl.random_case(800 + seed, T, K, N, n_a, ranks, max_seg=max_seg, frac_none=0.05, scales=(2.0, -0.5))
        run_delta_case(w, check_beta0=False, rows=np.sort(rng.choice(T, size=256, replace=False)))
        run_forward_case(w, n_sample=160)


def test_streaming_kernels_ragged_cases():
    # the prefill-sized (streaming) shrink / expand kernels forced onto small ragged batches: adapter
    # groups from 1 to a few hundred tokens (every tile shape: 8, 4, 2, 1 token blocks), all ranks up to
    # 128, K with a ragged last stage and a ragged last k-step, N with a ragged last chunk, tokens without
    # adapter, padded leading dimensions, K split over 1, 2, 4 workgroups, short and long feature ranges
    before = B.lora_tuning_get()
    B.lora_timing_begin()
    try:
        cases = [(420, 1096, 200, 3, 300), (333, 2048, 1352, 9, 90), (700, 2120, 72, 5, 40), (129, 1024, 64, 1, 1000)]
        settings = [dict(shrink_stream_wgs=1, expand_stream_stages=16), dict(shrink_stream_wgs=1 << 20, expand_stream_stages=1),
                    dict(shrink_stream_wgs=512, expand_stream_stages=2)]
        for seed, (T, K, N, n_a, max_seg) in enumerate(cases):
            w = wl.random_case(500 + seed, T, K, N, n_a, (8, 16, 24, 32, 40, 64, 96, 128), max_seg=max_seg,
                               frac_none=0.15, scales=(0.5, 1.0, 2.0, -1.5), empty_segments=True)
            for st in settings:
                B.lora_tuning_set(**before)
                B.lora_tuning_set(shrink_stream_min_tokens=1, **st)
                run_delta_case(w, B.LORA_VARIANT_TILED, check_beta0=(st is settings[0]))
            run_delta_case(w, B.LORA_VARIANT_TILED, ld_pad=8, check_beta0=False)
            run_forward_case(w, variant=B.LORA_VARIANT_TILED)
    finally:
        B.lora_tuning_set(**before)
        launched = B.lora_timing_end()
    assert {"shrink_stream_kernel", "expand_stream_kernel"} <= set(launched), sorted(launched)
    assert not {"shrink_tiled_kernel", "expand_tiled_kernel"} & set(launched), sorted(launched)


def test_general_kernels_take_odd_layouts():
    w = wl.random_case(200, 45, 77, 53, 5, (1, 3, 5, 12, 200, 256), max_seg=9, frac_none=0.2,
                       scales=(1.0, 2.0, -0.5))
    run_delta_case(w)                              # odd K, N, ranks: general family
    run_delta_case(w, ld_pad=3, check_beta0=False)
    run_forward_case(w)
    wf = wl.random_case(201, 33, 40, 48, 3, (4, 8), dtype="f32", max_seg=6, frac_none=0.2)
    run_delta_case(wf)
    run_forward_case(wf)


def test_degenerate_batches():
    # no tokens at all
    w = wl.random_case(300, 0, 64, 64, 2, (8,))
    run_delta_case(w)
    # every token without adapter: y must equal its input bit for bit, fused = x W
    w = wl.random_case(301, 40, 64, 128, 2, (8, 16), frac_none=1.0)
    run_delta_case(w)
    run_forward_case(w)
    # one long segment, one adapter, maximum tiled rank
    w = wl.random_case(302, 257, 256, 192, 1, (128,), max_seg=1000)
    run_delta_case(w)
    # single token
    w = wl.random_case(303, 1, 128, 64, 3, (8, 64))
    run_delta_case(w)
    run_forward_case(w)


def test_tiled_request_with_unaligned_leading_dimension_is_refused():
    w = wl.random_case(304, 20, 64, 64, 2, (8,))
    dl = device.to_device(w, DEV, with_w=False)
    plan = device.make_plan(w, B.LORA_VARIANT_TILED)
    R, _, _ = B.lora_plan_query(plan)
    x = torch.zeros((w.T, w.K + 3), dtype=torch.bfloat16, device=DEV)
    v = torch.zeros(B.lora_plan_query(plan)[1] // 4, dtype=torch.float32, device=DEV)
    with pytest.raises(B.LoraError) as e:
        B.lora_shrink(plan, x, w.K + 3, dl.At_ptrs, v)
    assert e.value.status == B.LORA_ERR_UNSUPPORTED
    torch.cuda.synchronize()
    plan.destroy()


# ---------------------------------------------------------------- shape table
NO_TABLE = [dict(tokens=0, k=1, n=1, max_rank=8, group_class=0, tunables={})]      # matches no batch


@pytest.mark.parametrize("name", ["cfg2", "cfg4"])
def test_shape_table_entries_change_the_plan_and_keep_parity(name):
    """The shape table (section 4.3.2) is consulted inside lora_plan_create: under an entry for the configuration's
    shape class the plan carries the entry's tunables, its tile lists differ from those the defaults give, and it
    passes parity -- with an entry made up here, and with the shipped table's own entry where it has one for the
    class (the offline search keeps an entry only where it beat the defaults on two machines)."""
    w = wl.CONFIGS[name](with_w=False)
    rows = None if w.T <= 1024 else np.arange(0, w.T, 8)
    rc = 8
    while rc < int(w.adapter_rank.max()):
        rc *= 2
    try:
        B.lora_tuning_table_set(NO_TABLE)
        plain = device.make_plan(w)
        vp = B.lora_plan_export(plain)
        plain.destroy()
        assert vp["tuning_source"] == 0 and vp["tuning"] == B.lora_tuning_get()
        made_up = dict(shrink_small_jb=2, expand_wave_bytes=4096, fused_delay=8) if name == "cfg2" else \
            dict(shrink_stream_wgs=4096, expand_stream_stages=2)
        tables = [("made up", [dict(tokens=w.T, k=w.K, n=w.N, max_rank=rc, group_class=0 if name == "cfg2" else 1, tunables=made_up)])]
        B.lora_tuning_table_set([])
        shipped = device.make_plan(w)
        has_entry = B.lora_plan_export(shipped)["tuning_source"] == 1
        shipped.destroy()
        print(f"  shipped table has an entry for {w.name}'s class: {has_entry}", flush=True)
        if has_entry:
            tables.append(("shipped", []))
        for label, table in tables:
            B.lora_tuning_table_set(table)
            p = device.make_plan(w)
            vs = B.lora_plan_export(p)
            p.destroy()
            assert vs["tuning_source"] == 1
            changed = {k for k in B.TUNING_FIELDS if vs["tuning"][k] != vp["tuning"][k]}
            assert changed, f"{label}: the entry changes no tunable"
            if label == "made up":
                assert all(vs["tuning"][k] == val for k, val in made_up.items())
            assert (vs["shrink_tiles"].shape != vp["shrink_tiles"].shape or vs["expand_tiles"].shape != vp["expand_tiles"].shape or
                    not np.array_equal(vs["shrink_tiles"], vp["shrink_tiles"]) or not np.array_equal(vs["expand_tiles"], vp["expand_tiles"]) or
                    vs["shrink_waves"] != vp["shrink_waves"]), f"{label}: entry {changed} left the plan as it was"
            view = run_delta_case(w, rows=rows, check_beta0=False)
            assert view["tuning_source"] == 1
            if name == "cfg2":
                _delta_case(w)                                           # the single launch under that entry
    finally:
        B.lora_tuning_table_set([])


# ---------------------------------------------------------------- one launch for both steps
def _delta_case(w, fallback=False):
    """lora_delta (single launch when the plan allows) vs the oracle and vs shrink + expand."""
    print(f"  delta {w.name} T={w.T} K={w.K} N={w.N} fallback={fallback}", flush=True)
    before = B.lora_tuning_get()
    try:
        if fallback:
            B.lora_tuning_set(fused_wait_us=1)      # never wait: every expand block recomputes its v rows
        dl = device.to_device(w, DEV, with_w=False)
        plan = device.make_plan(w)
    finally:
        B.lora_tuning_set(**before)
    tdt = device.torch_dtype(w)
    _, v_bytes, _ = B.lora_plan_query(plan)
    view = B.lora_plan_export(plan)
    waves = view["shrink_waves"]
    fused = view["kernel_family"] == B.LORA_VARIANT_TILED and view["expand_tiles"].shape[0] > 0 and \
        bool(np.all((view["expand_tiles"][:, 5] >> 8) & 0xfff > 0))
    tok = oracle.token_adapter(w.T, w.seg_indptr, w.seg_adapter)
    ad = oracle.Adapters(w.adapter_rank, w.adapter_scale, w.A, w.B)
    y0 = _y_in(w)
    v = torch.zeros(max(v_bytes // 4, 4), dtype=torch.float32, device=DEV)
    for beta in (1.0, 0.0):
        y_a = torch.from_numpy(y0).to(DEV, tdt)
        y_b = y_a.clone()
        for rep in range(3):                            # repeated launches reuse the plan's hand-off counters
            y_a.copy_(torch.from_numpy(y0).to(DEV, tdt))
            B.lora_delta(plan, dl.x, w.K, dl.At_ptrs, dl.Bt_ptrs, v, y_a, w.N, beta)
        B.lora_shrink(plan, dl.x, w.K, dl.At_ptrs, v)
        B.lora_expand(plan, v, dl.Bt_ptrs, y_b, w.N, beta)
        torch.cuda.synchronize()
        ranks_tok = np.where(tok >= 0, w.adapter_rank[np.clip(tok, 0, None)], 0)
        act = ranks_tok > 0
        ref = oracle.expand(w.x, tok, ad, w.N, y_in=(y0.astype(np.float64) if beta else None))
        got = _to_np(y_a)
        assert np.array_equal(got[~act], y0[~act]), "rows without adapter must stay bit-identical"
        if act.any():
            _assert_close(got[act], ref[act], _tol(w), f"lora_delta beta={beta}")
        if not fallback:
            # same arithmetic; bitwise equal when both paths slice K over 4 wavefronts, otherwise the fp32
            # summation order of v differs and a few y entries may round the other way
            if waves == 4 or not fused:
                assert torch.equal(y_a, y_b), "single launch and shrink+expand differ bitwise"
            else:
                assert oracle.error_metrics(_to_np(y_a), _to_np(y_b))[0] <= 5e-4
    torch.cuda.synchronize()
    plan.destroy()


def test_single_launch_delta_decode_config():
    w = wl.cfg2(with_w=False)
    plan = device.make_plan(w)
    plan.destroy()
    _delta_case(w)
    _delta_case(w, fallback=True)


def test_single_launch_delta_small_and_mixed_cases():
    for seed, (T, K, N, ranks) in enumerate([(37, 72, 200, (8, 16, 24, 32, 40, 64)), (120, 520, 1000, (8, 64)),
                                             (9, 4096, 256, (16,)), (300, 328, 72, (8, 16, 128))]):
        w = wl.random_case(400 + seed, T, K, N, 9, ranks, max_seg=12, frac_none=0.2,
                           scales=(0.5, 2.0, -1.5), empty_segments=True)
        _delta_case(w)                                  # rank 128 or big groups: falls back to two launches inside
        _delta_case(w, fallback=True)
    wf = wl.random_case(410, 33, 40, 48, 3, (4, 8), dtype="f32", max_seg=6, frac_none=0.2)
    _delta_case(wf)
    # more adapters than a wavefront has lanes, and exactly one
    wm = wl.random_case(411, 200, 1024, 320, 150, (8, 16, 32, 64), max_seg=2, scales=(1.0, 2.0))
    _delta_case(wm)
    _delta_case(wm, fallback=True)
    _delta_case(wl.random_case(412, 5, 2048, 128, 1, (64,), max_seg=8))


def test_single_launch_delta_large_decode_batch():
    # a decode batch several times the size of cfg2: far more workgroups than fit the GPU at once, so expand
    # blocks are dispatched long after their shrink blocks, and many adapter groups share the counters' table
    w = wl.random_case(413, 1536, 2048, 2048, 384, (8, 16, 32, 64), max_seg=1, scales=(1.0, 2.0, -0.5))
    _delta_case(w)


def test_traced_single_launch_gives_the_same_result_and_ordered_stamps():
    # the instrumented build of the single-launch kernel (lora_trace_set): same arithmetic as the ordinary build,
    # so the same bits in y; every workgroup's stamps are set and in phase order; a buffer that is too small
    # for the plan is an error and launches nothing
    w = wl.cfg2(with_w=False)
    dl = device.to_device(w, DEV, with_w=False)
    plan = device.make_plan(w)
    view = B.lora_plan_export(plan)
    assert (view["expand_tiles"][:, 5] >> 8).any(), "cfg2 is expected to run as one launch"
    S, E = view["shrink_tiles"].shape[0], view["expand_tiles"].shape[0]
    _, v_bytes, _ = B.lora_plan_query(plan)
    v = torch.zeros(v_bytes // 4, dtype=torch.float32, device=DEV)
    y0 = torch.from_numpy(wl.bf16_bits(wl.round_to_bf16(
        np.random.default_rng(5).standard_normal((w.T, w.N), dtype=np.float32))).view(np.int16)).to(DEV).view(torch.bfloat16)
    y_plain, y_traced = y0.clone(), y0.clone()
    B.lora_delta(plan, dl.x, w.K, dl.At_ptrs, dl.Bt_ptrs, v, y_plain, w.N, 1.0)
    trace = torch.zeros(S + E, 8, dtype=torch.int64, device=DEV)
    small = torch.zeros(S + E - 1, 8, dtype=torch.int64, device=DEV)
    try:
        B.lora_trace_set(small)
        with pytest.raises(B.LoraError) as err:
            B.lora_delta(plan, dl.x, w.K, dl.At_ptrs, dl.Bt_ptrs, v, y_traced, w.N, 1.0)
        assert err.value.status == B.LORA_ERR_WORKSPACE
        B.lora_trace_set(trace)
        B.lora_delta(plan, dl.x, w.K, dl.At_ptrs, dl.Bt_ptrs, v, y_traced, w.N, 1.0)
    finally:
        B.lora_trace_set(None)
    torch.cuda.synchronize()
    assert torch.equal(y_plain.view(torch.int16), y_traced.view(torch.int16))
    assert int(small.abs().sum()) == 0
    t = trace.cpu().numpy()
    sh, ex = t[:S], t[S:]
    assert (sh[:, :5] > 0).all() and (np.diff(sh[:, :5], axis=1) >= 0).all()
    assert (ex[:, :5] > 0).all() and (np.diff(ex[:, :5], axis=1) >= 0).all()
    done = ex[:, 5] > 0
    assert done.any() and (ex[done, 5] >= ex[done, 4]).all()
    assert set(np.unique(ex[:, 7])) <= {0, 1}
    assert (sh[:, 5] == 0).all() and (sh[:, 7] == 0).all()
    where = t[:, 6]
    assert ((where >> 32) < 8).all() and len(np.unique(where >> 32)) == 8, "every XCD takes part in a launch of this size"
    span_us = (t[:, :6].max() - t[:, 0].min()) * 1e3 / B.lora_trace_tick_khz()
    assert 1.0 < span_us < 1000.0, span_us                    # one launch of some microseconds
    # and the ordinary build again afterwards, untouched by the episode
    y_again = y0.clone()
    B.lora_delta(plan, dl.x, w.K, dl.At_ptrs, dl.Bt_ptrs, v, y_again, w.N, 1.0)
    torch.cuda.synchronize()
    assert torch.equal(y_plain.view(torch.int16), y_again.view(torch.int16))
    plan.destroy()


# ---------------------------------------------------------------- mixture mode (merged adapter + de-LoRA branch)
def run_mixture_case(w, m, n_sample=None, seed=11, variant=B.LORA_VARIANT_AUTO):
    """Mixture inference (section 4.4.1): adapter m is merged into the base weight (W' = W + s_m A_m B_m, stored in
    the workload's dtype), requests of m run on W' alone, every other request runs its own branch plus the removal
    of m.  The library gets the plain segment table, the plain pointer tables and `merged_adapter = m`; no
    concatenated matrix is built anywhere.  Checked:
      - lora_fused_forward on W' against the oracle on the same inputs (one rounding: the usual tolerance), and
        against plain unmerged inference on W (the identity of section 4.4.1; W' carries one more rounding);
      - lora_shrink's two shares of v against the oracle;
      - lora_delta (beta 1 and 0) against its contract: the removal is added first, the tokens' own branches are
        accumulated onto it, each pass rounding y once; rows of m's tokens stay bit-identical."""
    import dataclasses
    from oracle import plan_ref
    tdt = device.torch_dtype(w)
    rnd = wl.round_to_bf16 if w.dtype == "bf16" else (lambda a: np.asarray(a, np.float32))
    W_merged = rnd(oracle.merge(w.W, w.A[m], w.B[m], float(w.adapter_scale[m])).astype(np.float32))
    wm = dataclasses.replace(w, W=W_merged)
    dl = device.to_device(wm, DEV, with_w=True)
    plan = device.make_plan(w, variant, merged_adapter=m)
    view = B.lora_plan_export(plan)
    R, v_bytes, ws_bytes = B.lora_plan_query(plan)
    assert view["merged_adapter"] == m
    own_seg, removal = plan_ref.mixture_tables(w.T, w.seg_indptr, w.seg_adapter, w.adapter_rank, m)
    tok_plain = oracle.token_adapter(w.T, w.seg_indptr, w.seg_adapter)
    tok_own = oracle.token_adapter(w.T, w.seg_indptr, own_seg)
    tok_rem = np.where(removal, m, -1).astype(np.int32)
    ad = oracle.Adapters(w.adapter_rank, w.adapter_scale, w.A, w.B)
    neg = w.adapter_scale.copy()
    neg[m] = -neg[m]
    ad_neg = oracle.Adapters(w.adapter_rank, neg, w.A, w.B)
    rows = np.arange(w.T) if (n_sample is None or n_sample >= w.T) else _forward_rows(w, view, n_sample, seed)
    print(f"  mixture {w.name} merged={m} T={w.T} K={w.K} N={w.N} removal tokens={int(removal.sum())} "
          f"own-branch tokens={view['num_active']} oracle rows={rows.size}", flush=True)

    # whole layer in one call
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=DEV)
    y = torch.full((w.T, w.N), 9.0, dtype=tdt, device=DEV)
    B.lora_fused_forward(plan, dl.x, w.K, dl.Wt, w.K, dl.At_ptrs, dl.Bt_ptrs, y, w.N, ws, ws.numel())
    torch.cuda.synchronize()
    own_delta = oracle.expand(w.x, tok_own, ad, w.N, rows=rows)
    rem_delta = oracle.expand(w.x, tok_rem, ad_neg, w.N, rows=rows)
    y_ref = oracle.base(w.x, W_merged, rows=rows) + own_delta + rem_delta
    _assert_close(_to_np(y)[rows], y_ref, _tol(w), "mixture fused forward vs oracle on the merged weight")
    y_plain = oracle.forward(w.x, w.W, tok_plain, ad, rows=rows)
    nrm, _ = oracle.error_metrics(_to_np(y)[rows], y_plain)
    print(f"    mixture fused forward vs plain unmerged inference: normwise {nrm:.3e}", flush=True)
    # two independent roundings (W' and y) of 1.7e-3 normwise each
    assert nrm <= (3e-3 if w.dtype == "bf16" else 1e-5)

    # the two shares of v
    v = torch.full((max(v_bytes // 4, 4),), -12345.0, dtype=torch.float32, device=DEV)
    B.lora_shrink(plan, dl.x, w.K, dl.At_ptrs, v)
    torch.cuda.synchronize()
    v_np = v.cpu().numpy()
    vtol = V_TOL if w.dtype == "bf16" else F32_TOL
    for what, tok, a_, P, Rr, off in (("own", tok_own, ad, view["v_parts"], R, 0),
                                      ("removal", tok_rem, ad_neg, view["unmerge_v_parts"],
                                       view["unmerge_v_row_stride"], view["unmerge_v_offset"] // 4)):
        if not (tok >= 0).any():
            continue
        parts = v_np[off:off + P * w.T * Rr].reshape(P, w.T, Rr).astype(np.float64).sum(axis=0)
        ranks_tok = np.where(tok >= 0, w.adapter_rank[np.clip(tok, 0, None)], 0)
        valid = np.arange(Rr)[None, :] < ranks_tok[:, None]
        _assert_close(np.where(valid, parts, 0.0), oracle.shrink(w.x, tok, a_, apply_scale=True, R=Rr), vtol, f"mixture v ({what})")

    # lora_delta: two accumulating passes
    y0 = _y_in(w)
    is_m = ~removal
    for beta in (1.0, 0.0):
        yd = torch.from_numpy(y0).to(DEV, tdt)
        v.fill_(-12345.0)
        B.lora_delta(plan, dl.x, w.K, dl.At_ptrs, dl.Bt_ptrs, v, yd, w.N, beta)
        torch.cuda.synchronize()
        yd_np = _to_np(yd)
        assert np.array_equal(yd_np[is_m], y0[is_m]), "rows of the merged adapter's tokens must stay bit-identical"
        sel = rows[removal[rows]]
        if not sel.size:
            continue
        z1 = beta * y0[sel].astype(np.float64) + oracle.expand(w.x, tok_rem, ad_neg, w.N, rows=sel)
        own = oracle.expand(w.x, tok_own, ad, w.N, rows=sel)
        # Two roundings of y: the removal's pass leaves rnd(z1), z1 = beta y + removal, the own pass rnd(rnd(z1) + own).
        # Element by element against the exact z1 + own: |got - (z1 + own)| <= u |z1| + u |z1 + own| (+ fp32
        # accumulation slack) -- where the two terms cancel the result inherits the first rounding's error, which
        # a relative error of the small result would not bound.  Normwise against the two steps taken with the
        # oracle's values (the intermediate rounded as stored): one rounding apart, the usual tolerance.
        u = 2.0 ** -8 if w.dtype == "bf16" else 2.0 ** -24
        slack = 1e-4 if w.dtype == "bf16" else 1e-5
        nrm, _ = oracle.error_metrics(yd_np[sel], rnd(z1.astype(np.float32)).astype(np.float64) + own)
        excess = float((np.abs(yd_np[sel] - (z1 + own)) - (1.01 * u * (np.abs(z1) + np.abs(z1 + own)) + slack)).max())
        print(f"    mixture lora_delta beta={beta:g}: normwise {nrm:.3e}, worst excess over the two-rounding bound "
              f"{excess:.3e}", flush=True)
        assert nrm <= _tol(w)[0] and excess <= 0.0
    plan.destroy()


def test_mixture_mode_tiny_fp32_general_kernels():
    run_mixture_case(wl.cfg1(), 2)


def test_mixture_mode_small_cases():
    # unsorted segments, tokens without adapter, a rank-0 adapter, ragged sizes; merged adapter with few / many tokens
    w = wl.random_case(431, 300, 512, 328, 6, (8, 16, 32, 64), max_seg=40, frac_none=0.2, scales=(1.0, 2.0, -0.5))
    run_mixture_case(w, 1)
    run_mixture_case(w, 4, variant=B.LORA_VARIANT_GENERAL)
    # every token is the merged adapter's: nothing to compute
    T = 64
    one = wl.random_case(432, T, 256, 192, 2, (16,), max_seg=64)
    one = __import__("dataclasses").replace(one, seg_adapter=np.zeros_like(one.seg_adapter))
    run_mixture_case(one, 0)


def test_mixture_mode_cfg2_decode():
    w = wl.cfg2()
    counts = np.bincount(w.seg_adapter[w.seg_adapter >= 0], minlength=w.num_adapters)
    run_mixture_case(w, int(np.argmax(counts)))


def test_mixture_mode_cfg3_prefill():
    run_mixture_case(wl.cfg3(0), 1, n_sample=128)


def test_mixture_mode_cfg4_mixed():
    w = wl.cfg4()
    lens = np.diff(w.seg_indptr)
    counts = np.bincount(w.seg_adapter[w.seg_adapter >= 0], weights=lens[w.seg_adapter >= 0], minlength=w.num_adapters)
    run_mixture_case(w, int(np.argmax(counts)), n_sample=160)      # the most popular adapter is the merged one


# ---------------------------------------------------------------- mode switch (merge / unmerge)
def _merge_case(L, N, K, r, scale, dtype="bf16", variant=B.LORA_VARIANT_AUTO, ld_pad=0, seed=0, check_layers=None):
    print(f"  merge case L={L} N={N} K={K} r={r} s={scale} {dtype} variant={variant} ld_pad={ld_pad}", flush=True)
    rng = np.random.default_rng(700 + seed)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    rnd = wl.round_to_bf16 if dtype == "bf16" else (lambda a: np.asarray(a, np.float32))
    W = [rnd(rng.standard_normal((K, N), dtype=np.float32) * K ** -0.5) for _ in range(L)]
    A = [rnd(rng.standard_normal((K, r), dtype=np.float32) * K ** -0.5) for _ in range(L)]
    Bm = [rnd(rng.standard_normal((r, N), dtype=np.float32) * max(r, 1) ** -0.5) for _ in range(L)]
    ldw = K + ld_pad
    Wt = [torch.full((N, ldw), 7.0, dtype=tdt, device=DEV) for _ in range(L)]
    for l in range(L):
        Wt[l][:, :K] = torch.from_numpy(np.ascontiguousarray(W[l].T)).to(DEV, tdt)
    At = [torch.from_numpy(np.ascontiguousarray(a.T)).to(DEV, tdt).contiguous() for a in A]      # [r, K]
    Bt = [torch.from_numpy(np.ascontiguousarray(b.T)).to(DEV, tdt).contiguous() for b in Bm]     # [N, r]
    ptrs = lambda ts: torch.tensor([t.data_ptr() for t in ts] or [0], dtype=torch.int64, device=DEV)
    pW, pA, pB = ptrs(Wt), ptrs(At), ptrs(Bt)
    code = B.LORA_BF16 if dtype == "bf16" else B.LORA_F32
    B.lora_merge(L, N, K, r, scale, code, pW, ldw, pA, pB, variant)
    torch.cuda.synchronize()
    tol = BF16_TOL if dtype == "bf16" else F32_TOL
    layers = range(L) if check_layers is None else check_layers
    for l in layers:
        got = _to_np(Wt[l])
        assert np.all(got[:, K:] == 7.0), "written beyond column K"
        ref = oracle.merge(W[l], A[l], Bm[l], scale)                       # [K, N] float64
        _assert_close(got[:, :K], ref.T, tol, f"merged layer {l}")
    # unmerge: back to the original weights, to within the rounding of the two stores
    B.lora_merge(L, N, K, r, -scale, code, pW, ldw, pA, pB, variant)
    torch.cuda.synchronize()
    for l in layers:
        got = _to_np(Wt[l])[:, :K]
        if dtype != "bf16" or not r:
            _assert_close(got, W[l].T.astype(np.float64), tol, f"unmerged layer {l}")
        else:
            # not bit-exact: the merged weight was rounded to bf16 (half a step of |W'|, relative 2^-8 at
            # most), and so is the restored one (2^-8 of |W|)
            nrm, _ = oracle.error_metrics(got, W[l].T)
            bound = 2.0 ** -8 * (1.0 + np.linalg.norm(oracle.merge(W[l], A[l], Bm[l], scale)) / np.linalg.norm(W[l]))
            print(f"    unmerged layer {l}: normwise {nrm:.3e} (bound {bound:.3e})", flush=True)
            assert nrm <= bound
        if dtype == "bf16" and r:
            ulp = np.maximum(np.abs(W[l].T), 2.0 ** -126) * 2.0 ** -7       # one bf16 step at |w| (upper bound)
            big = np.maximum(ulp, np.abs(scale) * 2.0 ** -7 * np.abs(oracle.merge(0 * W[l], A[l], Bm[l], 1.0).T))
            assert np.all(np.abs(got - W[l].T) <= 2.5 * big + 1e-30), "unmerge is off by more than the two roundings"


def test_mode_switch_merge_unmerge():
    # streaming kernel: every rank class, ragged N (not a multiple of 128 / 16), ragged K (last stage, last
    # k-chunk), padded leading dimension, several layers; then the general kernel on the same and on odd shapes
    for seed, (L, N, K, r, s) in enumerate([(3, 192, 256, 8, 2.0), (2, 130, 1096, 96, -0.75), (1, 520, 2120, 128, 0.5),
                                            (4, 128, 64, 32, 1.0), (2, 1000, 328, 64, 2.0), (1, 16, 8, 16, 3.0)]):
        _merge_case(L, N, K, r, s, variant=B.LORA_VARIANT_TILED, seed=seed)
        _merge_case(L, N, K, r, s, variant=B.LORA_VARIANT_TILED, ld_pad=8, seed=seed)
        _merge_case(L, N, K, r, s, variant=B.LORA_VARIANT_GENERAL, seed=seed)
    _merge_case(2, 53, 77, 5, 1.5, ld_pad=3)                     # odd everything: general kernel
    _merge_case(2, 40, 48, 200, 0.25)                            # rank above 128: general kernel
    _merge_case(2, 33, 40, 4, 2.0, dtype="f32")
    _merge_case(0, 64, 64, 8, 1.0)
    _merge_case(2, 64, 64, 0, 1.0)
    with pytest.raises(B.LoraError):
        _merge_case(1, 53, 77, 5, 1.0, variant=B.LORA_VARIANT_TILED)


def test_mode_switch_model_sized():
    # the paper's mode-switch workload: every layer of a 7B-class model (32 x 4096 x 4096, rank 64) in one launch;
    # two layers are compared with the oracle in full
    _merge_case(32, 4096, 4096, 64, 2.0, check_layers=[0, 31])


# ---------------------------------------------------------------- vision task heads
def test_vision_task_heads_batched_through_the_shrink():
    # Vision task heads (paper section 4.2.2): a linear layer per adapter that maps the final feature of a
    # request's last token to C_a task outputs; heads of different width run in one batch.  In this library
    # that is the shrink with "rank" = C_a, Ht_a stored [C_a, K] like At_a, and scale 1: logits land in v.
    for seed, (classes, variant) in enumerate([((2, 5, 10, 101, 174, 256), B.LORA_VARIANT_AUTO),     # shrink alone tiled
                                               ((8, 16, 24, 64, 128), B.LORA_VARIANT_TILED)]):      # everything tiled
        w = wl.random_case(900 + seed, 96, 4096, 64, len(classes), classes, max_seg=1, frac_none=0.1,
                           scales=(1.0,), with_w=False)
        w.adapter_rank = np.asarray(classes, dtype=np.int32)         # one head of every width
        rng = np.random.default_rng(910 + seed)
        w.A = [wl.round_to_bf16(rng.standard_normal((w.K, c), dtype=np.float32) * w.K ** -0.5) for c in classes]
        w.B = [np.zeros((c, w.N), np.float32) for c in classes]
        dl = device.to_device(w, DEV, with_w=False)
        plan = device.make_plan(w, variant)
        R, v_bytes, _ = B.lora_plan_query(plan)
        view = B.lora_plan_export(plan)
        # widths of any kind run on the MFMA shrink (the rank demands of the tuned kernels are the expand's)
        assert view["shrink_kernel_family"] == B.LORA_VARIANT_TILED and view["shrink_tiles"].shape[0] > 0
        P = view["v_parts"]
        v = torch.full((P, w.T, R), -12345.0, dtype=torch.float32, device=DEV)
        B.lora_shrink(plan, dl.x, w.K, dl.At_ptrs, v)
        torch.cuda.synchronize()
        tok = oracle.token_adapter(w.T, w.seg_indptr, w.seg_adapter)
        ref = oracle.shrink(w.x, tok, oracle.Adapters(w.adapter_rank, w.adapter_scale, w.A, w.B), apply_scale=True, R=R)
        got = _to_np(v)
        width = np.where(tok >= 0, w.adapter_rank[np.clip(tok, 0, None)], 0)
        valid = np.arange(R)[None, :] < width[:, None]
        logits = np.where(valid, got.astype(np.float64).sum(axis=0), 0.0)
        assert np.all(got[0][~valid] == -12345.0), "written outside a head's C_a outputs"
        _assert_close(logits, ref, V_TOL, f"task-head logits, widths {classes}")
        # the decision a head exists for: the arg max agrees wherever the oracle's top two are not a near tie
        for t in np.nonzero(width > 1)[0]:
            top = np.sort(ref[t, :width[t]])[-2:]
            if top[1] - top[0] > 1e-3 * max(1.0, abs(top[1])):
                assert int(np.argmax(logits[t, :width[t]])) == int(np.argmax(ref[t, :width[t]]))
        plan.destroy()

