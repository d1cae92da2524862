"""lora_delta_static -- the entry point that allocates nothing -- against lora_delta.

Both run the same kernels on the same plan; only the home of v and of the hand-off counters differs (a device array
inside the library instead of caller / plan memory), so the outputs must agree bit for bit -- tighter than the
tolerance the parity tests grant against the oracle, which is checked here as well.  Two calls in a row share the
array, the second with a smaller batch of another shape class (single launch with counters after the two-launch
streaming path, and the other way round)."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
from paper_2411_00915_amd import binding as B
from paper_2411_00915_amd import device, workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(w, beta):
    dl = device.to_device(w, DEV, with_w=False)
    tdt = device.torch_dtype(w)
    plan = device.make_plan(w)
    _, v_bytes, _ = B.lora_plan_query(plan)
    assert v_bytes <= B.LORA_STATIC_V_BYTES
    B.lora_plan_upload(plan)                                   # set-up: the only step that allocates
    rng = np.random.default_rng(5)
    y0 = rng.standard_normal((w.T, w.N), dtype=np.float32)
    y0 = wl.round_to_bf16(y0) if w.dtype == "bf16" else y0
    y_ref_path = torch.from_numpy(y0).to(DEV, tdt)
    v = torch.zeros(max(v_bytes // 4, 4), dtype=torch.float32, device=DEV)
    B.lora_delta(plan, dl.x, w.K, dl.At_ptrs, dl.Bt_ptrs, v, y_ref_path, w.N, beta)
    y_static = torch.from_numpy(y0).to(DEV, tdt)
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    B.lora_delta_static(plan, dl.x, w.K, dl.At_ptrs, dl.Bt_ptrs, y_static, w.N, beta)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before, "device memory was allocated or freed during the call"
    assert torch.equal(y_static, y_ref_path), f"{w.name}: lora_delta_static differs from lora_delta"
    tok = oracle.token_adapter(w.T, w.seg_indptr, w.seg_adapter)
    ad = oracle.Adapters(w.adapter_rank, w.adapter_scale, w.A, w.B)
    ref = oracle.expand(w.x, tok, ad, w.N, y_in=(y0.astype(np.float64) if beta else None))
    act = np.where(tok >= 0, w.adapter_rank[np.clip(tok, 0, None)], 0) > 0
    got = y_static.float().cpu().numpy()
    assert np.array_equal(got[~act], y0[~act])
    nrm, elem = oracle.error_metrics(got[act], ref[act])
    print(f"  {w.name} T={w.T} beta={beta}: normwise {nrm:.3e} elementwise {elem:.3e}", flush=True)
    assert nrm <= 2e-3 and elem <= 1e-2
    plan.destroy()


def test_static_entry_point_matches_lora_delta_on_two_calls_in_a_row():
    big_stream = wl.random_case(951, 2900, 1024, 1536, 14, (16, 32, 64, 128), max_seg=400, frac_none=0.1, scales=(2.0, -0.5))
    small_decode = wl.random_case(952, 150, 1024, 640, 40, (8, 16, 32, 64), max_seg=2, frac_none=0.1, scales=(1.0, 2.0))
    big_decode = wl.random_case(953, 700, 512, 1024, 200, (8, 16, 32, 64), max_seg=1, scales=(1.0, -2.0))
    tiny_general = wl.random_case(954, 33, 77, 53, 4, (3, 5, 12), max_seg=6, frac_none=0.2)
    odd_ranks = wl.random_case(955, 90, 1024, 328, 6, (3, 12, 100, 200), max_seg=4, frac_none=0.1)   # tiled shrink, general expand
    for first, second in ((big_stream, small_decode), (big_decode, small_decode), (small_decode, tiny_general),
                          (big_decode, odd_ranks)):
        for beta in (1.0, 0.0):
            _case(first, beta)
            _case(second, beta)


def test_static_entry_point_refuses_what_does_not_fit_or_is_not_uploaded():
    # v of 40000 x 128 floats is 20 MB: beyond the array (refused before anything is launched)
    w = wl.random_case(955, 40000, 64, 64, 2, (128,), max_seg=5000, with_w=False)
    plan = device.make_plan(w)
    assert B.lora_plan_query(plan)[1] > B.LORA_STATIC_V_BYTES
    dummy = torch.zeros(64, dtype=torch.bfloat16, device=DEV)
    ptrs = torch.zeros(2, dtype=torch.int64, device=DEV)
    with pytest.raises(B.LoraError) as e:
        B.lora_delta_static(plan, dummy, w.K, ptrs, ptrs, dummy, w.N, 1.0)
    assert e.value.status == B.LORA_ERR_UNSUPPORTED
    plan.destroy()
    # a plan that is not on the device yet: the call must not upload (allocate) it
    w = wl.random_case(956, 20, 64, 64, 2, (8,), with_w=False)
    plan = device.make_plan(w)
    with pytest.raises(B.LoraError) as e:
        B.lora_delta_static(plan, dummy, w.K, ptrs, ptrs, dummy, w.N, 1.0)
    assert e.value.status == B.LORA_ERR_INVALID_ARG
    torch.cuda.synchronize()
    plan.destroy()
