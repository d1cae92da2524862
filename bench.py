#!/usr/bin/env python3
"""Benchmark of the heterogeneous-LoRA operator on one MI355X.

Default workload: the decode-shaped configuration (256 single-token requests,
hidden 4096 -> 4096, 64 adapters of rank {8,16,32,64}, unsorted adapter ids),
the 4096-d heterogeneous batch the headline metric is quoted on.  A *step* is
one batch through LAYERS distinct layer-projections: one lora_plan (host
planning + table upload) followed, per layer, by the delta path
y += s (x A_a) B_a  (lora_delta: shrink + expand; one launch for decode-shaped
batches), accumulating onto a resident base output.  Every layer has its own
x, A, B and y buffers (> 1 GB in total for the default) so that nothing is
served from the 256 MB last-level cache across layers.  All inputs are
resident in HBM before the timed region.

Other legs: --path two-launches (lora_shrink + lora_expand), --path fused
(lora_fused_forward: base GEMM with the delta in its epilogue, MFMA roofline),
--workload cfg3|cfg4|cfg4d|cfg5|cfg5mlp.

Prints ONE JSON line: value = microseconds per layer of the whole step (lower
is better), the roofline of the dominant kernel (per-kernel durations from an
event pair attached to each launch) and the CPU oracle timed on this host.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
# HBM bytes per launch from rocprofv3 FETCH_SIZE / WRITE_SIZE runs, scaled by a 256 MiB copy
# (profiles/decode_cfg2_hbm_traffic.txt); keyed by workload and kernel
MEASURED_TRAFFIC = {("cfg2_decode", "delta_fused_small_kernel"): 46.00e6,
                    ("cfg5_large_attn", "expand_stream_kernel"): 534.80e6,     # profiles/prefill_cfg5_shrink_expand_hbm_traffic.txt
                    ("cfg5_large_attn", "shrink_stream_kernel"): 332.00e6}

KERNEL_KEYS = {"shrink_tiled_kernel": "shrink", "expand_tiled_kernel": "expand", "delta_fused_small_kernel": "delta",
               "shrink_stream_kernel": "shrink", "expand_stream_kernel": "expand", "v_split_kernel": "v_split",
               "gemm_tiled_kernel": "gemm", "gemm_tiled_kernel<delta>": "gemm_delta",
               "gemm_ring_kernel": "gemm", "gemm_ring_kernel<delta>": "gemm_delta",
               "shrink_general_kernel": "shrink", "expand_general_kernel": "expand", "gemm_general_kernel": "gemm"}


def algorithmic_work(w, beta=1.0):
    """Bytes and flops the method itself must move / do per launch: every active
    adapter's factor once, x / y rows of active tokens once, v once (fp32)."""
    import numpy as np
    tok = w.token_adapter()
    ranks_tok = np.where(tok >= 0, w.adapter_rank[np.clip(tok, 0, None)], 0)
    act_tok = ranks_tok > 0
    r_tok = int(ranks_tok.sum())
    r_act = int(w.adapter_rank[np.unique(tok[act_tok])].sum())
    t_act = int(act_tok.sum())
    e = 4 if w.dtype == "f32" else 2
    shrink = t_act * w.K * e + r_act * w.K * e + 4 * r_tok
    expand = 4 * r_tok + r_act * w.N * e + int((1 + beta) * t_act * w.N * e)
    gemm = (w.T * w.K + w.K * w.N + w.T * w.N) * e
    return dict(shrink_bytes=shrink, expand_bytes=expand, delta_bytes=shrink + expand,
                gemm_bytes=gemm, gemm_delta_bytes=gemm + r_act * w.N * e + 4 * r_tok,
                delta_flops=2 * r_tok * (w.K + w.N), shrink_flops=2 * r_tok * w.K, expand_flops=2 * r_tok * w.N,
                gemm_flops=2 * w.T * w.K * w.N, gemm_delta_flops=2 * w.T * w.K * w.N + 2 * r_tok * w.N)


def bench_merge(args, torch, B, dev):
    """Mode switch: one adapter (rank 64) merged into every one of 32 4096x4096 projections in one launch
    (lora_merge), alternating merge / unmerge; a step is one such launch."""
    L, N, K, r, s = 32, 4096, 4096, 64, 2.0
    gen = torch.Generator(device=dev)
    gen.manual_seed(24110915)
    rnd = lambda n, std: (torch.randn(n, generator=gen, device=dev) * std).to(torch.bfloat16)
    Wt = [rnd(N * K, K ** -0.5).view(N, K) for _ in range(L)]
    At = [rnd(r * K, K ** -0.5).view(r, K) for _ in range(L)]
    Bt = [rnd(N * r, r ** -0.5).view(N, r) for _ in range(L)]
    ptrs = lambda ts: torch.tensor([t.data_ptr() for t in ts], dtype=torch.int64, device=dev)
    pW, pA, pB = ptrs(Wt), ptrs(At), ptrs(Bt)
    stream = torch.cuda.current_stream()
    sign = [1.0]

    def step():
        B.lora_merge(L, N, K, r, s * sign[0], B.LORA_BF16, pW, K, pA, pB, stream=stream)
        sign[0] = -sign[0]

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    B.lora_timing_begin()
    for _ in range(min(args.steps, 20)):
        step()
    torch.cuda.synchronize()
    kern = B.lora_timing_end()["merge_kernel"]
    by = L * (2 * N * K * 2 + (N + K) * r * 2)           # every weight read and written once, the factors read once
    fl = 2 * L * N * K * r
    print(json.dumps({
        "metric": "mode switch ms (one adapter merged into / removed from all layers, one launch)",
        "value": round(ms_per_step, 4), "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "merge7b", "layers": L, "n": N, "k": K, "rank": r,
                   "launch": "eager, lora_merge per step, alternating +scale / -scale"},
        "roofline": {"bound": "hbm", "kernel": "merge_stream_kernel", "achieved": round(by / kern["avg_us"] * 1e-3, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(by / kern["avg_us"] * 1e-3 / HBM_PEAK_GBS, 4),
                     "traffic": None, "avg_kernel_us": round(kern["avg_us"], 3), "algorithmic_bytes": by},
        "cpu_baseline": None,
        "kernels": {"merge": {"kernel": "merge_stream_kernel", "avg_us": round(kern["avg_us"], 3),
                              "min_us": round(kern["min_us"], 3), "launches": kern["count"],
                              "algorithmic_bytes": by, "algorithmic_flops": fl}}}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--workload", default="cfg2", choices=["cfg2", "cfg3", "cfg4", "cfg4d", "cfg5", "cfg5mlp", "merge7b"])
    ap.add_argument("--path", default="delta", choices=["delta", "two-launches", "fused"])
    ap.add_argument("--cpu-seconds", type=float, default=10.0, help="CPU time budget of the oracle leg (0 = skip)")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--calib-copy-mb", type=int, default=0,
                    help="also run one plain device copy of this many MiB (a known-size reference for profiler counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is a single-GPU kernel path; it has no multi-GPU mode. "
              "Run with --gpus 1 (throughput of N replicas is N times this figure by construction).",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2411_00915_amd import binding as B
    from paper_2411_00915_amd import device, workloads as wl

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.workload == "merge7b":
        return bench_merge(args, torch, B, dev)
    fused = args.path == "fused"

    if args.workload in ("cfg5", "cfg5mlp"):
        w = wl.cfg5("attn" if args.workload == "cfg5" else "mlp", with_w=False)
    else:
        w = wl.CONFIGS[args.workload](with_w=False)
    # big configurations: fewer buffer sets are enough to exceed the last-level cache
    per_layer_bytes = 2 * (w.T * w.K + w.T * w.N + sum(a.size for a in w.A) + sum(b.size for b in w.B)
                           + (w.K * w.N if fused else 0))
    L = max(2, min(args.layers, int(24e9 // max(per_layer_bytes, 1))))

    # ---- layer buffer sets: layer 0 holds the seeded numpy draw, the others are
    # drawn on the device with the same shapes and variances
    layer0 = device.to_device(w, dev, with_w=False)
    gen = torch.Generator(device=dev)
    gen.manual_seed(24110915)

    def randn_bf16(n, std):
        return (torch.randn(n, generator=gen, device=dev) * std).to(torch.bfloat16)

    layers = []
    for l in range(L):
        if l == 0:
            x, At_buf, Bt_buf, At_ptrs, Bt_ptrs = layer0.x, layer0.At_buf, layer0.Bt_buf, layer0.At_ptrs, layer0.Bt_ptrs
        else:
            x = randn_bf16(w.T * w.K, 1.0).view(w.T, w.K)
            At_buf = torch.empty_like(layer0.At_buf)
            Bt_buf = torch.empty_like(layer0.Bt_buf)
            for a in range(w.num_adapters):
                r = int(w.adapter_rank[a])
                oa, ob = int(layer0.At_off[a]), int(layer0.Bt_off[a])
                At_buf[oa:oa + r * w.K] = randn_bf16(r * w.K, w.K ** -0.5)
                Bt_buf[ob:ob + r * w.N] = randn_bf16(r * w.N, max(r, 1) ** -0.5)
            es = At_buf.element_size()
            At_ptrs = torch.tensor([At_buf.data_ptr() + int(o) * es for o in layer0.At_off], dtype=torch.int64, device=dev)
            Bt_ptrs = torch.tensor([Bt_buf.data_ptr() + int(o) * es for o in layer0.Bt_off], dtype=torch.int64, device=dev)
        y = randn_bf16(w.T * w.N, 1.0).view(w.T, w.N)
        Wt = randn_bf16(w.N * w.K, w.K ** -0.5).view(w.N, w.K) if fused else None
        layers.append((x, At_ptrs, Bt_ptrs, y, Wt, At_buf, Bt_buf))

    plan0 = device.make_plan(w)
    _, v_bytes, ws_bytes = B.lora_plan_query(plan0)
    v = torch.zeros(max(v_bytes // 4, 64), dtype=torch.float32, device=dev)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)
    abi_dtype = device.abi_dtype(w)

    def run_layers(plan, stream):
        for (x, At_ptrs, Bt_ptrs, y, Wt, _a, _b) in layers:
            if args.path == "delta":
                B.lora_delta(plan, x, w.K, At_ptrs, Bt_ptrs, v, y, w.N, 1.0, stream)
            elif args.path == "two-launches":
                B.lora_shrink(plan, x, w.K, At_ptrs, v, stream)
                B.lora_expand(plan, v, Bt_ptrs, y, w.N, 1.0, stream)
            else:
                B.lora_fused_forward(plan, x, w.K, Wt, w.K, At_ptrs, Bt_ptrs, y, w.N, ws, ws.numel(), stream)

    stream = torch.cuda.current_stream()
    keep = []

    def step():
        plan = B.lora_plan(w.T, w.seg_indptr, w.seg_adapter, w.adapter_rank, w.adapter_scale, w.K, w.N, abi_dtype)
        B.lora_plan_upload(plan, stream)
        run_layers(plan, stream)
        keep.append(plan)          # destroyed after the work has finished

    def drain():
        torch.cuda.synchronize()
        for p in keep:
            p.destroy()
        keep.clear()

    for _ in range(args.warmup):
        step()
    drain()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    drain()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    us_per_layer = ms_per_step * 1e3 / L

    # ---- host planning cost alone
    tp0 = time.perf_counter()
    for _ in range(100):
        B.lora_plan(w.T, w.seg_indptr, w.seg_adapter, w.adapter_rank, w.adapter_scale, w.K, w.N, abi_dtype).destroy()
    plan_us = (time.perf_counter() - tp0) * 1e6 / 100

    # ---- per-kernel durations (event pair attached to every launch)
    B.lora_plan_upload(plan0, stream)
    torch.cuda.synchronize()
    B.lora_timing_begin()
    for _ in range(max(2, min(args.steps, 10))):
        run_layers(plan0, stream)
    kern = B.lora_timing_end()

    # ---- the same sweep replayed from a HIP graph (no host launch cost)
    graph_us_per_layer = None
    if not args.no_graph:
        try:
            g = torch.cuda.CUDAGraph()
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                with torch.cuda.graph(g, stream=side):
                    run_layers(plan0, side)
            torch.cuda.current_stream().wait_stream(side)
            for _ in range(3):
                g.replay()
            torch.cuda.synchronize()
            reps = max(5, args.steps)
            tg0 = time.perf_counter()
            for _ in range(reps):
                g.replay()
            torch.cuda.synchronize()
            graph_us_per_layer = (time.perf_counter() - tg0) * 1e6 / reps / L
        except Exception as exc:  # report, never hide
            print(f"bench.py: graph replay leg failed: {exc}", file=sys.stderr)

    if args.calib_copy_mb > 0:
        src = torch.empty(args.calib_copy_mb << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()

    work = algorithmic_work(w, beta=1.0)
    ksum = {}
    for nm, d in kern.items():
        key = KERNEL_KEYS.get(nm, nm)
        by, fl = work.get(key + "_bytes"), work.get(key + "_flops")
        ksum[key] = dict(kernel=nm, avg_us=d["avg_us"], min_us=d["min_us"], launches=d["count"],
                         algorithmic_bytes=by, achieved_GBs=(by / d["avg_us"] * 1e-3 if by else None),
                         algorithmic_flops=fl, achieved_TFLOPs=(fl / d["avg_us"] * 1e-6 if fl else None))
    roofline = None
    if ksum:
        dom = max(ksum.values(), key=lambda d: d["avg_us"])
        if dom["kernel"].startswith("gemm"):
            roofline = dict(bound="mfma", kernel=dom["kernel"], achieved=round(dom["achieved_TFLOPs"], 1),
                            peak=MFMA_BF16_PEAK_TFLOPS, unit="TFLOP/s",
                            frac=round(dom["achieved_TFLOPs"] / MFMA_BF16_PEAK_TFLOPS, 4), traffic=None,
                            avg_kernel_us=round(dom["avg_us"], 3), algorithmic_flops=dom["algorithmic_flops"])
        else:
            roofline = dict(bound="hbm", kernel=dom["kernel"], achieved=round(dom["achieved_GBs"], 1), peak=HBM_PEAK_GBS,
                            unit="GB/s", frac=round(dom["achieved_GBs"] / HBM_PEAK_GBS, 4),
                            traffic=MEASURED_TRAFFIC.get((w.name, dom["kernel"])),
                            avg_kernel_us=round(dom["avg_us"], 3), algorithmic_bytes=dom["algorithmic_bytes"])

    # ---- CPU oracle on this host's cores: the delta path (shrink + expand-add) of layer 0
    cpu = None
    if args.cpu_seconds > 0:
        import oracle
        tok = oracle.token_adapter(w.T, w.seg_indptr, w.seg_adapter)
        ad = oracle.Adapters(w.adapter_rank, w.adapter_scale, w.A, w.B)
        n_rows = min(w.T, 512)                                   # bounded sample for the big configurations
        rows = None if n_rows == w.T else np.arange(0, w.T, w.T // n_rows)[:n_rows]
        sel = np.arange(w.T) if rows is None else rows
        y_in = layers[0][3].float().cpu().numpy().astype(np.float64)[sel]
        oracle.expand(w.x, tok, ad, w.N, y_in=y_in[:8], rows=sel[:8])       # warm the library
        tc0 = time.perf_counter()
        reps = 0
        while True:
            oracle.expand(w.x, tok, ad, w.N, y_in=y_in, rows=rows)
            reps += 1
            if time.perf_counter() - tc0 >= args.cpu_seconds or reps >= 1000:
                break
        cpu_us = (time.perf_counter() - tc0) * 1e6 / reps * (w.T / n_rows)
        cpu = dict(value=round(cpu_us, 1), unit="us/layer", cores=oracle.num_threads(), kind="oracle",
                   sample=(f"{n_rows} of {w.T} tokens of layer 0 of {w.name} (float64 shrink + expand-add), "
                           f"{reps} repetitions" + ("" if rows is None else ", scaled linearly to all tokens")))

    def rnd(d):
        return {k: (round(x, 3) if isinstance(x, float) else x) for k, x in d.items() if x is not None}

    what = {"delta": "lora_delta per layer", "two-launches": "lora_shrink + lora_expand per layer",
            "fused": "lora_fused_forward per layer (shrink + base GEMM with delta epilogue)"}[args.path]
    out = {
        "metric": ("LoRA-delta us/layer (shrink+expand, plan amortised over the layers of a step)" if not fused else
                   "fused layer us/layer (xW + delta, plan amortised over the layers of a step)"),
        "value": round(us_per_layer, 3),
        "unit": "us/layer",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": w.name, "tokens": w.T, "k": w.K, "n": w.N, "adapters": w.num_adapters,
                   "ranks": sorted(set(int(r) for r in w.adapter_rank)), "layers_per_step": L,
                   "launch": "eager, one lora_plan per step, " + what},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "kernels": {k: rnd(d) for k, d in ksum.items()},
        "gpu_kernel_us_per_layer": round(sum(d["avg_us"] for d in ksum.values()), 3) if ksum else None,
        "graph_replay_us_per_layer": round(graph_us_per_layer, 3) if graph_us_per_layer else None,
        "plan_host_us": round(plan_us, 2),
    }
    print(json.dumps(out))
    plan0.destroy()


if __name__ == "__main__":
    main()
