#!/usr/bin/env python3
"""Benchmark of the heterogeneous-LoRA delta path on one MI355X.

Workload: the decode-shaped configuration (256 single-token requests, hidden
4096 -> 4096, 64 adapters of rank {8,16,32,64}, unsorted adapter ids), the
4096-d heterogeneous batch the headline metric is quoted on.  A *step* is one
batch through LAYERS distinct layer-projections: one lora_plan (host planning +
table upload) followed, per layer, by lora_shrink and lora_expand (beta = 1,
accumulating onto a resident base output).  Every layer has its own x, A, B and
y buffers (> 1 GB in total) so that nothing is served from the 256 MB last-level
cache across layers.  All inputs are resident in HBM before the timed region.

Prints ONE JSON line: value = microseconds per layer of the whole step
(lower is better), plus the roofline of the dominant kernel (per-kernel
durations from event pairs attached to each launch) and the CPU oracle timed on
this host's cores.
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
# HBM bytes per launch from rocprofv3 FETCH_SIZE / WRITE_SIZE runs, scaled by a 256 MiB copy
# (profiles/decode_cfg2_hbm_traffic.txt); keyed by workload and kernel
MEASURED_TRAFFIC = {("cfg2_decode", "delta_fused_small_kernel"): 45.81e6}


def algorithmic_bytes(w, beta=1.0):
    """Bytes the method itself must move per launch: every active adapter's
    factor once, x / y rows of active tokens once, v once (fp32)."""
    import numpy as np
    tok = w.token_adapter()
    active = tok >= 0
    ranks_tok = np.where(active, w.adapter_rank[np.clip(tok, 0, None)], 0)
    act_tok = ranks_tok > 0
    r_tok = int(ranks_tok.sum())
    used = np.unique(tok[act_tok])
    r_act = int(w.adapter_rank[used].sum())
    t_act = int(act_tok.sum())
    e = 4 if w.dtype == "f32" else 2
    shrink = t_act * w.K * e + r_act * w.K * e + 4 * r_tok
    expand = 4 * r_tok + r_act * w.N * e + int((1 + beta) * t_act * w.N * e)
    flops = 2 * r_tok * (w.K + w.N)
    return shrink, expand, flops


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--workload", default="cfg2", choices=["cfg2", "cfg3", "cfg4", "cfg4d", "cfg5"])
    ap.add_argument("--cpu-seconds", type=float, default=10.0, help="CPU time budget of the oracle leg (0 = skip)")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--two-launches", action="store_true", help="lora_shrink + lora_expand instead of lora_delta")
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

    if args.workload == "cfg5":
        w = wl.cfg5("attn", with_w=False)
    else:
        w = wl.CONFIGS[args.workload](with_w=False)
    L = args.layers
    # big configurations: fewer buffer sets are enough to exceed the last-level cache
    per_layer_bytes = 2 * (w.T * w.K + w.T * w.N + sum(a.size for a in w.A) + sum(b.size for b in w.B))
    L = max(2, min(L, int(24e9 // max(per_layer_bytes, 1))))

    # ---- layer buffer sets: layer 0 holds the seeded numpy draw, the others are
    # drawn on the device with the same shapes and variances
    layer0 = device.to_device(w, dev, with_w=False)
    gen = torch.Generator(device=dev)
    gen.manual_seed(24110915)
    layers = []
    for l in range(L):
        if l == 0:
            x, At_buf, Bt_buf, At_ptrs, Bt_ptrs = layer0.x, layer0.At_buf, layer0.Bt_buf, layer0.At_ptrs, layer0.Bt_ptrs
        else:
            x = torch.randn(w.T, w.K, generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
            At_buf = torch.empty_like(layer0.At_buf)
            Bt_buf = torch.empty_like(layer0.Bt_buf)
            for a in range(w.num_adapters):
                r = int(w.adapter_rank[a])
                oa, ob = int(layer0.At_off[a]), int(layer0.Bt_off[a])
                At_buf[oa:oa + r * w.K] = (torch.randn(r * w.K, generator=gen, device=dev) * (w.K ** -0.5)).to(torch.bfloat16)
                Bt_buf[ob:ob + r * w.N] = (torch.randn(r * w.N, generator=gen, device=dev) * (max(r, 1) ** -0.5)).to(torch.bfloat16)
            es = At_buf.element_size()
            At_ptrs = torch.tensor([At_buf.data_ptr() + int(o) * es for o in layer0.At_off], dtype=torch.int64, device=dev)
            Bt_ptrs = torch.tensor([Bt_buf.data_ptr() + int(o) * es for o in layer0.Bt_off], dtype=torch.int64, device=dev)
        y = torch.randn(w.T, w.N, generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
        layers.append((x, At_buf, Bt_buf, At_ptrs, Bt_ptrs, y))

    plan0 = device.make_plan(w)
    R, v_bytes, _ = B.lora_plan_query(plan0)
    v = torch.zeros(v_bytes // 4, dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()
    abi_dtype = device.abi_dtype(w)

    def run_layers(plan):
        for (x, _a, _b, At_ptrs, Bt_ptrs, y) in layers:
            if args.two_launches:
                B.lora_shrink(plan, x, w.K, At_ptrs, v, stream)
                B.lora_expand(plan, v, Bt_ptrs, y, w.N, 1.0, stream)
            else:
                B.lora_delta(plan, x, w.K, At_ptrs, Bt_ptrs, v, y, w.N, 1.0, stream)

    keep = []

    def step():
        plan = B.lora_plan(w.T, w.seg_indptr, w.seg_adapter, w.adapter_rank, w.adapter_scale, w.K, w.N, abi_dtype)
        B.lora_plan_upload(plan, stream)
        run_layers(plan)
        keep.append(plan)          # destroyed after the work has finished

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    for p in keep:
        p.destroy()
    keep.clear()

    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for p in keep:
        p.destroy()
    keep.clear()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    us_per_layer = ms_per_step * 1e3 / L

    # ---- host planning cost alone
    tp0 = time.perf_counter()
    for _ in range(200):
        B.lora_plan(w.T, w.seg_indptr, w.seg_adapter, w.adapter_rank, w.adapter_scale, w.K, w.N, abi_dtype).destroy()
    plan_us = (time.perf_counter() - tp0) * 1e6 / 200

    # ---- per-kernel durations (event pair attached to every launch)
    B.lora_plan_upload(plan0, stream)
    torch.cuda.synchronize()
    B.lora_timing_begin()
    for _ in range(max(2, min(args.steps, 10))):
        run_layers(plan0)
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
                    for (x, _a, _b, At_ptrs, Bt_ptrs, y) in layers:
                        if args.two_launches:
                            B.lora_shrink(plan0, x, w.K, At_ptrs, v, side)
                            B.lora_expand(plan0, v, Bt_ptrs, y, w.N, 1.0, side)
                        else:
                            B.lora_delta(plan0, x, w.K, At_ptrs, Bt_ptrs, v, y, w.N, 1.0, side)
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
            graph_us_per_layer = None
            print(f"bench.py: graph replay leg failed: {exc}", file=sys.stderr)

    if args.calib_copy_mb > 0:
        src = torch.empty(args.calib_copy_mb << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()

    sh_bytes, ex_bytes, flops = algorithmic_bytes(w, beta=1.0)
    names = {"shrink": "shrink_tiled_kernel", "expand": "expand_tiled_kernel", "delta": "delta_fused_small_kernel"}
    ksum = {}
    for key, nm in names.items():
        if nm in kern:
            by = {"shrink": sh_bytes, "expand": ex_bytes, "delta": sh_bytes + ex_bytes}[key]
            ksum[key] = dict(kernel=nm, avg_us=kern[nm]["avg_us"], min_us=kern[nm]["min_us"], launches=kern[nm]["count"],
                             algorithmic_bytes=by, achieved_GBs=by / kern[nm]["avg_us"] * 1e-3)
    dom = max(ksum.values(), key=lambda d: d["avg_us"]) if ksum else None
    roofline = None
    if dom:
        roofline = dict(bound="hbm", kernel=dom["kernel"], achieved=round(dom["achieved_GBs"], 1), peak=HBM_PEAK_GBS,
                        unit="GB/s", frac=round(dom["achieved_GBs"] / HBM_PEAK_GBS, 4),
                        traffic=MEASURED_TRAFFIC.get((w.name, dom["kernel"])),
                        avg_kernel_us=round(dom["avg_us"], 3), algorithmic_bytes=dom["algorithmic_bytes"])

    # ---- CPU oracle on this host's cores: the same delta path (shrink + expand-add), layer 0's inputs
    cpu = None
    if args.cpu_seconds > 0:
        import oracle
        tok = oracle.token_adapter(w.T, w.seg_indptr, w.seg_adapter)
        ad = oracle.Adapters(w.adapter_rank, w.adapter_scale, w.A, w.B)
        y_in = layers[0][5].float().cpu().numpy().astype(np.float64)
        n_rows = w.T
        rows = None
        oracle.expand(w.x, tok, ad, w.N, y_in=y_in[:8], rows=np.arange(8))       # warm the library
        tc0 = time.perf_counter()
        reps = 0
        while True:
            oracle.expand(w.x, tok, ad, w.N, y_in=y_in, rows=rows)
            reps += 1
            if time.perf_counter() - tc0 >= args.cpu_seconds or reps >= 1000:
                break
        cpu_us = (time.perf_counter() - tc0) * 1e6 / reps
        cpu = dict(value=round(cpu_us, 1), unit="us/layer", cores=oracle.num_threads(), kind="oracle",
                   sample=f"all {n_rows} tokens of layer 0 of {w.name} (float64 shrink + expand-add), {reps} repetitions")

    out = {
        "metric": "LoRA-delta us/layer (shrink+expand, plan amortised over the layers of a step)",
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
                   "launch": "eager, one lora_plan per step, " +
                             ("lora_shrink + lora_expand per layer" if args.two_launches else "lora_delta per layer")},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "kernels": {k: {kk: (round(vv, 3) if isinstance(vv, float) else vv) for kk, vv in d.items()} for k, d in ksum.items()},
        "gpu_kernel_us_per_layer": round(sum(d["avg_us"] for d in ksum.values()), 3) if ksum else None,
        "graph_replay_us_per_layer": round(graph_us_per_layer, 3) if graph_us_per_layer else None,
        "plan_host_us": round(plan_us, 2),
        "delta_flops_per_layer": flops,
    }
    print(json.dumps(out))
    plan0.destroy()


if __name__ == "__main__":
    main()
