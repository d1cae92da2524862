#!/usr/bin/env python3
"""Benchmark of the heterogeneous-LoRA operator on one MI355X.

Headline workload: the decode-shaped configuration (256 single-token requests, hidden 4096 -> 4096, 64 adapters of
rank {8,16,32,64}, unsorted adapter ids), the 4096-d heterogeneous batch the metric is quoted on.  A *step* is one
batch through LAYERS distinct layer-projections: one lora_plan (host planning, shape-table lookup, table upload)
followed, per layer, by the delta path  y += s (x A_a) B_a  (lora_delta: shrink + expand; one launch for
decode-shaped batches), accumulating onto a resident base output.  Every layer has its own x, A, B and y buffers
(> 1 GB in total for the headline) so that nothing is served from the 256 MB last-level cache across layers.  All
inputs are resident in HBM before the timed region.  Protocol (the paper's, section 6.3.2): warm-up steps, then the
timed steps; per-step durations give median / p90 / p95.

Prints ONE JSON line.  value = microseconds per layer of the headline step (lower is better), with the roofline of
its dominant kernel (per-kernel durations from an event pair attached to each launch) and the CPU oracle timed on
this host.  Two more objects ride on the line:
  configs   the other configurations (vision prefill, mixed serving batch and its companion with decode requests,
            the large fused-layer case in both shapes) through lora_delta, lora_base_gemm and lora_fused_forward --
            microseconds per layer with median / p90 / p95, per-kernel averages, algorithmic bytes / flops, roofline
            fraction of the dominant kernel, fusion gain -- and the mode switch (lora_merge over 32 layers)
  ceilings  what plain kernels reach on this machine in this run: a device copy, a dependency-free one-shot read of the
            size of the decode launch, an empty launch, a register-only MFMA loop and the shader clock it ran at

Other legs: --workload cfg3|cfg4|cfg4d|cfg5|cfg5mlp|merge7b, --path two-launches|fused|base (one workload only).
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
# HBM bytes per launch from rocprofv3 FETCH_SIZE / WRITE_SIZE runs, scaled by a 256 MiB copy; measured in a separate
# profiler run of this benchmark, not in this run (keyed by workload and kernel; the file holds the figures)
PROFILED_TRAFFIC = {("cfg2_decode", "delta_fused_small_kernel"): (45.80e6, "profiles/decode_cfg2_hbm_traffic.txt"),
                    ("cfg5_large_attn", "expand_stream_kernel"): (533.80e6, "profiles/prefill_cfg5_shrink_expand_hbm_traffic.txt"),
                    ("cfg5_large_attn", "shrink_stream_kernel"): (332.16e6, "profiles/prefill_cfg5_shrink_expand_hbm_traffic.txt"),
                    ("cfg4_mixed", "expand_stream_kernel"): (487.72e6, "profiles/prefill_cfg4_shrink_expand_hbm_traffic.txt")}

KERNEL_KEYS = {"shrink_tiled_kernel": "shrink", "expand_tiled_kernel": "expand", "delta_fused_small_kernel": "delta",
               "shrink_stream_kernel": "shrink", "expand_stream_kernel": "expand", "v_split_kernel": "v_split",
               "gemm_tiled_kernel": "gemm", "gemm_tiled_kernel<delta>": "gemm_delta",
               "gemm_ring_kernel": "gemm", "gemm_ring_kernel<delta>": "gemm_delta",
               "shrink_general_kernel": "shrink", "expand_general_kernel": "expand", "gemm_general_kernel": "gemm"}
WORKLOADS = ["cfg2", "cfg3", "cfg4", "cfg4d", "cfg5", "cfg5mlp"]


def load_workload(name, tables_only):
    from paper_2411_00915_amd import workloads as wl

    def make():
        if name in ("cfg5", "cfg5mlp"):
            return wl.cfg5("attn" if name == "cfg5" else "mlp", with_w=False)
        return wl.CONFIGS[name](with_w=False)
    if tables_only:
        with wl.tables_only():
            return make()
    return make()


def algorithmic_work(w, beta=1.0):
    """Bytes and flops the method itself must move / do per launch: every active adapter's factor once, x / y rows
    of active tokens once, v once (fp32)."""
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


def percentiles(ms):
    import numpy as np
    a = np.asarray(ms, dtype=np.float64)
    return dict(median=float(np.median(a)), p90=float(np.percentile(a, 90)), p95=float(np.percentile(a, 95)))


class LayerSets:
    """Distinct x / A / B / y (/ W) buffers per layer, resident on the device.  Layer 0 holds the seeded host draw
    when the workload has one; the others (all of them for table-only workloads) are drawn on the device with the
    same shapes and variances."""

    def __init__(self, w, L, need_w, torch, device, dev):
        self.w = w
        import numpy as np
        gen = torch.Generator(device=dev)
        gen.manual_seed(24110915)

        def randn_bf16(n, std):
            return (torch.randn(n, generator=gen, device=dev) * std).to(torch.bfloat16)

        a_off = np.concatenate([[0], np.cumsum([(int(r) * w.K + 7) // 8 * 8 for r in w.adapter_rank])])
        b_off = np.concatenate([[0], np.cumsum([(int(r) * w.N + 7) // 8 * 8 for r in w.adapter_rank])])
        layer0 = device.to_device(w, dev, with_w=False) if w.x is not None else None
        self.layers = []
        for l in range(L):
            if l == 0 and layer0 is not None:
                x, At_buf, Bt_buf, At_ptrs, Bt_ptrs = layer0.x, layer0.At_buf, layer0.Bt_buf, layer0.At_ptrs, layer0.Bt_ptrs
            else:
                x = randn_bf16(w.T * w.K, 1.0).view(w.T, w.K)
                if layer0 is not None:
                    offs_a, offs_b = layer0.At_off, layer0.Bt_off
                    At_buf, Bt_buf = torch.empty_like(layer0.At_buf), torch.empty_like(layer0.Bt_buf)
                else:
                    offs_a, offs_b = a_off[:-1], b_off[:-1]
                    At_buf = torch.empty(int(a_off[-1]) + 8, dtype=torch.bfloat16, device=dev)
                    Bt_buf = torch.empty(int(b_off[-1]) + 8, dtype=torch.bfloat16, device=dev)
                At_buf.copy_(randn_bf16(At_buf.numel(), w.K ** -0.5))
                Bt_buf.copy_(randn_bf16(Bt_buf.numel(), 0.18))            # (1 / sqrt(r) for the mean rank)
                At_ptrs = torch.tensor([At_buf.data_ptr() + int(o) * 2 for o in offs_a], dtype=torch.int64, device=dev)
                Bt_ptrs = torch.tensor([Bt_buf.data_ptr() + int(o) * 2 for o in offs_b], dtype=torch.int64, device=dev)
            y = randn_bf16(w.T * w.N, 1.0).view(w.T, w.N)
            Wt = randn_bf16(w.N * w.K, w.K ** -0.5).view(w.N, w.K) if need_w else None
            self.layers.append((x, At_ptrs, Bt_ptrs, y, Wt, At_buf, Bt_buf))


def measure(w, path, steps, warmup, layers_max, torch, B, device, dev, graph=True, merged_adapter=None):
    """One workload through one path: steps of (lora_plan + L layers), per-step event pairs, per-kernel timers."""
    import numpy as np
    need_w = path in ("fused", "base", "vendor-gemm")
    per_layer_bytes = 2 * (w.T * w.K + w.T * w.N + int(w.adapter_rank.sum()) * (w.K + w.N) + (w.K * w.N if need_w else 0))
    L = int(max(2, min(layers_max, 8e9 // max(per_layer_bytes, 1))))
    sets = LayerSets(w, L, need_w, torch, device, dev)
    abi_dtype = B.LORA_BF16
    make_plan = lambda: B.lora_plan(w.T, w.seg_indptr, w.seg_adapter, w.adapter_rank, w.adapter_scale, w.K, w.N, abi_dtype,
                                    merged_adapter=merged_adapter)
    plan0 = make_plan()
    _, v_bytes, ws_bytes = B.lora_plan_query(plan0)
    v = torch.zeros(max(v_bytes // 4, 64), dtype=torch.float32, device=dev)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)

    def run_layers(plan, stream):
        for (x, At_ptrs, Bt_ptrs, y, Wt, _a, _b) in sets.layers:
            if path == "delta":
                B.lora_delta(plan, x, w.K, At_ptrs, Bt_ptrs, v, y, w.N, 1.0, stream)
            elif path == "two-launches":
                B.lora_shrink(plan, x, w.K, At_ptrs, v, stream)
                B.lora_expand(plan, v, Bt_ptrs, y, w.N, 1.0, stream)
            elif path == "base":
                B.lora_base_gemm(w.T, w.K, w.N, abi_dtype, x, w.K, Wt, w.K, y, w.N, stream)
            elif path == "vendor-gemm":
                torch.matmul(x, Wt.t(), out=y)
            else:
                B.lora_fused_forward(plan, x, w.K, Wt, w.K, At_ptrs, Bt_ptrs, y, w.N, ws, ws.numel(), stream)

    stream = torch.cuda.current_stream()
    keep = []

    def step():
        plan = make_plan()
        B.lora_plan_upload(plan, stream)
        run_layers(plan, stream)
        keep.append(plan)          # destroyed after the work has finished

    def drain():
        torch.cuda.synchronize()
        for p in keep:
            p.destroy()
        keep.clear()

    for _ in range(warmup):
        step()
    drain()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    marks[0].record(stream)
    for i in range(steps):
        step()
        marks[i + 1].record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    drain()
    ms_per_step = (t1 - t0) * 1e3 / steps
    step_ms = [marks[i].elapsed_time(marks[i + 1]) for i in range(steps)]

    tp0 = time.perf_counter()
    for _ in range(20):
        make_plan().destroy()
    plan_us = (time.perf_counter() - tp0) * 1e6 / 20

    # per-kernel durations (event pair attached to every launch)
    B.lora_plan_upload(plan0, stream)
    torch.cuda.synchronize()
    B.lora_timing_begin()
    sweeps = max(2, min(steps, 10))
    for _ in range(sweeps):
        run_layers(plan0, stream)
    kern = B.lora_timing_end()
    # per layer: a kernel that runs more than once per layer (mixture mode: the removal's batch, then the tokens'
    # own) counts with all its launches
    for d in kern.values():
        d["avg_us"] = d["avg_us"] * d["count"] / (sweeps * L)

    graph_us = None
    if graph:
        try:                                       # the same sweep replayed from a HIP graph (no host launch cost)
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
            reps = max(5, min(steps, 50))
            tg0 = time.perf_counter()
            for _ in range(reps):
                g.replay()
            torch.cuda.synchronize()
            graph_us = (time.perf_counter() - tg0) * 1e6 / reps / L
        except Exception as exc:  # report, never hide
            print(f"bench.py: graph replay leg failed: {exc}", file=sys.stderr)

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
            prof = PROFILED_TRAFFIC.get((w.name, dom["kernel"]))
            roofline = dict(bound="hbm", kernel=dom["kernel"], achieved=round(dom["achieved_GBs"], 1), peak=HBM_PEAK_GBS,
                            unit="GB/s", frac=round(dom["achieved_GBs"] / HBM_PEAK_GBS, 4),
                            traffic=prof[0] if prof else None,
                            avg_kernel_us=round(dom["avg_us"], 3), algorithmic_bytes=dom["algorithmic_bytes"])
            if prof:
                roofline["traffic_source"] = prof[1] + " (rocprofv3 counters of a separate run of this benchmark; static, not measured in this run)"
    view = B.lora_plan_export(plan0)
    plan0.destroy()
    us_per_layer = ms_per_step * 1e3 / L
    if path == "vendor-gemm":                     # not this library's kernel: rate from the per-layer wall time
        tf = 2.0 * w.T * w.K * w.N / us_per_layer * 1e-6
        roofline = dict(bound="mfma", kernel="vendor library GEMM behind torch.matmul", achieved=round(tf, 1),
                        peak=MFMA_BF16_PEAK_TFLOPS, unit="TFLOP/s", frac=round(tf / MFMA_BF16_PEAK_TFLOPS, 4), traffic=None,
                        avg_kernel_us=None, algorithmic_flops=2 * w.T * w.K * w.N)
    pct = {k: round(val * 1e3 / L, 3) for k, val in percentiles(step_ms).items()}
    del sets
    return dict(w=w, L=L, ms_per_step=ms_per_step, us_per_layer=us_per_layer, step_us_per_layer=pct,
                kernels=ksum, roofline=roofline, graph_us_per_layer=graph_us, plan_host_us=plan_us,
                gpu_kernel_us_per_layer=sum(d["avg_us"] for d in ksum.values()) if ksum else None,
                tuning_source=view["tuning_source"])


def rnd(d):
    return {k: (round(x, 3) if isinstance(x, float) else x) for k, x in d.items() if x is not None}


def brief(m, path):
    """The entry of one (workload, path) in the `configs` object."""
    r = m["roofline"]
    out = {"us_per_layer": round(m["us_per_layer"], 2), **{k + "_us_per_layer": val for k, val in m["step_us_per_layer"].items()},
           "layers_per_step": m["L"], "gpu_kernel_us_per_layer": round(m["gpu_kernel_us_per_layer"], 2),
           "kernels": {k: {"kernel": d["kernel"], "avg_us": round(d["avg_us"], 2),
                           **({"algorithmic_bytes": d["algorithmic_bytes"], "GBs": round(d["achieved_GBs"], 1)} if d["algorithmic_bytes"] and not d["kernel"].startswith("gemm") else {}),
                           **({"algorithmic_flops": d["algorithmic_flops"], "TFLOPs": round(d["achieved_TFLOPs"], 1)} if d["algorithmic_flops"] and d["kernel"].startswith("gemm") else {})}
                       for k, d in m["kernels"].items()},
           "roofline": {"bound": r["bound"], "kernel": r["kernel"], "frac": r["frac"]} if r else None,
           "shape_table_entry": bool(m["tuning_source"] & 1)}
    return out


def measure_merge(steps, warmup, torch, B, dev):
    """Mode switch: one adapter (rank 64) merged into every one of 32 4096x4096 projections in one launch
    (lora_merge), alternating merge / unmerge; a step is one such launch."""
    L, N, K, r, s = 32, 4096, 4096, 64, 2.0
    gen = torch.Generator(device=dev)
    gen.manual_seed(24110915)
    rnd_ = lambda n, std: (torch.randn(n, generator=gen, device=dev) * std).to(torch.bfloat16)
    Wt = [rnd_(N * K, K ** -0.5).view(N, K) for _ in range(L)]
    At = [rnd_(r * K, K ** -0.5).view(r, K) for _ in range(L)]
    Bt = [rnd_(N * r, r ** -0.5).view(N, r) for _ in range(L)]
    ptrs = lambda ts: torch.tensor([t.data_ptr() for t in ts], dtype=torch.int64, device=dev)
    pW, pA, pB = ptrs(Wt), ptrs(At), ptrs(Bt)
    stream = torch.cuda.current_stream()
    sign = [1.0]

    def step():
        B.lora_merge(L, N, K, r, s * sign[0], B.LORA_BF16, pW, K, pA, pB, stream=stream)
        sign[0] = -sign[0]

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    marks[0].record(stream)
    for i in range(steps):
        step()
        marks[i + 1].record(stream)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
    step_ms = [marks[i].elapsed_time(marks[i + 1]) for i in range(steps)]
    B.lora_timing_begin()
    for _ in range(min(steps, 20)):
        step()
    torch.cuda.synchronize()
    kern = B.lora_timing_end()["merge_kernel"]
    by = L * (2 * N * K * 2 + (N + K) * r * 2)           # every weight read and written once, the factors read once
    return dict(ms_per_step=ms_per_step, step_ms=percentiles(step_ms), kernel_avg_us=kern["avg_us"], kernel_min_us=kern["min_us"],
                launches=kern["count"], algorithmic_bytes=by, algorithmic_flops=2 * L * N * K * r,
                GBs=by / kern["avg_us"] * 1e-3, config=dict(layers=L, n=N, k=K, rank=r))


def measure_heads(steps, torch, B, device, dev):
    """Task heads (section 4.2.2): 256 requests, one final feature each, 64 heads of different widths in one batch
    through lora_shrink (rank = outputs of the head, scale 1); rotating, cold head matrices."""
    import numpy as np
    from paper_2411_00915_amd import workloads as wl
    widths = (2, 5, 10, 101, 174, 256)
    with wl.tables_only():
        w = wl.random_case(4220, 256, 4096, 64, 64, widths, max_seg=1, scales=(1.0,), with_w=False)
    w.adapter_rank = np.asarray([widths[i % len(widths)] for i in range(64)], dtype=np.int32)
    plan = B.lora_plan(w.T, w.seg_indptr, w.seg_adapter, w.adapter_rank, w.adapter_scale, w.K, w.N, B.LORA_BF16)
    view = B.lora_plan_export(plan)
    _, v_bytes, _ = B.lora_plan_query(plan)
    gen = torch.Generator(device=dev)
    gen.manual_seed(4220)
    off = np.concatenate([[0], np.cumsum([(int(r) * w.K + 7) // 8 * 8 for r in w.adapter_rank])])
    L = 16
    sets = []
    for _ in range(L):
        Ht = (torch.randn(int(off[-1]) + 8, generator=gen, device=dev) * w.K ** -0.5).to(torch.bfloat16)
        ptrs = torch.tensor([Ht.data_ptr() + int(o) * 2 for o in off[:-1]], dtype=torch.int64, device=dev)
        x = torch.randn(w.T * w.K, generator=gen, device=dev).to(torch.bfloat16).view(w.T, w.K)
        sets.append((x, ptrs, Ht))
    v = torch.zeros(max(v_bytes // 4, 64), dtype=torch.float32, device=dev)
    B.lora_plan_upload(plan)
    for x, ptrs, _h in sets:
        B.lora_shrink(plan, x, w.K, ptrs, v)
    torch.cuda.synchronize()
    B.lora_timing_begin()
    for _ in range(max(2, min(steps, 10))):
        for x, ptrs, _h in sets:
            B.lora_shrink(plan, x, w.K, ptrs, v)
    kern = B.lora_timing_end()
    plan.destroy()
    (name, d), = kern.items()
    used = np.bincount(w.seg_adapter[w.seg_adapter >= 0], minlength=64) > 0
    by = 2 * (w.T * w.K + int(w.adapter_rank[used].sum()) * w.K) + 4 * int(w.adapter_rank[w.seg_adapter].sum())
    return {"requests": w.T, "k": w.K, "heads": 64, "widths": list(widths), "kernel": name,
            "shrink_kernel_family": "tiled" if view["shrink_kernel_family"] == B.LORA_VARIANT_TILED else "general",
            "kernel_avg_us": round(d["avg_us"], 2), "algorithmic_bytes": by, "GBs": round(by / d["avg_us"] * 1e-3, 1),
            "roofline": {"bound": "hbm", "kernel": name, "frac": round(by / d["avg_us"] * 1e-3 / HBM_PEAK_GBS, 4)}}


def measure_ceilings(torch, B, dev):
    """What plain kernels reach on this machine, now: a device copy, an empty launch, a dependency-free one-shot read
    of the decode launch's size (rotating buffers), a register-only MFMA loop and the clock it ran at."""
    out = {}
    n = 256 << 20
    src = torch.empty(3 * n, dtype=torch.uint8, device=dev).random_(0, 255)
    dst = torch.empty(n, dtype=torch.uint8, device=dev)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    for _ in range(2):
        dst.copy_(src[:n])
    ev[0].record()
    for i in range(9):
        dst.copy_(src[(i % 3) * n:(i % 3 + 1) * n])
    ev[1].record()
    torch.cuda.synchronize()
    out["device_copy_GBs"] = round(2 * n * 9 / (ev[0].elapsed_time(ev[1]) * 1e-3) * 1e-9, 1)        # read + write
    out["device_copy_note"] = "torch copy of 256 MiB, bytes read + bytes written per second"
    del dst
    for mb, tag in ((41.9, "read_42MB"), (16.8, "read_17MB"), (167.8, "read_168MB")):
        nbytes = int(mb * 1e6) // 32768 * 32768
        stride = (nbytes + 64 + 255) // 256 * 256
        bufs = min(16, (3 * n) // stride)                           # rotating buffers: nothing is served from cache
        for i in range(bufs):                                       # first touch untimed
            B.lora_probe(B.LORA_PROBE_READ, src.data_ptr() + i * stride, nbytes + 64)
        torch.cuda.synchronize()
        B.lora_timing_begin()
        for rep in range(3):
            for i in range(bufs):
                B.lora_probe(B.LORA_PROBE_READ, src.data_ptr() + i * stride, nbytes + 64)
        k = B.lora_timing_end()["probe_read_kernel"]
        out[tag] = dict(bytes=nbytes, avg_us=round(k["avg_us"], 2), min_us=round(k["min_us"], 2),
                        GBs=round(nbytes / k["avg_us"] * 1e-3, 1), frac_of_peak=round(nbytes / k["avg_us"] * 1e-3 / HBM_PEAK_GBS, 3))
    B.lora_timing_begin()
    for _ in range(20):
        B.lora_probe(B.LORA_PROBE_EMPTY, src, 64)
    out["empty_launch_us"] = round(B.lora_timing_end()["probe_empty_kernel"]["avg_us"], 2)
    iters = 2000
    scratch = torch.zeros(64, dtype=torch.int64, device=dev)
    B.lora_probe(B.LORA_PROBE_MFMA, scratch, 512, iters)
    torch.cuda.synchronize()
    B.lora_timing_begin()
    for _ in range(5):
        B.lora_probe(B.LORA_PROBE_MFMA, scratch, 512, iters)
    k = B.lora_timing_end()["probe_mfma_kernel"]
    flops = 2048 * 4 * iters * 16 * (2 * 16 * 16 * 32)
    ticks = scratch.cpu().numpy()
    out["mfma_register_loop_TFLOPs"] = round(flops / k["avg_us"] * 1e-6, 1)
    out["mfma_register_loop_frac_of_peak"] = round(flops / k["avg_us"] * 1e-6 / MFMA_BF16_PEAK_TFLOPS, 3)
    # shader-clock ticks over wall-clock ticks of one wavefront's loop, times the wall clock's rate
    out["shader_clock_MHz_under_mfma_load"] = round(float(ticks[0]) / max(float(ticks[1]), 1.0) * float(ticks[2]) * 1e-3, 0)
    out["vendor_peaks"] = {"hbm_GBs": HBM_PEAK_GBS, "mfma_bf16_TFLOPs": MFMA_BF16_PEAK_TFLOPS}
    return out


def oracle_leg(w, y0, cpu_seconds):
    """CPU oracle on this host's cores: the delta path (float64 shrink + expand-add) of layer 0, a bounded sample."""
    import numpy as np
    import oracle
    tok = oracle.token_adapter(w.T, w.seg_indptr, w.seg_adapter)
    ad = oracle.Adapters(w.adapter_rank, w.adapter_scale, w.A, w.B)
    n_rows = min(w.T, 512)                                   # bounded sample for the big configurations
    rows = None if n_rows == w.T else np.arange(0, w.T, w.T // n_rows)[:n_rows]
    sel = np.arange(w.T) if rows is None else rows
    y_in = y0.float().cpu().numpy().astype(np.float64)[sel]
    oracle.expand(w.x, tok, ad, w.N, y_in=y_in[:8], rows=sel[:8])       # warm the library
    tc0 = time.perf_counter()
    reps = 0
    while True:
        oracle.expand(w.x, tok, ad, w.N, y_in=y_in, rows=rows)
        reps += 1
        if time.perf_counter() - tc0 >= cpu_seconds or reps >= 1000:
            break
    cpu_us = (time.perf_counter() - tc0) * 1e6 / reps * (w.T / n_rows)
    return dict(value=round(cpu_us, 1), unit="us/layer", cores=oracle.num_threads(), kind="oracle",
                sample=(f"{n_rows} of {w.T} tokens of layer 0 of {w.name} (float64 shrink + expand-add), "
                        f"{reps} repetitions" + ("" if rows is None else ", scaled linearly to all tokens")))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--workload", default="cfg2", choices=WORKLOADS + ["merge7b"])
    ap.add_argument("--path", default="delta", choices=["delta", "two-launches", "fused", "base", "vendor-gemm"],
                    help="vendor-gemm: torch.matmul (the vendor library) on the operands of `base`, for comparison and for counter runs")
    ap.add_argument("--cpu-seconds", type=float, default=10.0, help="CPU time budget of the oracle leg (0 = skip)")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="skip the `configs` and `ceilings` objects")
    ap.add_argument("--no-shape-table", action="store_true", help="plan with the default tunables only (A/B of the shape table)")
    ap.add_argument("--configs-steps", type=int, default=100, help="timed steps of every entry of `configs`")
    ap.add_argument("--calib-copy-mb", type=int, default=0,
                    help="also run one plain device copy of this many MiB (a known-size reference for profiler counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is a single-GPU kernel path; it has no multi-GPU mode. "
              "Run with --gpus 1 (throughput of N replicas is N times this figure by construction).",
              file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2411_00915_amd import binding as B
    from paper_2411_00915_amd import device

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.no_shape_table:
        B.lora_tuning_table_set([dict(tokens=0, k=1, n=1, max_rank=8, group_class=0, tunables={})])     # matches no batch

    if args.workload == "merge7b":
        m = measure_merge(args.steps, args.warmup, torch, B, dev)
        print(json.dumps({
            "metric": "mode switch ms (one adapter merged into / removed from all layers, one launch)",
            "value": round(m["ms_per_step"], 4), "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": round(m["ms_per_step"], 4), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
            "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "merge7b", **m["config"], "launch": "eager, lora_merge per step, alternating +scale / -scale"},
            "roofline": {"bound": "hbm", "kernel": "merge_stream_kernel", "achieved": round(m["GBs"], 1),
                         "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(m["GBs"] / HBM_PEAK_GBS, 4),
                         "traffic": None, "avg_kernel_us": round(m["kernel_avg_us"], 3), "algorithmic_bytes": m["algorithmic_bytes"]},
            "cpu_baseline": None, "step_ms": rnd(m["step_ms"])}))
        return

    fused = args.path in ("fused", "base", "vendor-gemm")
    w = load_workload(args.workload, tables_only=False)
    head = measure(w, args.path, args.steps, args.warmup, args.layers, torch, B, device, dev, graph=not args.no_graph)

    if args.calib_copy_mb > 0:
        src = torch.empty(args.calib_copy_mb << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    cpu = None
    if args.cpu_seconds > 0 and args.path not in ("base", "vendor-gemm"):
        y0 = (torch.randn(w.T * w.N, device=dev)).to(torch.bfloat16).view(w.T, w.N)
        cpu = oracle_leg(w, y0, args.cpu_seconds)

    configs, ceilings = None, None
    if not args.no_configs and args.workload == "cfg2" and args.path == "delta":
        configs = {}
        for name in WORKLOADS[1:]:
            wt = load_workload(name, tables_only=True)
            entry = {"tokens": wt.T, "k": wt.K, "n": wt.N, "adapters": wt.num_adapters}
            res = {}
            for path in ("delta", "base", "fused"):
                res[path] = measure(wt, path, args.configs_steps, args.warmup, 8, torch, B, device, dev, graph=False)
                entry[{"delta": "lora_delta", "base": "lora_base_gemm", "fused": "lora_fused_forward"}[path]] = brief(res[path], path)
                torch.cuda.empty_cache()
            sep = res["base"]["gpu_kernel_us_per_layer"] + res["delta"]["gpu_kernel_us_per_layer"]
            entry["fusion_gain"] = round(sep / res["fused"]["gpu_kernel_us_per_layer"], 3)
            entry["fusion_gain_note"] = "(own base GEMM + lora_delta) / lora_fused_forward, GPU kernel time per layer"
            configs[wt.name] = entry
        # mixture mode (section 4.4.1) on the mixed batch: its most popular adapter stays merged in the weight
        wm = load_workload("cfg4", tables_only=True)
        import numpy as np
        seg_len = np.diff(wm.seg_indptr)
        popular = int(np.argmax(np.bincount(wm.seg_adapter[wm.seg_adapter >= 0], weights=seg_len[wm.seg_adapter >= 0], minlength=wm.num_adapters)))
        mix = {}
        for path in ("delta", "fused"):
            r = measure(wm, path, args.configs_steps, args.warmup, 8, torch, B, device, dev, graph=False, merged_adapter=popular)
            e = brief(r, path)
            e["roofline"] = None                     # (the byte and flop counts above are those of plain cfg4)
            for kd in e["kernels"].values():
                for key in ("algorithmic_bytes", "GBs", "algorithmic_flops", "TFLOPs"):
                    kd.pop(key, None)
            mix[{"delta": "lora_delta", "fused": "lora_fused_forward"}[path]] = e
            torch.cuda.empty_cache()
        mix["merged_adapter"] = popular
        mix["note"] = "cfg4 with its most popular adapter merged: every other token also takes that adapter's update off again"
        configs["cfg4_mixture"] = mix
        configs["task_heads"] = measure_heads(args.configs_steps, torch, B, device, dev)
        torch.cuda.empty_cache()
        m = measure_merge(args.configs_steps, args.warmup, torch, B, dev)
        configs["merge7b"] = {"ms_per_launch": round(m["ms_per_step"], 4), **{k + "_ms": round(val, 4) for k, val in m["step_ms"].items()},
                              "kernel_avg_us": round(m["kernel_avg_us"], 1), "algorithmic_bytes": m["algorithmic_bytes"],
                              "GBs": round(m["GBs"], 1), "roofline": {"bound": "hbm", "kernel": "merge_stream_kernel",
                                                                       "frac": round(m["GBs"] / HBM_PEAK_GBS, 4)}, **m["config"]}
        torch.cuda.empty_cache()
        ceilings = measure_ceilings(torch, B, dev)

    what = {"delta": "lora_delta per layer", "two-launches": "lora_shrink + lora_expand per layer",
            "fused": "lora_fused_forward per layer (shrink + base GEMM with delta epilogue)",
            "base": "lora_base_gemm per layer", "vendor-gemm": "torch.matmul per layer (vendor library, comparison only)"}[args.path]
    out = {
        "metric": ("LoRA-delta us/layer (shrink+expand, plan amortised over the layers of a step)" if not fused else
                   "fused layer us/layer (xW + delta, plan amortised over the layers of a step)"),
        "value": round(head["us_per_layer"], 3),
        "unit": "us/layer",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(head["ms_per_step"], 4),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": w.name, "tokens": w.T, "k": w.K, "n": w.N, "adapters": w.num_adapters,
                   "ranks": sorted(set(int(r) for r in w.adapter_rank)), "layers_per_step": head["L"],
                   "launch": "eager, one lora_plan per step, " + what,
                   "shape_table_entry": bool(head["tuning_source"] & 1)},
        "roofline": head["roofline"],
        "cpu_baseline": cpu,
        "step_us_per_layer": head["step_us_per_layer"],
        "kernels": {k: rnd(d) for k, d in head["kernels"].items()},
        "gpu_kernel_us_per_layer": round(head["gpu_kernel_us_per_layer"], 3) if head["kernels"] else None,
        "graph_replay_us_per_layer": round(head["graph_us_per_layer"], 3) if head["graph_us_per_layer"] else None,
        "plan_host_us": round(head["plan_host_us"], 2),
    }
    if configs is not None:
        out["configs"] = configs
        out["ceilings"] = ceilings
    print(json.dumps(out))


if __name__ == "__main__":
    main()
