"""Profile-based search of the planner's tunables on the GPU at hand.

The paper fills its shape -> tile-configuration table by profiling every
candidate offline (section 4.3.2, Algorithm 2: loop over input shapes, ranks
and tile configurations, profile, keep the best).  This is the same loop for
this library: for a workload shape it sweeps a grid of planner tunables, times
the delta path with the library's per-kernel timers on rotating buffers, and
prints the best setting with a `lora_tuning_set(...)` line for it; `--out FILE` also stores it in a
shape-keyed table (tuning_table.py) that `apply_for_shape` consults before planning.

    python -m paper_2411_00915_amd.autotune --workload cfg2
    python -m paper_2411_00915_amd.autotune --workload cfg3 --grid '{"expand_wave_bytes_big": [65536, 131072]}'
"""
from __future__ import annotations

import argparse
import itertools
import json

DEFAULT_GRIDS = {
    "decode": {"shrink_target_wgs": [256, 512, 768], "expand_wave_bytes": [8192, 16384, 32768], "fused_delay": [1, 3, 5]},
    "prefill": {"shrink_stream_wgs": [1, 512, 2048], "expand_stream_stages": [8, 16, 32]},
}


def measure(w, layers, v, B, path="delta", reps=3):
    """Mean GPU microseconds per layer of the delta path under the current tunables."""
    # (v is sized for four K parts, the most a plan can ask for)
    import torch
    from . import device
    plan = device.make_plan(w)
    total = 0.0
    for rep in range(2):
        if rep == 1:
            B.lora_timing_begin()
        for _ in range(reps):
            for (x, Ap, Bp, y) in layers:
                B.lora_delta(plan, x, w.K, Ap, Bp, v, y, w.N, 1.0)
        torch.cuda.synchronize()
    for d in B.lora_timing_end().values():
        total += d["avg_us"]
    plan.destroy()
    return total


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="cfg2", choices=["cfg2", "cfg3", "cfg4", "cfg4d", "cfg5"])
    ap.add_argument("--layers", type=int, default=8)
    ap.add_argument("--grid", default=None, help="JSON object: tunable name -> list of values")
    ap.add_argument("--out", default=None, help="shape-keyed table (JSON) to store the best setting in")
    args = ap.parse_args()

    import torch
    from . import binding as B, device, workloads as wl

    w = wl.cfg5("attn", with_w=False) if args.workload == "cfg5" else wl.CONFIGS[args.workload](with_w=False)
    grid = json.loads(args.grid) if args.grid else DEFAULT_GRIDS["decode" if w.T <= 1024 else "prefill"]
    dev = "cuda:0"
    l0 = device.to_device(w, dev, with_w=False)
    layers = []
    for _ in range(args.layers):
        x = torch.randn(w.T, w.K, device=dev).to(torch.bfloat16)
        At = (torch.randn(l0.At_buf.numel(), device=dev) * w.K ** -0.5).to(torch.bfloat16)
        Bt = (torch.randn(l0.Bt_buf.numel(), device=dev) * 0.2).to(torch.bfloat16)
        Ap = torch.tensor([At.data_ptr() + int(o) * 2 for o in l0.At_off], dtype=torch.int64, device=dev)
        Bp = torch.tensor([Bt.data_ptr() + int(o) * 2 for o in l0.Bt_off], dtype=torch.int64, device=dev)
        y = torch.randn(w.T, w.N, device=dev).to(torch.bfloat16)
        layers.append((x, Ap, Bp, y, At, Bt))
    layers_call = [(x, Ap, Bp, y) for (x, Ap, Bp, y, _a, _b) in layers]
    base = B.lora_tuning_get()
    big = max(B.lora_plan_query(device.make_plan(w))[1] for _ in range(1))
    v = torch.zeros(4 * big // 4 + 64, dtype=torch.float32, device=dev)      # room for up to 4 parts of v
    keys = list(grid)
    results = []
    try:
        for combo in itertools.product(*[grid[k] for k in keys]):
            B.lora_tuning_set(**base)
            B.lora_tuning_set(**dict(zip(keys, combo)))
            us = measure(w, layers_call, v, B)
            results.append((us, dict(zip(keys, combo))))
            print(f"{us:9.2f} us/layer  {dict(zip(keys, combo))}", flush=True)
    finally:
        B.lora_tuning_set(**base)
    results.sort(key=lambda r: r[0])
    best_us, best = results[0]
    base_us = [u for u, c in results if all(base[k] == c[k] for k in keys)]
    print(json.dumps({"workload": w.name, "best_us_per_layer": round(best_us, 2), "best": best,
                      "defaults_us_per_layer": round(base_us[0], 2) if base_us else None,
                      "apply": "lora_tuning_set(" + ", ".join(f"{k}={val}" for k, val in best.items()) + ")"}))
    if args.out:
        from . import tuning_table
        key = tuning_table.shape_key(w.T, w.K, w.N, int(w.adapter_rank.max()))
        tuning_table.store(key, best, args.out)
        print(f"stored under {key} in {args.out}")


if __name__ == "__main__":
    main()
