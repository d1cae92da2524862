"""Where the time of lora_delta's single launch goes: per-workgroup phase time stamps of the instrumented build
(lora_trace_set) on the decode-shaped workload, summarised per phase.

    python -m paper_2411_00915_amd.decode_timeline [--layers 16] [--reps 4]

Operands rotate over `layers` sets, so every launch reads cold adapters as in the benchmark; the launches of the last
repetition are traced and summarised.  Times are microseconds after the earliest start stamp of the same launch.  The
instrumented build is a little slower than the ordinary one (stores of the stamps, two extra waits per workgroup);
the ordinary build's duration is printed next to it for comparison.
"""
import argparse
import sys

import numpy as np
import torch

from . import binding as B
from . import device, workloads as wl

SHRINK_PHASES = [(1, "descriptor, tokens, adapter pointer arrived"), (2, "v stores issued (first wavefront)"),
                 (3, "all v stores acknowledged"), (4, "group's count added")]
EXPAND_PHASES = [(1, "descriptor, tokens, adapter pointer arrived"), (2, "first Bt / y loads requested"),
                 (3, "group's count seen"), (4, "rows of v in LDS"), (5, "first wavefront's y stores acknowledged")]


def _line(name, us):
    us = us[np.isfinite(us)]
    if us.size == 0:
        return f"  {name:46s} (none)"
    q = np.percentile(us, [10, 50, 90])
    return f"  {name:46s} min {us.min():6.2f}  p10 {q[0]:6.2f}  median {q[1]:6.2f}  p90 {q[2]:6.2f}  max {us.max():6.2f}"


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--layers", type=int, default=16)
    ap.add_argument("--reps", type=int, default=4)
    args = ap.parse_args(argv)
    dev = "cuda:0"
    w = wl.cfg2(with_w=False)
    base = device.to_device(w, dev, with_w=False)
    gen = torch.Generator(device=dev)
    gen.manual_seed(1)

    def rnd(n, std):
        return (torch.randn(n, generator=gen, device=dev) * std).to(torch.bfloat16)

    layers = []
    for _ in range(args.layers):
        At_buf, Bt_buf = rnd(base.At_buf.numel(), w.K ** -0.5), rnd(base.Bt_buf.numel(), 0.2)
        At_ptrs = torch.tensor([At_buf.data_ptr() + int(o) * 2 for o in base.At_off], dtype=torch.int64, device=dev)
        Bt_ptrs = torch.tensor([Bt_buf.data_ptr() + int(o) * 2 for o in base.Bt_off], dtype=torch.int64, device=dev)
        layers.append((rnd(w.T * w.K, 1.0).view(w.T, w.K), At_ptrs, Bt_ptrs, rnd(w.T * w.N, 1.0).view(w.T, w.N), At_buf, Bt_buf))
    plan = device.make_plan(w)
    view = B.lora_plan_export(plan)
    if not (view["expand_tiles"][:, 5] >> 8).any():        # an expand tile carries its group's tile counts only then
        print("the plan does not use the single launch", file=sys.stderr)
        return 1
    S, E = view["shrink_tiles"].shape[0], view["expand_tiles"].shape[0]
    _, v_bytes, _ = B.lora_plan_query(plan)
    v = torch.zeros(v_bytes // 4, dtype=torch.float32, device=dev)
    B.lora_plan_upload(plan)
    tick_khz = B.lora_trace_tick_khz()
    if tick_khz <= 0:
        print("the device does not report the rate of its wall clock", file=sys.stderr)
        return 1

    def run(trace):
        for rep in range(args.reps):
            last = rep == args.reps - 1
            if last:
                B.lora_timing_begin()
            for l, (x, Ap, Bp, y, _a, _b) in enumerate(layers):
                if last and trace is not None:
                    B.lora_trace_set(trace[l])
                B.lora_delta(plan, x, w.K, Ap, Bp, v, y, w.N, 1.0)
        t = B.lora_timing_end()
        B.lora_trace_set(None)
        return next(iter(t.values()))["avg_us"]

    plain_us = run(None)
    trace = torch.zeros(args.layers, S + E, 8, dtype=torch.int64, device=dev)
    traced_us = run(trace)
    torch.cuda.synchronize()
    raw = trace.cpu().numpy()
    where = raw[:, :, 6]                                   # XCD << 32 | hardware id (CU 8..11, array 12, engine 13..15)
    cu = ((where >> 32) << 8) | ((where >> 8) & 0xff)
    t = raw.astype(np.float64)
    t[:, :, 6] = 0
    t[t == 0] = np.nan
    seen = np.nan_to_num(t[:, S:, 7], nan=0.0)
    t0 = np.nanmin(t[:, :, 0], axis=1)[:, None, None]
    us = (t - t0) * 1e3 / tick_khz
    print(f"cfg2 decode batch: {w.T} tokens, {w.num_adapters} adapters, {S} shrink + {E} expand workgroups, "
          f"{view['v_parts']} K part(s); {args.layers} launches summarised")
    print(f"kernel duration (event pair): ordinary build {plain_us:.2f} us, instrumented build {traced_us:.2f} us")
    print(f"expand tiles that saw their group's count: {int(seen.sum())} of {seen.size} (the others recomputed v)")
    print("microseconds after the launch's first start stamp")
    print("shrink workgroups")
    print(_line("start", us[:, :S, 0].ravel()))
    for k, name in SHRINK_PHASES:
        print(_line(name, us[:, :S, k].ravel()))
    print("expand workgroups")
    print(_line("start", us[:, S:, 0].ravel()))
    for k, name in EXPAND_PHASES:
        print(_line(name, us[:, S:, k].ravel()))
    print("per launch")
    last_pub = np.nanmax(us[:, :S, 4], axis=1)
    last_end = np.nanmax(us[:, S:, 5], axis=1)
    print(_line("last shrink count added", last_pub))
    print(_line("last y store acknowledged", last_end))
    print(_line("  ... minus last count added", last_end - last_pub))
    print("the expand workgroup whose y stores are acknowledged last, per launch")
    ex = us[:, S:, :]
    last = np.nanargmax(ex[:, :, 5], axis=1)
    rows = ex[np.arange(ex.shape[0]), last, :]
    print(_line("its start", rows[:, 0]))
    for k, name in EXPAND_PHASES:
        print(_line("its " + name, rows[:, k]))
    late = (ex[:, :, 0] > 2.0).sum(axis=1)
    first_late = [int(np.nonzero(ex[l, :, 0] > 2.0)[0].min()) + S if late[l] else -1 for l in range(ex.shape[0])]
    print(f"expand workgroups that start later than 2 us after the launch's first: median {int(np.median(late))} of {E}"
          f" (the launch has {S + E} workgroups; lowest index among them: {min(first_late)} .. {max(first_late)})")
    d12 = ex[:, :, 2] - ex[:, :, 1]
    print(_line("descriptor -> loads requested, on-time starters", d12[ex[:, :, 0] <= 2.0]))
    print(_line("descriptor -> loads requested, late starters", d12[ex[:, :, 0] > 2.0]))
    print("placement (last launch): workgroups per compute unit")
    for name, sel in (("shrink", cu[-1, :S]), ("expand", cu[-1, S:]), ("all", cu[-1])):
        ids, cnt = np.unique(sel, return_counts=True)
        hist = np.bincount(cnt)
        print(f"  {name:7s} on {ids.size} compute units; per unit: " + ", ".join(f"{n}: {c} units" for n, c in enumerate(hist) if c))
    xcd = np.bincount((where[-1] >> 32).astype(np.int64), minlength=8)
    print("  per XCD: " + " ".join(str(int(c)) for c in xcd) + f"; workgroup i ran on XCD i mod 8: {bool(((where[-1] >> 32) == np.arange(S + E) % 8).all())}")
    steps = [("start -> descriptor", us[:, S:, 1] - us[:, S:, 0]), ("count seen -> v in LDS", us[:, S:, 4] - us[:, S:, 3]),
             ("v in LDS -> y stores acknowledged", us[:, S:, 5] - us[:, S:, 4])]
    print("expand workgroups, differences")
    for name, d in steps:
        print(_line(name, d.ravel()))
    sh = [("start -> descriptor", us[:, :S, 1] - us[:, :S, 0]), ("descriptor -> v stores issued", us[:, :S, 2] - us[:, :S, 1]),
          ("v stores issued -> acknowledged", us[:, :S, 3] - us[:, :S, 2]), ("acknowledged -> count added", us[:, :S, 4] - us[:, :S, 3])]
    print("shrink workgroups, differences")
    for name, d in sh:
        print(_line(name, d.ravel()))
    plan.destroy()
    return 0


if __name__ == "__main__":
    sys.exit(main())
