"""Offline, profile-based search that fills the library's shape table on the GPU at hand.

The paper fills its shape -> tile-configuration hash table offline (section 4.3.2, Algorithm 2): loops over the
input shapes (token counts in steps of 32, the model's hidden sizes), over the LoRA ranks, and over the tile
configurations; every candidate is profiled and the fastest is stored under the shape's key.  This is that loop for
this library.  A shape class is (tokens with an adapter, K, N, rank class, group class) -- the key lora_plan_create
looks up -- and a candidate is a setting of the planner's tunables (tile sizes, K split, wavefronts per workgroup,
streaming-tile sizes, the head start of the shrink loads in the single decode launch).  Every candidate is timed with
the library's per-kernel timers on rotating layer buffers (nothing served from cache), through plans that carry the
candidate in their descriptor, so no process-wide state is involved.

    python -m paper_2411_00915_amd.autotune                      # search, print the report
    python -m paper_2411_00915_amd.autotune --write [FILE]       # ... and write csrc/tuning_table.inc (rebuild after)
    python -m paper_2411_00915_amd.autotune --quick              # a thinned search (for a look)

An entry is kept only where it beats the defaults by more than `--min-gain` (3 %), so the table stays small and
shapes without entry run on the defaults.
"""
from __future__ import annotations

import argparse
import itertools
import json
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
TABLE_INC = os.path.join(HERE, "csrc", "tuning_table.inc")

SHAPES = [(4096, 4096), (4096, 11008), (5120, 5120), (5120, 13824)]
# decode-shaped classes (every adapter group below 64 tokens): token counts in multiples of 32, as the paper's loop
DECODE_TOKENS = [32, 64, 96, 128, 160, 192, 224, 256, 320, 384, 448, 512, 640, 768, 896, 992]
DECODE_RANKS = [8, 16, 32, 64]
DECODE_GRID = {"shrink_target_wgs": [384, 768, 1152, 1536], "expand_wave_bytes": [4096, 8192, 16384, 32768],
               "fused_delay": [1, 3, 5, 8], "shrink_small_waves": [4, 8, 16], "shrink_small_jb": [1, 2]}
# prefill-sized classes (some adapter group of 64 tokens or more)
PREFILL_TOKENS = [1024, 2048, 4096, 8192, 16384]
PREFILL_RANKS = [16, 64, 128]
PREFILL_GRID = {"shrink_stream_wgs": [256, 512, 1024, 2048], "expand_stream_stages": [4, 8, 16, 32]}


class Case:
    """Segment table and rank table of a synthetic batch (the search needs no matrix values)."""

    def __init__(self, T, K, N, seg_indptr, seg_adapter, adapter_rank):
        self.T, self.K, self.N = T, K, N
        self.seg_indptr = np.asarray(seg_indptr, np.int32)
        self.seg_adapter = np.asarray(seg_adapter, np.int32)
        self.adapter_rank = np.asarray(adapter_rank, np.int32)
        self.adapter_scale = np.full(len(adapter_rank), 2.0, np.float32)
        self.num_adapters = len(adapter_rank)


def make_case(tokens, K, N, rank_class, group_class, seed):
    """A synthetic batch of the class: ranks drawn from the rank classes within a factor 8 below rank_class;
    decode-shaped = single-token requests over about tokens / 4 adapters; prefill-sized = requests of lognormal
    length (mean 64, sigma 1, as the mixed serving configuration) over about tokens / 64 adapters; long requests =
    requests of 1024 tokens, each with an adapter of its own of the class's rank (image-sized prefill)."""
    rng = np.random.default_rng(seed)
    ranks = [r for r in (8, 16, 32, 64, 128) if r <= rank_class and r * 8 >= rank_class]
    if group_class == 2:
        n_a = max(1, -(-tokens // 1024))
        lengths = np.asarray([min(1024, tokens - 1024 * i) for i in range(n_a)], np.int64)
        return Case(tokens, K, N, np.concatenate([[0], np.cumsum(lengths)]), np.arange(n_a), np.full(n_a, rank_class))
    if group_class == 0:
        lengths = np.ones(tokens, np.int64)
        n_a = max(2, tokens // 4)
    else:
        lengths = []
        while sum(lengths) < tokens:
            lengths.append(int(np.clip(np.rint(rng.lognormal(np.log(64) - 0.5, 1.0)), 1, 2048)))
        lengths[-1] -= sum(lengths) - tokens
        lengths = np.asarray([l for l in lengths if l > 0], np.int64)
        n_a = max(2, tokens // 64)
    seg_adapter = rng.integers(0, n_a, len(lengths))
    if group_class == 1:
        seg_adapter[int(np.argmax(lengths))] = 0
    adapter_rank = rng.choice(ranks, n_a)
    adapter_rank[0] = rank_class                                          # the class's top rank is in use
    seg_adapter[0] = 0
    return Case(tokens, K, N, np.concatenate([[0], np.cumsum(lengths)]), seg_adapter, adapter_rank)


def layers_for(per_layer_bytes):
    """Layer buffer sets of a class: enough that a sweep touches well over the 256 MB last-level cache several
    times (1.2 GB), so that every launch reads from HBM as it does inside a model."""
    return int(max(2, min(64, -(-1.2e9 // per_layer_bytes))))


class Bench:
    """Rotating layer buffers of one shape class and the timing of one candidate."""

    def __init__(self, w, layers, B, device, torch):
        self.w, self.B, self.device, self.torch = w, B, device, torch
        dev = "cuda:0"
        # the matrices are random bf16 of the right sizes: the search times kernels, it checks no values
        n_a = w.num_adapters
        a_off = np.concatenate([[0], np.cumsum([int(r) * w.K for r in w.adapter_rank])])
        b_off = np.concatenate([[0], np.cumsum([int(r) * w.N for r in w.adapter_rank])])
        self.layers = []
        for _ in range(layers):
            x = torch.randn(w.T, w.K, device=dev).to(torch.bfloat16)
            At = (torch.randn(int(a_off[-1]) + 64, device=dev) * w.K ** -0.5).to(torch.bfloat16)
            Bt = (torch.randn(int(b_off[-1]) + 64, device=dev) * 0.2).to(torch.bfloat16)
            Ap = torch.tensor([At.data_ptr() + int(o) * 2 for o in a_off[:n_a]], dtype=torch.int64, device=dev)
            Bp = torch.tensor([Bt.data_ptr() + int(o) * 2 for o in b_off[:n_a]], dtype=torch.int64, device=dev)
            y = torch.randn(w.T, w.N, device=dev).to(torch.bfloat16)
            self.layers.append((x, Ap, Bp, y, At, Bt))
        self.v = torch.zeros(4 * w.T * 256 + 64, dtype=torch.float32, device=dev)      # room for any K split

    def time(self, tuning, reps=3):
        reps = max(1, (reps * 8) // len(self.layers))      # (about reps x 8 timed launches whatever the number of layers)
        B, w = self.B, self.w
        plan = B.lora_plan(w.T, w.seg_indptr, w.seg_adapter, w.adapter_rank, w.adapter_scale, w.K, w.N, B.LORA_BF16,
                           tuning=tuning)
        for rep in range(2):                           # one untimed sweep, then the timed ones
            if rep == 1:
                B.lora_timing_begin()
            for _ in range(1 if rep == 0 else reps):
                for (x, Ap, Bp, y, _a, _b) in self.layers:
                    B.lora_delta(plan, x, w.K, Ap, Bp, self.v, y, w.N, 1.0)
            self.torch.cuda.synchronize()
        us = sum(d["avg_us"] for d in B.lora_timing_end().values())
        plan.destroy()
        return us


def search_classes(quick=False, group_classes=(0, 1, 2)):
    """The shape classes of the search: (tokens, K, N, rank class, group class)."""
    classes = []
    for (K, N) in (SHAPES[:1] if quick else SHAPES):
        if 0 in group_classes:
            for T in (DECODE_TOKENS[3:8:4] if quick else DECODE_TOKENS):
                for r in DECODE_RANKS:
                    classes.append((T, K, N, r, 0))
        for gc in (1, 2):
            if gc in group_classes:
                for T in (PREFILL_TOKENS[1:3] if quick else PREFILL_TOKENS):
                    for r in (PREFILL_RANKS[1:2] if quick else PREFILL_RANKS):
                        classes.append((T, K, N, r, gc))
    return classes


def read_table(path):
    """Rows of a tuning_table.inc: [(tokens, k, n, max_rank, group_class, [values])]."""
    import re
    rows = re.findall(r"^\{(\d+), (\d+), (\d+), (\d+), (\d+), \{([^}]*)\}\},", open(path).read(), flags=re.M)
    return [tuple(int(q) for q in row[:5]) + ([int(q) for q in row[5].split(",")],) for row in rows]


def write_table(path, entries, note, B, classes=()):
    """entries: the classes that keep tunables of their own.  Every other class of `classes` gets a row without
    values: the search found nothing better than the defaults for it, and without a row of its own a batch of that
    class would be planned with the entry of the next larger token count, which was tuned for another size."""
    have = {(e["tokens"], e["k"], e["n"], e["max_rank"], e["group_class"]) for e in entries}
    rows = list(entries) + [dict(tokens=c[0], k=c[1], n=c[2], max_rank=c[3], group_class=c[4], tunables={})
                            for c in classes if tuple(c) not in have]
    rows.sort(key=lambda e: (e["k"], e["n"], e["group_class"], e["max_rank"], e["tokens"]))
    with open(path, "w") as f:
        f.write("// Shape table shipped with the library: { tokens, k, n, max_rank, group_class, { tunables in the order of\n"
                "// lora_tuning_set; 0 = default } }; a row of zeros = the class was searched and keeps the defaults.\n"
                "// Written by `python -m paper_2411_00915_amd.autotune --write` on\n"
                f"// {note}\n")
        for e in rows:
            vals = ", ".join(str(int(e["tunables"].get(k, 0))) for k in B.TUNING_FIELDS)
            f.write(f"{{{e['tokens']}, {e['k']}, {e['n']}, {e['max_rank']}, {e['group_class']}, {{{vals}}}}},\n")
        if not rows:
            f.write("{0, 1, 1, 8, 0, {0}},   // (no class beat the defaults)\n")


def revalidate(args, torch, B, device):
    import re
    text = open(args.revalidate).read()
    note = " ".join(l[2:].strip() for l in text.split("\n")[3:] if l.startswith("//"))
    rows = re.findall(r"^\{(\d+), (\d+), (\d+), (\d+), (\d+), \{([^}]*)\}\},", text, flags=re.M)
    kept, lines = [], []
    t_start = time.time()
    for ci, row in enumerate(rows):
        T, K, N, r, gc = (int(q) for q in row[:5])
        if K == 1:
            continue
        vals = [int(q) for q in row[5].split(",")]
        tun = {k: val for k, val in zip(B.TUNING_FIELDS, vals) if val > 0}
        if not tun:
            continue                                                        # (a class that keeps the defaults)
        w = make_case(T, K, N, r, gc, seed=77000 + ci)                      # a fresh batch of the class
        per_layer = 2 * (w.T * w.K + w.T * w.N + sum(int(q) * (w.K + w.N) for q in w.adapter_rank))
        bench = Bench(w, layers_for(per_layer), B, device, torch)
        base = min(bench.time({}, reps=10), bench.time({}, reps=10))
        best = min(bench.time(tun, reps=10), bench.time(tun, reps=10))
        gain = base / best - 1.0
        lines.append(f"| {T} | {K} | {N} | {r} | {gc} | {base:.2f} | {best:.2f} | {100 * gain:+.1f} % | {'kept' if gain > args.min_gain else 'dropped'} |")
        print(lines[-1], flush=True)
        if gain > args.min_gain:
            kept.append(dict(tokens=T, k=K, n=N, max_rank=r, group_class=gc, tunables=tun))
        del bench
        torch.cuda.empty_cache()
    B.lora_tuning_table_set([])
    n_entries = len(lines)                                                  # (rows that carry values)
    print(f"{len(kept)} of {n_entries} entries kept ({time.time() - t_start:.0f} s)")
    if args.write:
        write_table(args.write, kept, note + f"  Re-timed on a second machine on fresh batches: {len(kept)} of {n_entries} entries kept "
                                             f"(gain over the defaults above {100 * args.min_gain:.0f} % both times).", B, search_classes())
    if args.summary:
        with open(args.summary, "a") as f:
            f.write(f"\nRevalidation on a second machine (fresh batches of each class, ten sweeps, twice): {len(kept)} of {n_entries} "
                    f"entries still beat the defaults by more than {100 * args.min_gain:.0f} % and are kept.\n")
    return 0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--quick", action="store_true", help="two token counts, one shape, thinned grids")
    ap.add_argument("--write", nargs="?", const=TABLE_INC, default=None, metavar="FILE",
                    help=f"write the table (default {TABLE_INC}; the library includes that file when it is built)")
    ap.add_argument("--min-gain", type=float, default=0.03)
    ap.add_argument("--group-class", type=int, action="append", default=None,
                    help="search these group classes only (0 decode-shaped, 1 mixed prefill, 2 long requests; repeatable)")
    ap.add_argument("--keep", default=None, metavar="FILE",
                    help="with --group-class: carry the rows of the other group classes over from this table")
    ap.add_argument("--report", default=None, help="also write the report (markdown) to this file")
    ap.add_argument("--summary", default=None, help="write a short summary of the report (markdown) to this file")
    ap.add_argument("--revalidate", default=None, metavar="FILE",
                    help="no search: time the entries of this table (a tuning_table.inc) against the defaults on fresh "
                         "batches of their classes and keep those that still win by --min-gain (run it on another "
                         "machine of the same model than the search: an entry must not be one machine's noise)")
    args = ap.parse_args()

    import torch
    from . import binding as B, device

    assert torch.cuda.is_available(), "the search profiles on the GPU"
    defaults = B.lora_tuning_get()
    # no table during the search: every plan = defaults + the candidate in its descriptor
    B.lora_tuning_table_set([dict(tokens=0, k=1, n=1, max_rank=8, group_class=0, tunables={})])
    if args.revalidate:
        return revalidate(args, torch, B, device)
    searched = tuple(args.group_class) if args.group_class else (0, 1, 2)
    classes = search_classes(args.quick, searched)
    lines, entries, n_candidates = [], [], 0
    t_start = time.time()
    for ci, (T, K, N, r, gc) in enumerate(classes):
        w = make_case(T, K, N, r, gc, seed=9000 + ci)
        per_layer = 2 * (w.T * w.K + w.T * w.N + sum(int(q) * (w.K + w.N) for q in w.adapter_rank))
        bench = Bench(w, layers_for(per_layer), B, device, torch)
        grid = DECODE_GRID if gc == 0 else PREFILL_GRID
        if args.quick:
            grid = {k: v[::2] for k, v in grid.items()}
        keys = list(grid)
        results = []
        for combo in itertools.product(*[grid[k] for k in keys]):
            cand = dict(zip(keys, combo))
            results.append((bench.time(cand), cand))
            n_candidates += 1
        results.sort(key=lambda q: q[0])
        # the three fastest and the defaults once more, with more sweeps: the pick must not be timing noise
        base_us = bench.time({}, reps=10)
        best_us, best = min(((bench.time(c, reps=10), c) for _, c in results[:3]), key=lambda q: q[0])
        gain = base_us / best_us - 1.0
        keep = {k: v for k, v in best.items() if v != defaults[k]} if gain > args.min_gain else {}
        lines.append(f"| {T} | {K} | {N} | {r} | {gc} | {base_us:.2f} | {best_us:.2f} | {100 * gain:+.1f} % | "
                     f"{json.dumps(keep) if keep else 'defaults'} |")
        print(lines[-1], flush=True)
        if keep:
            entries.append(dict(tokens=T, k=K, n=N, max_rank=r, group_class=gc, tunables=keep))
        del bench
        torch.cuda.empty_cache()
    elapsed = time.time() - t_start
    B.lora_tuning_table_set([])
    report = [f"# Tile search on {torch.cuda.get_device_name(0)} ({torch.cuda.get_device_properties(0).gcnArchName})", "",
              f"{len(classes)} shape classes x the candidate grids = {n_candidates} profiled candidates in {elapsed:.0f} s "
              f"(each: one plan carrying the candidate, one untimed sweep and about 24 timed launches over rotating layer buffers of 1.2 GB in all, "
              f"sum of the per-kernel timers; the three fastest of a class and the defaults are then timed again over about 80 launches).  {len(entries)} classes keep an entry (gain over the defaults above "
              f"{100 * args.min_gain:.0f} %).", "",
              "| tokens | K | N | rank class | group class | defaults us/layer | best us/layer | gain | entry |",
              "|---|---|---|---|---|---|---|---|---|"] + lines
    text = "\n".join(report) + "\n"
    if args.summary:
        rows = [l.split("|")[1:-1] for l in lines]
        agg = {}
        for q in rows:
            key = (int(q[1]), int(q[2]), int(q[4]))
            agg.setdefault(key, []).append(float(q[7].replace("%", "")))
        with open(args.summary, "w") as f:
            f.write("\n".join(report[:3]) + "\n\n| K | N | group class | classes | mean gain of the best candidate | largest | classes with an entry |\n|---|---|---|---|---|---|---|\n")
            for (K, N, gc), g in sorted(agg.items()):
                f.write(f"| {K} | {N} | {gc} | {len(g)} | {np.mean(g):+.1f} % | {max(g):+.1f} % | {sum(x > 100 * args.min_gain for x in g)} |\n")
            f.write("\nClasses of the benchmark configurations:\n\n" + "\n".join(report[4:6]) + "\n")
            for l in lines:
                q = [c.strip() for c in l.split("|")[1:-1]]
                if (q[0], q[1], q[2], q[3], q[4]) in {("256", "4096", "4096", "64", "0"), ("4096", "4096", "4096", "64", "1"),
                                                     ("8192", "4096", "11008", "128", "1"), ("16384", "5120", "5120", "128", "1"),
                                                     ("16384", "5120", "13824", "128", "1")}:
                    f.write(l + "\n")
    print(text)
    if args.report:
        with open(args.report, "w") as f:
            f.write(text)
    if args.write:
        carried = []
        if args.keep:
            for (T, K, N, r, gc, vals) in read_table(args.keep):
                if gc not in searched:
                    carried.append(dict(tokens=T, k=K, n=N, max_rank=r, group_class=gc,
                                        tunables={k: v for k, v in zip(B.TUNING_FIELDS, vals) if v > 0}))
        write_table(args.write, entries + [e for e in carried if e["tunables"]],
                    f"{torch.cuda.get_device_name(0)} ({torch.cuda.get_device_properties(0).gcnArchName}): "
                    f"{n_candidates} candidates over {len(classes)} shape classes"
                    + (f" (group classes {list(searched)}; the other rows carried over from an earlier search)" if args.keep else "") + ".",
                    B, classes + [(e["tokens"], e["k"], e["n"], e["max_rank"], e["group_class"]) for e in carried])
        print(f"wrote {args.write}: the library takes csrc/tuning_table.inc in when it is built")


if __name__ == "__main__":
    sys.exit(main())
