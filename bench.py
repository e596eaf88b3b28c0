#!/usr/bin/env python3
"""Benchmark of the dedup dispatch + combine hot path on one MI355X.

A step is one pass of the whole forward path over one batch of synthetic routing and
activations already resident in HBM:
    hm_plan -> hm_expert_load -> hm_dispatch_pack -> (identity experts) -> hm_combine
Default workload: the DeepSeek-V3-shaped layer (T=8192, H=7168, E=256, top-8 group-limited,
4 nodes x 8 ranks, node-level dedup).  Prints ONE JSON line on stdout; details go to stderr.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload dsv3] [--level node]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak
LEVELS = {"none": 0, "gpu": 1, "node": 2}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def measured_traffic(workload: str, level: str, kernel: str):
    """HBM bytes per launch from the committed rocprofv3 counter summaries (None if not measured)."""
    pdir = os.path.join(ROOT, "profiles")
    if not os.path.isdir(pdir):
        return None
    for name in sorted(os.listdir(pdir)):
        if not name.endswith(".txt"):
            continue
        for line in open(os.path.join(pdir, name)):
            f = line.split()
            if len(f) == 5 and f[0] == "traffic" and f[1:4] == [workload, level, kernel]:
                return int(f[4])
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="dsv3")
    ap.add_argument("--level", default=None, help="none|gpu|node (default: the workload's first level)")
    ap.add_argument("--sets", type=int, default=4, help="rotating buffer sets (cold HBM reads)")
    ap.add_argument("--warm-y", action="store_true",
                    help="combine reads the buffer dispatch wrote in the same step (partly cache-resident) instead of "
                         "an identical one written sets/2 steps earlier")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--with-transpose", action="store_true", help="also time hm_combine_transpose (stderr only)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch a plain 1 GiB device copy a few times (reference for rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (destinations are simulated index partitions; there are "
              "no collectives and no sharding) -- rerun with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2508_09591_amd import binding as B
    from paper_2508_09591_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU path", file=sys.stderr)
        return 2
    B.lib()
    torch.cuda.set_device(0)
    wl = W.WORKLOADS[args.workload]
    level = LEVELS[args.level] if args.level else wl.levels[0]
    level_name = W.LEVEL_NAMES[level]
    T, K, H, E = wl.T, wl.K, wl.H, wl.E

    # ---- inputs, resident in HBM before anything is timed ------------------------------------
    t0 = time.time()
    r = W.make_routing(wl)
    x = W.make_activations(wl)
    log("inputs generated in %.1f s" % (time.time() - t0))
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    ids_d, w_d, e2r_d = dev(r.topk_ids), dev(r.topk_weights), dev(r.expert_to_rank)
    x0 = dev(x.view(np.int16)).view(torch.bfloat16)

    stream = torch.cuda.Stream()          # default priority
    with torch.cuda.stream(stream):
        plan = B.hm_plan(ids_d, w_d, e2r_d, wl.nodes, wl.ranks_per_node, level)
        st, total_rows = B.hm_plan_status(plan)
    assert st == 0, B.status_string(st)
    c = total_rows / T
    nsets = max(1, args.sets)
    xs = [x0] + [x0.clone() for _ in range(nsets - 1)]
    packs = [torch.empty((total_rows, H), dtype=torch.bfloat16, device="cuda") for _ in range(nsets)]
    outs = [torch.empty((T, H), dtype=torch.bfloat16, device="cuda") for _ in range(nsets)]
    le = torch.empty(E, dtype=torch.int32, device="cuda")
    lr = torch.empty(wl.G, dtype=torch.int32, device="cuda")
    ln = torch.empty(wl.nodes, dtype=torch.int32, device="cuda")
    log("workload %s level %s: T=%d H=%d K=%d E=%d %dx%d ranks, rows=%d (c=%.3f), %d buffer sets = %.2f GB"
        % (wl.name, level_name, T, H, K, E, wl.nodes, wl.ranks_per_node, total_rows, c, nsets,
           nsets * (2 * T + total_rows) * H * 2 / 1e9))

    # Expert outputs arrive from the exchange, not from this GPU's caches: combine therefore reads
    # the pack buffer written sets/2 steps earlier.  With identity experts and identical X copies
    # it holds the same rows as the one dispatch has just written.
    y_shift = 0 if args.warm_y else nsets // 2
    with torch.cuda.stream(stream):
        for s in range(nsets):
            B.hm_dispatch_pack(xs[s], plan, packs[s], stream=stream)
    torch.cuda.synchronize()

    def step(i, ev=None):
        s = i % nsets
        ys = (s + y_shift) % nsets
        if ev: ev[0].record(stream)
        B.hm_plan(ids_d, w_d, e2r_d, wl.nodes, wl.ranks_per_node, level, plan=plan, stream=stream)
        if ev: ev[1].record(stream)
        B.hm_expert_load(ids_d, e2r_d, wl.nodes, wl.ranks_per_node, le, lr, ln, stream=stream)
        if ev: ev[2].record(stream)
        B.hm_dispatch_pack(xs[s], plan, packs[s], stream=stream)
        if ev: ev[3].record(stream)
        B.hm_combine(packs[ys], w_d, plan, outs[s], stream=stream)     # identity experts: Y = packed rows
        if ev: ev[4].record(stream)

    # ---- warm-up, then the timed region: exactly `steps` steps between two synchronisations ----
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_begin
    ms_per_step = elapsed * 1e3 / args.steps
    tokens_per_s = T / (elapsed / args.steps)

    # ---- per-kernel durations: the same steps again with HIP events on the launch stream ------
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(args.steps)]
    for i in range(args.steps):
        step(i, events[i])
    torch.cuda.synchronize()
    names = ["hm_plan", "hm_expert_load", "hm_dispatch_pack", "hm_combine"]
    avg_ms = {n: sum(e[j].elapsed_time(e[j + 1]) for e in events) / args.steps for j, n in enumerate(names)}
    min_ms = {n: min(e[j].elapsed_time(e[j + 1]) for e in events) for j, n in enumerate(names)}

    # correctness of what was timed: identity experts + weights summing to 1 -> output == input
    assert torch.equal(outs[(args.steps - 1) % nsets], xs[(args.steps - 1) % nsets]), "round trip failed"
    st, tr = B.hm_plan_status(plan, stream=stream)
    assert st == 0 and tr == total_rows

    row_bytes = 2 * H
    alg_bytes = {"hm_dispatch_pack": (1 + c) * T * row_bytes, "hm_combine": (c + 1) * T * row_bytes}
    kern = {}
    for n in ("hm_dispatch_pack", "hm_combine"):
        gbs = alg_bytes[n] / (avg_ms[n] * 1e-3) / 1e9
        kern[n] = {"avg_ms": round(avg_ms[n], 5), "min_ms": round(min_ms[n], 5), "alg_bytes": int(alg_bytes[n]),
                   "achieved_GBps": round(gbs, 1), "frac": round(gbs / HBM_PEAK_GBS, 4),
                   "traffic": measured_traffic(wl.name, level_name, n)}
    dominant = max(kern, key=lambda n: kern[n]["avg_ms"])
    pair_ms = avg_ms["hm_dispatch_pack"] + avg_ms["hm_combine"]
    pair_gbs = (alg_bytes["hm_dispatch_pack"] + alg_bytes["hm_combine"]) / (pair_ms * 1e-3) / 1e9
    log("per-call (HIP events, avg/min ms): " + ", ".join("%s %.4f/%.4f" % (n, avg_ms[n], min_ms[n]) for n in names))
    log("dispatch+combine: %.4f ms -> %.1f GB/s algorithmic = %.1f%% of %.0f GB/s; %.2f M tokens/s (pair only)"
        % (pair_ms, pair_gbs, 100 * pair_gbs / HBM_PEAK_GBS, HBM_PEAK_GBS, T / (pair_ms * 1e-3) / 1e6))

    if args.with_transpose:
        gout = torch.randn((T, H), dtype=torch.float32, device="cuda") * 1e-2
        gy = torch.empty((total_rows, H), dtype=torch.float32, device="cuda")
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
        with torch.cuda.stream(stream):
            for i in range(args.warmup):
                B.hm_combine_transpose(gout, plan, gy, stream=stream)
            for a, b in evs:
                a.record(stream)
                B.hm_combine_transpose(gout, plan, gy, stream=stream)
                b.record(stream)
        torch.cuda.synchronize()
        tms = sum(a.elapsed_time(b) for a, b in evs) / len(evs)
        tb = (1 + c) * T * 4 * H
        log("hm_combine_transpose: %.4f ms -> %.1f GB/s algorithmic (%.1f%% of peak)"
            % (tms, tb / (tms * 1e-3) / 1e9, 100 * tb / (tms * 1e-3) / 1e9 / HBM_PEAK_GBS))

    if args.calibrate_copy:
        src = torch.empty(1 << 29, dtype=torch.bfloat16, device="cuda").fill_(1.0)      # 1 GiB
        dst = torch.empty_like(src)
        with torch.cuda.stream(stream):
            for _ in range(5):
                dst.copy_(src)
        torch.cuda.synchronize()
        log("calibration: 5 plain copies of %d bytes launched" % (src.numel() * 2))
        del src, dst

    # ---- the oracle on this machine's host cores (reported baseline, not the target) ---------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        best = None
        reps = 0
        t_all = time.perf_counter()
        while reps < 3 and (time.perf_counter() - t_all) < 25:
            t1 = time.perf_counter()
            op = oracle.plan(r.topk_ids, r.topk_weights, r.expert_to_rank, wl.nodes, wl.ranks_per_node, level)
            oracle.expert_load(r.topk_ids, r.expert_to_rank, wl.nodes, wl.ranks_per_node)
            opk = oracle.dispatch_pack(x, op.row_token)
            oo = oracle.combine(opk, r.topk_weights, op.slot_row)
            dt = time.perf_counter() - t1
            best = dt if best is None else min(best, dt)
            reps += 1
        assert op.total_rows == total_rows
        cpu = {"value": round(T / best, 1), "unit": "tokens/s", "cores": 1, "kind": "oracle",
               "sample": "the whole %s batch (T=%d, level %s), same call sequence, best of %d passes, %.2f s per pass"
                         % (wl.name, T, level_name, reps, best)}
        log("cpu oracle: %.2f s per pass -> %.0f tokens/s on 1 core (%d cores visible)" % (best, T / best, os.cpu_count()))

    result = {
        "metric": "dedup dispatch+combine tokens/s (plan + expert_load + dispatch_pack + combine per step)",
        "value": round(tokens_per_s, 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "%s: T=%d H=%d E=%d top-%d, %d nodes x %d ranks, dedup level %s, identity experts"
                               % (wl.name, T, H, E, K, wl.nodes, wl.ranks_per_node, level_name),
                   "rows_per_token": round(c, 4), "buffer_sets": nsets,
                   "combine_input": "same-step buffer (warm)" if args.warm_y else "identical buffer written %d steps earlier (cold)" % y_shift},
        "roofline": {"bound": "hbm", "kernel": dominant, "achieved": kern[dominant]["achieved_GBps"],
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": kern[dominant]["frac"],
                     "traffic": measured_traffic(wl.name, level_name, dominant)},
        "cpu_baseline": cpu,
        "kernels": kern,
        "pair": {"ms": round(pair_ms, 5), "achieved_GBps": round(pair_gbs, 1), "frac": round(pair_gbs / HBM_PEAK_GBS, 4),
                 "tokens_per_s": round(T / (pair_ms * 1e-3), 1)},
        "plan_ms": round(avg_ms["hm_plan"], 5),
        "expert_load_ms": round(avg_ms["hm_expert_load"], 5),
    }
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
