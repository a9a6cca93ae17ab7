#!/usr/bin/env python3
"""Benchmark of the exact partition-and-placement search on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload headline] [--no-cpu-baseline]

A step is one pass of the whole hot path over one batch that is already resident in HBM:
tables (ppo_prepare), every ordering's full DP and the argmin (ppo_solve_range over [0, k!)),
and the traceback (ppo_finalize).  Prints one JSON line: node orderings evaluated per second,
the enumeration kernel's rate against the chip's vector-ALU peak, and the CPU oracle's rate on
a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# 256 compute units x 4 SIMDs x 16 lanes x 2.4 GHz: simple 32-bit vector operations per second
# (the 157.3 TFLOP/s fp32 vector figure counts an FMA as 2 and the packed form as 2 more).
VALU_PEAK_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12


def algorithmic_ops_per_ordering(w):
    """Mean over all k! orderings and all instances of the work the DP recurrence itself asks for:
    one min per (segment start i -> segment end e) candidate inside the memory window, and one max per
    row entry to form max(D[i], q[i-1]).  Rows 1..k-2 are counted over their whole range of segment
    ends; of the last row only D[L] is counted, because that is all the result depends on and all the
    kernel evaluates.  Row s uses node pi_s only through its window table, and every node sits at every
    position in (k-1)! orderings, so the mean is a sum over (row, node) pairs."""
    L, k = w.L, w.k
    cand = 0.0
    for n in range(w.n_inst):
        P = np.concatenate([[0.0], np.cumsum(w.m[n].astype(np.float64))])
        for j in range(k):
            cap = float(w.M[n, j])
            # lo[e] = first i with P[e] - P[i] <= cap
            lo = np.array([int(np.argmax(P[e] - P[: e + 1] <= cap)) for e in range(L + 1)])
            for s in range(1, k):
                e = np.arange(s + 1, L - (k - 1 - s) + 1) if s < k - 1 else np.array([L])
                cand += np.maximum(e - np.maximum(lo[e], s), 0).sum() / k
    cand /= w.n_inst
    maxops = (k - 1) * (L - k + 1)
    return cand, maxops


def run_sharing(w):
    """How much of that work the paired kernel's run sharing leaves: outputs of a DP row whose windows start at the
    same entry are prefix minima of one another, so a run of r outputs whose lowest window has w entries costs
    ceil((w - 1) / 2) three-input minima and r - 1 two-input ones instead of one chain per output.  Returns (outputs
    per run, vector instructions per output with one chain per output, with run sharing), means over rows 1..k-2,
    all nodes and up to 16 instances."""
    L, k = w.L, w.k
    outputs = runs = per_output = shared = 0
    for n in range(min(w.n_inst, 16)):
        P = np.concatenate([[0.0], np.cumsum(w.m[n].astype(np.float64))])
        for j in range(k):
            cap = float(w.M[n, j])
            lo = np.array([int(np.argmax(P[e] - P[: e + 1] <= cap)) for e in range(L + 1)])
            for s in range(1, k - 1):
                e = np.arange(s + 1, L - (k - 1 - s) + 1)
                start = np.maximum(lo[e], s)
                width = np.maximum(e - start, 0)
                base = np.ones(len(e), dtype=bool)          # lowest output of its run
                base[1:] = (start[1:] != start[:-1]) | (width[1:] == 0) | (width[:-1] == 0)
                outputs += len(e)
                runs += int(base.sum())
                per_output += int((width // 2).sum())       # ceil((w - 1) / 2) per output
                shared += int((width[base] // 2).sum()) + int((~base).sum())
    if outputs == 0:
        return None
    return outputs / runs, per_output / outputs, shared / outputs


def profiled(name, version):
    """Figures that only a profiler run can give (HBM traffic, share of the vector issue slots), read from the
    summary under profiles/ that `python -m paper_2210_12219_amd.profile_summary` wrote from rocprofv3 output, and
    only while that summary is of the library version that is running; otherwise {}."""
    from paper_2210_12219_amd.profile_summary import read_summary
    got = read_summary(os.path.join(ROOT, "profiles", name + ".md"))
    return got if got.get("ppo_version") == float(version) else {}


def copy_probe(torch):
    """One plain elementwise kernel of known traffic, for scaling the HBM counters of a rocprofv3 --pmc run."""
    src = torch.zeros(64 * 1024 * 1024, dtype=torch.float32, device="cuda:0")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    torch.add(src, 1.0, out=dst)   # one dispatch: 256 MiB read, 256 MiB written
    torch.cuda.synchronize()
    del src, dst


def bench_partition(args, torch, ppo, workloads):
    """Not the headline: the paper's partitioning step (least sum of transfer sizes), instances per second."""
    w = workloads.transformer_encoder()
    t, m, _, _ = ppo.to_device(w)
    kappa = torch.full((w.n_inst,), 0.2 * float(w.m[0].sum()), dtype=torch.float32, device="cuda:0")
    out = None
    for _ in range(args.warmup):
        out = ppo.ppo_min_sum_partition(t, m, kappa)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        out = ppo.ppo_min_sum_partition(t, m, kappa)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    print(json.dumps({
        "metric": f"chains partitioned/sec at L={w.L} (least sum of transfer sizes, the paper's Alg. 1)",
        "value": w.n_inst / (wall / args.steps), "unit": "instances/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": wall * 1e3 / args.steps, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.n_inst} chains of L={w.L}, capacity 0.2 of the model",
                   "segments_found": [int(x) for x in out[0].cpu().numpy()[:8]]},
        "roofline": None}), flush=True)


def bench_ct(args, torch, ppo, workloads):
    """Not the headline: the search with the compute-time term of the paper's Eq. 1 (ppo_solve_ct), whole solves."""
    w = getattr(workloads, args.workload)() if args.workload != "headline" else workloads.resnet50_shaped()
    work, speed = workloads.compute_terms(w, seconds=10.0)
    t, m, M, B = ppo.to_device(w)
    wd, vd = torch.from_numpy(work).cuda(), torch.from_numpy(speed).cuda()
    out = None
    for _ in range(args.warmup):
        out = ppo.ppo_solve_ct(t, m, wd, M, vd, B, out=out)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        out = ppo.ppo_solve_ct(t, m, wd, M, vd, B, out=out)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kf = math.factorial(w.k)
    print(json.dumps({
        "metric": f"node orderings evaluated/sec with the compute-time term at k={w.k},L={w.L}",
        "value": w.n_inst * kf / (wall / args.steps), "unit": "orderings/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": wall * 1e3 / args.steps, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.n_inst} instances x (L={w.L}, k={w.k}), {kf} orderings each, "
                               "work per layer log-uniform over a factor of 30, node speeds 1x/2x/4x, 10 s for the model",
                   "orderings_per_step": w.n_inst * kf},
        "roofline": None}), flush=True)


def bench_approx(args, torch, ppo, workloads):
    """Not the headline: the experiment of the paper's Sec. V with the true optimum in place of Theorem 1's bound:
    bottleneck latency of the paper's placement algorithm (and of its greedy comparison system) over the exact
    optimum of the same instance, on the paper-shaped clusters (Sec. IV)."""
    rows = []
    t_exact = t_heur = 0.0
    for n, caps in ((5, (32, 16)), (10, (32, 16)), (15, (32, 16)), (20, (32, 16)), (30, (64, 32)), (50, (64, 32))):
        for cap in caps:
            n_inst = 32 if n < 20 else 12
            w = workloads.cluster_geometric(n, cap, n_inst=n_inst, seed=500 + n)
            dev = ppo.to_device(w)
            kappa = torch.from_numpy(np.ascontiguousarray(w.M[:, 0])).cuda()
            torch.cuda.synchronize()
            c0 = time.perf_counter()
            heur, hsegs = ppo.ppo_place_kpath(dev[0], dev[1], kappa, dev[3], args.classes)[:2]
            joint = ppo.ppo_place_baseline(dev[0], dev[1], kappa, dev[3], ppo.PPO_BASELINE_JOINT)[0]
            torch.cuda.synchronize()
            c1 = time.perf_counter()
            if n <= ppo.PPO_CLUSTER_MAX_N:
                limit = None          # any number of segments
                exact = ppo.ppo_solve_cluster(*dev)[0]
            else:
                # beyond 20 nodes: the optimum over at most as many segments as the paper's partitioner made
                limit = int(hsegs.max().item())
                if not 1 <= limit <= ppo.PPO_CLUSTER_FEW_MAX_SEGMENTS:
                    continue
                exact = ppo.ppo_solve_cluster_few(*dev, max_segments=limit)[0]
            torch.cuda.synchronize()
            c2 = time.perf_counter()
            t_heur += c1 - c0
            t_exact += c2 - c1
            e, h, j = (x.cpu().numpy().astype(np.float64) for x in (exact, heur, joint))
            ok = np.isfinite(e) & np.isfinite(h) & (e > 0)
            okj = ok & np.isfinite(j)
            rows.append({"nodes": n, "capacity_mb": cap, "instances": int(ok.sum()), "exact_max_segments": limit,
                         "heuristic_over_exact": float(np.mean(h[ok] / e[ok])) if ok.any() else None,
                         "heuristic_optimal_share": float(np.mean(h[ok] == e[ok])) if ok.any() else None,
                         "joint_over_exact": float(np.mean(j[okj] / e[okj])) if okj.any() else None})
    ratios = [r["heuristic_over_exact"] for r in rows if r["heuristic_over_exact"] is not None]
    print(json.dumps({
        "metric": f"bottleneck latency of the paper's placement algorithm ({args.classes} classes) over the exact optimum, mean",
        "value": float(np.mean(ratios)), "unit": "ratio", "n_gpus": 1, "steps": 1, "warmup": 0,
        "ms_per_step": (t_exact + t_heur) * 1e3, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "cluster_geometric: 50-layer chain, n = 5..50 devices of 16 to 64 MB, Shannon-rate links",
                   "by_cluster": rows, "seconds_exact": t_exact, "seconds_heuristic_and_joint": t_heur},
        "roofline": None}), flush=True)


def bench_valu_probe(args, torch, ppo):
    """Not the headline: the measured issue rate of packed 16-bit vector instructions, 1 to 4 waves per SIMD."""
    iters = 25000
    rates = {}
    for wps in (1, 2, 3, 4):
        sink = ppo.ppo_probe_valu(wps, 1000)
        for _ in range(30):   # a few hundred milliseconds of the same work first, so that the clocks have settled
            ppo.ppo_probe_valu(wps, iters, sink)
        torch.cuda.synchronize()
        ms = []
        for _ in range(5):
            t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            t0.record()
            ppo.ppo_probe_valu(wps, iters, sink)
            t1.record()
            torch.cuda.synchronize()
            ms.append(t0.elapsed_time(t1))
        ns_per_instr = sorted(ms)[len(ms) // 2] * 1e6 / (64.0 * iters * wps)
        rates[wps] = {"ns_per_simd_instruction": ns_per_instr, "clocks_at_2.4GHz": ns_per_instr * 2.4,
                      "Tlane_op_per_s": 256 * 4 * 64 / ns_per_instr / 1e3}
    best = max(r["Tlane_op_per_s"] for r in rates.values())
    print(json.dumps({
        "metric": "measured issue rate of packed 16-bit vector instructions (eight independent accumulators per wave, 64 instructions per loop trip)",
        "value": best, "unit": "Tlane-op/s", "n_gpus": 1, "steps": 1, "warmup": 1, "ms_per_step": None,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u16", "data": "synthetic",
        "config": {"workload": "valu probe: 256 workgroups, 1..4 waves per SIMD", "by_waves_per_simd": rates},
        "roofline": {"bound": "alu", "achieved": best, "peak": VALU_PEAK_TOPS, "unit": "Tlane-op/s",
                     "frac": best / VALU_PEAK_TOPS, "traffic": None}}), flush=True)


def bench_cluster(args, torch, ppo, workloads):
    """Not the headline: whole exact solves per second of the cluster form (ppo_solve_cluster)."""
    N = args.cluster
    n_inst = args.cluster_instances or (64 if N <= 12 else 8 if N <= 16 else 1)
    pmax = args.max_segments or N
    w = workloads.cluster_mixed(N, L=100, n_inst=n_inst)
    dev = ppo.to_device(w)
    ws = torch.empty(ppo.ppo_cluster_workspace_bytes(w.L, N, n_inst), dtype=torch.uint8, device="cuda:0")
    out = None
    if args.copy_probe:
        copy_probe(torch)
    for _ in range(args.warmup):
        out = ppo.ppo_solve_cluster(*dev, max_segments=pmax, workspace=ws, out=out)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        out = ppo.ppo_solve_cluster(*dev, max_segments=pmax, workspace=ws, out=out)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    rows = sum(math.comb(N, r) * r for r in range(N - pmax + 1, N + 1))
    # every DP row (L 16-bit entries, rounded up to even) is written once and has to be read at least once
    row_bytes = 2 * ((w.L + 1) & ~1)
    alg_bytes = 2 * rows * row_bytes * n_inst
    achieved = alg_bytes / (wall / args.steps) / 1e9
    result = {
        "metric": f"clusters solved exactly/sec at n={N},L={w.L}, up to {pmax} segments (dynamic programming over sets of unused nodes)",
        "value": n_inst / (wall / args.steps), "unit": "instances/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": wall * 1e3 / args.steps, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u16", "data": "synthetic",
        "config": {"workload": f"{w.name}: {n_inst} instances x (L={w.L}, n={N}), seed={w.seed}",
                   "dp_rows_per_instance": rows, "segments_found": [int(x) for x in out[1].cpu().numpy()[:8]]},
        # against the whole call (tables, one launch per level, trace), not the level kernel alone
        "roofline": {"bound": "hbm", "kernel": "cluster_level_kernel (all levels) + tables + trace",
                     "achieved": achieved, "peak": 8000.0, "unit": "GB/s", "frac": achieved / 8000.0,
                     "traffic": profiled(f"cluster_solve_n{N}", ppo.load().ppo_version()).get("traffic_bytes_per_launch")
                     if (n_inst == 1 and pmax == N) else None,
                     "bytes_per_step": alg_bytes},
    }
    print(json.dumps(result), flush=True)


def bench_cluster_few(args, torch, ppo, workloads):
    """Not the headline: whole exact solves per second of the cluster form for large clusters and few segments
    (ppo_solve_cluster_few), on the paper's largest cluster shape by default (50 devices, 5 segments)."""
    N = args.cluster
    pmax = args.max_segments or 5
    n_inst = args.cluster_instances or 1
    # every node small enough that the chain needs the segments it is allowed
    w = workloads.cluster_mixed(N, L=100, n_inst=n_inst, capacity_factor=0.8 / pmax)
    dev = ppo.to_device(w)
    ws = torch.empty(ppo.ppo_cluster_few_workspace_bytes(w.L, N, pmax, n_inst), dtype=torch.uint8, device="cuda:0")
    out = None
    for _ in range(args.warmup):
        out = ppo.ppo_solve_cluster_few(*dev, max_segments=pmax, workspace=ws, out=out)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        out = ppo.ppo_solve_cluster_few(*dev, max_segments=pmax, workspace=ws, out=out)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    full = sum(math.comb(N, c) * c for c in range(1, max(pmax, 2)))
    top = math.comb(N, pmax) * pmax if pmax > 1 else 0
    # every full row (L binary32 entries, rounded up to even) is written once and read once by the level above,
    # every entry of the last level is written once; the passes that rebuild the answer read them again
    row_bytes = 4 * ((w.L + 1) & ~1)
    alg_bytes = (2 * full * row_bytes + 4 * top) * n_inst
    achieved = alg_bytes / (wall / args.steps) / 1e9
    print(json.dumps({
        "metric": f"clusters solved exactly/sec at n={N},L={w.L}, up to {pmax} segments (dynamic programming over sets of nodes still to be used)",
        "value": n_inst / (wall / args.steps), "unit": "instances/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": wall * 1e3 / args.steps, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: {n_inst} instances x (L={w.L}, n={N}), capacities for {pmax} segments, seed={w.seed}",
                   "dp_rows_per_instance": full + top, "segments_found": [int(x) for x in out[1].cpu().numpy()[:8]]},
        "roofline": {"bound": "hbm", "kernel": "few_level_kernel (all levels) + tables + answer passes",
                     "achieved": achieved, "peak": 8000.0, "unit": "GB/s", "frac": achieved / 8000.0, "traffic": None,
                     "bytes_per_step": alg_bytes}}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="headline")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--bounded", action="store_true",
                    help="time ppo_solve_range_bounded (prefix rows shared, groups skipped) instead of the full "
                         "enumeration: a separate figure, not the headline's unit of work")
    ap.add_argument("--subsets", action="store_true",
                    help="time ppo_solve_subsets (dynamic programming over node subsets) instead of the "
                         "enumeration: a separate figure in instances per second")
    ap.add_argument("--cluster", type=int, default=0, metavar="N",
                    help="time ppo_solve_cluster on clusters of N nodes (hosting nodes and number of segments "
                         "free; L=100, mixed capacities): a separate figure in instances per second; N > 20: "
                         "ppo_solve_cluster_few with --max-segments (default 5)")
    ap.add_argument("--cluster-instances", type=int, default=0, help="instances per step with --cluster")
    ap.add_argument("--max-segments", type=int, default=0, help="with --cluster: most segments allowed (default N; 5 beyond 20 nodes)")
    ap.add_argument("--partition", action="store_true",
                    help="time ppo_min_sum_partition (the paper's own partitioning step) on 4096 chains of L=96: "
                         "a separate figure in instances per second")
    ap.add_argument("--ct", action="store_true",
                    help="time ppo_solve_ct (the search with the compute-time term of Eq. 1) on --workload "
                         "(default resnet50_shaped): a separate figure")
    ap.add_argument("--approx", action="store_true",
                    help="the paper's placement algorithm against the exact optimum on paper-shaped clusters "
                         "(ppo_place_kpath / ppo_place_baseline / ppo_solve_cluster): mean ratio of bottleneck latencies")
    ap.add_argument("--classes", type=int, default=5, help="with --approx: number of transfer-size classes")
    ap.add_argument("--valu-probe", action="store_true",
                    help="measure the issue rate of packed 16-bit vector instructions (ppo_probe_valu): the measured "
                         "peak to set beside the nominal one")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also launch one plain elementwise kernel that reads and writes 256 MiB: the known "
                         "traffic the HBM counters of a rocprofv3 --pmc run are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU; --gpus N with N > 1 is not supported "
                 "(rank ranges and instances are independent, so the search shards trivially, but no multi-GPU path is built)")

    import torch
    from paper_2210_12219_amd import binding as ppo
    from paper_2210_12219_amd import workloads

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    ppo.load()
    if args.cluster > ppo.PPO_CLUSTER_MAX_N:
        return bench_cluster_few(args, torch, ppo, workloads)
    if args.cluster:
        return bench_cluster(args, torch, ppo, workloads)
    if args.partition:
        return bench_partition(args, torch, ppo, workloads)
    if args.ct:
        return bench_ct(args, torch, ppo, workloads)
    if args.approx:
        return bench_approx(args, torch, ppo, workloads)
    if args.valu_probe:
        return bench_valu_probe(args, torch, ppo)
    w = workloads.WORKLOADS[args.workload]()
    L, k, n = w.L, w.k, w.n_inst
    kf = math.factorial(k)
    dev = ppo.to_device(w)
    ws = ppo.alloc_workspace(L, k, n)
    keys = torch.empty(n, dtype=torch.int64, device="cuda:0")
    out = ppo.alloc_outputs(n, k)
    stream = torch.cuda.current_stream()
    skipped = torch.zeros(n, dtype=torch.int64, device="cuda:0")

    def step(events=None):
        if events:
            events[0].record(stream)
        ppo.ppo_prepare(*dev, ws)
        ppo.ppo_init_keys(keys)
        if events:
            events[1].record(stream)
        if args.subsets:
            ppo.ppo_solve_subsets(L, k, n, ws, keys)
        elif args.bounded:
            ppo.ppo_solve_range_bounded(L, k, n, ws, 0, kf, keys, skipped)
        else:
            ppo.ppo_solve_range(L, k, n, ws, 0, kf, keys)
        if events:
            events[2].record(stream)
        ppo.ppo_finalize(L, k, n, ws, keys, out=out)
        if events:
            events[3].record(stream)

    if args.copy_probe:
        copy_probe(torch)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(evs[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    enum_ms = float(np.mean([e[1].elapsed_time(e[2]) for e in evs]))
    prep_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in evs]))
    fin_ms = float(np.mean([e[2].elapsed_time(e[3]) for e in evs]))
    value = n * kf / (wall / args.steps)

    cand, maxops = algorithmic_ops_per_ordering(w)
    ops_per_launch = (cand + maxops) * n * kf
    achieved = ops_per_launch / (enum_ms * 1e-3) / 1e12

    prof = profiled(f"enumerate_paired_{args.workload}", ppo.load().ppo_version())
    result = {
        "metric": "node orderings (full DPs) evaluated/sec at k=10,L=100; % of VALU peak",
        "value": value, "unit": "orderings/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u16", "data": "synthetic",
        "config": {"workload": f"{w.name}: {n} instances x (L={L}, k={k}), {kf} orderings each, seed={w.seed}",
                   "orderings_per_step": n * kf},
        "candidates_per_s": value * cand,
        "stage_ms": {"prepare": prep_ms, "enumerate": enum_ms, "finalize": fin_ms},
        # achieved: the min and max operations the DP recurrence asks for (counted from the inputs, not from the
        # kernel) per second of the enumeration kernel; peak: 32-bit lane operations of the vector ALUs.  The kernel
        # works on packed 16-bit halves, whose peak is twice that (frac_packed16); valu_issue is the share of the
        # vector issue slots the kernel filled according to the hardware counters (from the committed profile of
        # this library version, else null), as is traffic.
        "roofline": {"bound": "alu", "kernel": "enumerate", "achieved": achieved, "peak": VALU_PEAK_TOPS,
                     "unit": "Tlane-op/s", "frac": achieved / VALU_PEAK_TOPS,
                     "frac_packed16": achieved / (2.0 * VALU_PEAK_TOPS),
                     "valu_issue": prof.get("valu_issue"),
                     "traffic": prof.get("traffic_bytes_per_launch"),
                     "min_ops_per_ordering": cand, "max_ops_per_ordering": maxops,
                     "run_sharing": dict(zip(("outputs_per_run", "vector_instructions_per_output_unshared",
                                              "vector_instructions_per_output"), run_sharing(w) or (None,) * 3)),
                     "kernel_ms": enum_ms},
    }

    if args.subsets:
        # not the headline: whole exact solves per second by the subset DP (no ordering is enumerated)
        result["metric"] = f"instances solved exactly/sec at k={k},L={L} (dynamic programming over node subsets)"
        result["value"] = n / (wall / args.steps)
        result["unit"] = "instances/s"
        result["roofline"] = None
        print(json.dumps(result), flush=True)
        return
    if args.bounded:
        # not the headline: orderings disposed of (evaluated with shared prefix rows, or skipped under the bound)
        runs = args.steps + args.warmup
        frac = float(skipped.sum().item()) * 360.0 / (n * kf * runs)
        result["metric"] = "node orderings disposed of/sec at k=10,L=100 (prefix rows shared, groups skipped under the bound)"
        result["skipped_fraction"] = frac
        result["roofline"] = None
        print(json.dumps(result), flush=True)
        return

    if not args.no_cpu_baseline:
        from oracle import ppo_oracle
        threads = ppo_oracle.default_threads()
        n_s = min(n, 16)
        span = min(kf, 1600000 * threads // n_s + 1)   # about 15 s of the oracle on every host thread
        s = w.take(n_s)
        ppo_oracle.lib()
        c0 = time.perf_counter()
        ppo_oracle.exhaustive(s.t, s.m, s.M, s.B, n_threads=threads, rank_range=(0, span))
        dt = time.perf_counter() - c0
        # the same oracle on one thread, on a fixed sample: the first million ranks of the first instance
        one = w.take(1)
        span1 = min(kf, 1000000)
        c1 = time.perf_counter()
        ppo_oracle.exhaustive(one.t, one.m, one.M, one.B, n_threads=1, rank_range=(0, span1))
        dt1 = time.perf_counter() - c1
        result["cpu_baseline"] = {"value": n_s * span / dt, "unit": "orderings/s", "cores": threads, "kind": "oracle",
                                  "sample": f"ranks [0,{span}) of the first {n_s} instances of {w.name}, "
                                            f"{dt:.1f} s on {threads} threads",
                                  "one_thread": {"value": span1 / dt1, "unit": "orderings/s",
                                                 "sample": f"ranks [0,{span1}) of instance 0, {dt1:.1f} s"}}
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
