#!/usr/bin/env python3
"""Benchmark of the sampling-verification hot path on one MI355X.

A step = one pass of the whole path over one batch of synthetic token trees:
spechub_draft (pair sampling for every internal node), spechub_verify (every
node) and the tree walk, which the verify kernel runs itself at this batch size
(two launches per step; a third launch for large batches, see --separate-walk).  Inputs are resident in HBM; the step rotates over
several distinct copies of the batch so that the working set exceeds the
256 MiB Infinity Cache and "HBM GB/s" is not cache bandwidth.

Prints ONE JSON line (see the keys below).  --gpus above 1 is refused: this
build runs on one GPU.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published peak
METRIC = "verified tree nodes/sec and HBM GB/s (% peak) at V=32000, 31-node tree"
KERNEL_REPS = 200
SETTLE_S = 0.1       # launches in each differential event bracket, whatever --steps is


def metric_name(wl):
    """The headline metric's name; for another workload than the headline's, the same metric
    with that workload's vocabulary and tree size."""
    if wl.V == 32000 and wl.N == 31:
        return METRIC
    return "verified tree nodes/sec and HBM GB/s (%% peak) at V=%d, %d-node tree" % (wl.V, wl.N)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--config", default="3",
                    help="workload configuration 1..5 (3 = the metric's), or `toy`: the toy experiment of "
                         "App. D as a batch (V = 50, T = 0.25, lambda = 0.7; 200 (p, q) pairs x 512 repeats, "
                         "one draft step each), reported in pairs/s")
    ap.add_argument("--method", default="spechub", choices=["spechub", "rrs", "rrsw"])
    ap.add_argument("--batch", type=int, default=0, help="trees per batch (0 = the configuration's own)")
    ap.add_argument("--copies", type=int, default=0, help="distinct input copies to rotate over (0 = auto)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-stats", action="store_true",
                    help="spechub_verify recomputes the draft row's hub and normalisers instead of "
                         "taking them from spechub_draft")
    ap.add_argument("--separate-walk", action="store_true",
                    help="three launches per step (draft, verify, walk) whatever the batch size")
    ap.add_argument("--walk-in-verify", action="store_true",
                    help="two launches per step whatever the batch size: the verify kernel walks each tree "
                         "itself when the tree's last node is done (the default up to "
                         "binding.WALK_IN_VERIFY_MAX_NODES tree nodes per batch, three launches beyond)")
    ap.add_argument("--graph", action="store_true",
                    help="replay one HIP graph per step instead of launching its kernels one by one "
                         "(measured slower on this workload: 58.8 against 53.8 us per step)")
    ap.add_argument("--no-path-only", action="store_true",
                    help="skip the extra measurement of the path-only step (draft + *_verify_path)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a plain 512 MiB device copy three times (reference dispatch for "
                         "scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    return ap.parse_args()


def read_traffic(kernel_key: str):
    """HBM bytes per launch measured OFFLINE with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE) in runs
    of this same command, kept as a small text summary under profiles/ (a counter run cannot be
    made from inside the timed process); None when no summary exists for this kernel and workload."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        f = line.split()
        if len(f) >= 2 and f[0] == kernel_key:
            return float(f[1])
    return None


def cpu_baseline(wl_cpu_rows, k, depth, temps, method_id, repeats, threads):
    """The fp64 oracle, as it stands, on a bounded sample of the same workload."""
    import numpy as np
    import oracle
    t_np, d_np = wl_cpu_rows
    B, N, V = t_np.shape
    u_d = oracle.philox_uniform(1, 1, B * N, k).reshape(B, N, k)
    u_v = oracle.philox_uniform(1, 2, B * N, k + 1).reshape(B, N, k + 1)
    kw = dict(dtype=oracle.BF16 if t_np.dtype == np.uint16 else oracle.FP32, kind=oracle.LOGITS, k=k,
              depth=depth, nthreads=threads)
    t0 = time.perf_counter()
    for _ in range(repeats):
        od = oracle.batch_draft(method_id, d_np, u_d, temp_draft=temps[1], **kw)
        oracle.batch_verify(method_id, t_np, d_np, od["tokens"], u_v, temp_target=temps[0],
                            temp_draft=temps[1], **kw)
    dt = time.perf_counter() - t0
    return B * N * repeats / dt, dt


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2411_05289_amd import binding as B
    from paper_2411_05289_amd import workloads as W
    if not torch.cuda.is_available():
        print("bench.py needs the GPU: there is no CPU path", file=sys.stderr)
        sys.exit(3)
    B.lib()
    dev = "cuda:0"
    torch.cuda.set_device(0)

    over = {}
    toy = args.config == "toy"
    if not toy:
        args.config = int(args.config)
    if args.config == 5 and args.method == "spechub":
        over = dict(k=2, depth=4)
    if args.batch > 0:
        over["B"] = args.batch

    def make_workload(seed):
        if toy:
            repeats = max(1, args.batch // 200) if args.batch > 0 else 512
            return W.toy_pairs(0.25, 0.7, 200, repeats=repeats, seed=seed, device=dev)
        w = W.config(args.config, device=dev, seed=seed, **over)
        if args.batch > 0 and "_B%d_" % args.batch not in w.name:
            # another batch size than the configuration's: its own name, so that no profile
            # summary of the configuration's own size is taken for it
            w.name += "@B=%d" % args.batch
        return w

    wl0 = make_workload(args.seed)
    alg_bytes = wl0.algorithmic_bytes()
    copies = args.copies or max(2, -(-3 * 256 * 2 ** 20 // alg_bytes))   # >= 3x the Infinity Cache
    if alg_bytes > 2 ** 30:
        copies = args.copies or 2
    wls = [wl0] + [make_workload(args.seed + 1 + i) for i in range(copies - 1)]
    k, N, Bn = wl0.k, wl0.N, wl0.B
    pbs = [B.Problem.from_workload(w) for w in wls]
    u_d = [B.philox_uniform(args.seed + i, 1, Bn * N, k, device=dev).view(Bn, N, k) for i in range(copies)]
    u_v = [B.philox_uniform(args.seed + i, 2, Bn * N, k + 1, device=dev).view(Bn, N, k + 1) for i in range(copies)]
    plans = [B.StepPlan(args.method, pbs[i], u_d[i], u_v[i], hand_stats=not args.no_stats) for i in range(copies)]
    stream = B._stream()

    # where the tree walk runs: inside the verify kernel (two launches per step) or as a launch
    # of its own (three); by default the binding's rule by batch size decides
    fused = plans[0].walk_in_verify
    if args.separate_walk:
        fused = False
    if args.walk_in_verify:
        fused = True

    def step(i, ev=None):
        pl = plans[i % copies]
        pl.draft(stream)
        if ev is not None:
            ev[0].record()
        if fused:
            pl.verify_and_walk(stream)
        else:
            pl.verify(stream)
        if ev is not None:
            ev[1].record()
        if not fused:
            pl.walk(stream)
        return pl.out["accept_depth"]

    if args.calibration_copy:
        src = torch.empty(512 * 2 ** 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    # Set-up, untimed and apart from the W warmup steps: the step is run for SETTLE_S seconds so that
    # the GPU's clocks are at their working point whatever W is (a timed region that starts within
    # the first milliseconds of GPU work reads about 2 % slow on this workload: 55.5 against 54.4 us)
    t_settle = time.perf_counter()
    i_settle = 0
    while time.perf_counter() - t_settle < SETTLE_S:
        for _ in range(50):
            step(i_settle)
            i_settle += 1
        torch.cuda.synchronize()
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    # Optional: one HIP graph per input copy holding the step's three launches, replayed in the
    # timed region.
    graphs = []
    if args.graph:
        side = torch.cuda.Stream()          # default priority
        side.wait_stream(torch.cuda.current_stream())
        for pl in plans:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                st = B._stream()
                pl.draft(st)
                if fused:
                    pl.verify_and_walk(st)
                else:
                    pl.verify(st)
                    pl.walk(st)
            graphs.append(g)
        torch.cuda.synchronize()
        # a replay must give what the eager step gives (checked on every copy, twice, with eager work between)
        for rnd in range(2):
            for i, g in enumerate(graphs):
                want = step(i).clone()
                want_tok = plans[i].out["emitted"].clone()
                plans[i].out["accept_depth"].fill_(-7)
                plans[i].out["emitted"].fill_(-7)
                g.replay()
                torch.cuda.synchronize()
                if not (torch.equal(plans[i].out["accept_depth"], want) and torch.equal(plans[i].out["emitted"], want_tok)):
                    print("bench.py: graph replay differs from the eager step", file=sys.stderr)
                    sys.exit(4)
        for i in range(min(args.warmup, 10)):
            graphs[i % copies].replay()
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    if graphs:
        for i in range(args.steps):
            graphs[i % copies].replay()
        ad = plans[(args.steps - 1) % copies].out["accept_depth"]
    else:
        for i in range(args.steps):
            ad = step(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # the verify kernel inside eager steps, bracketed by events on the launch stream
    events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range(KERNEL_REPS)]
    for i, ev in enumerate(events):
        step(i, ev)
    torch.cuda.synchronize()

    ms_per_step = 1e3 * dt / args.steps
    nodes_per_s = Bn * N * args.steps / dt
    bracket_ms = sum(e0.elapsed_time(e1) for e0, e1 in events) / len(events)
    # A bracket also holds what the two event markers cost (a few microseconds, as much as a
    # tenth of this kernel).  The kernel's own duration is taken as the difference between a
    # bracket around two launches and a bracket around one, both measured after the timed
    # region on the rotating inputs: the markers cancel, one launch (with the gap to its
    # neighbour) remains.  rocprofv3's kernel trace, which has no markers, is the cross-check.
    reps = KERNEL_REPS

    def differential(prepare, launch):
        """Average duration of launch(plan): (bracket around two launches) - (bracket around one)."""
        one = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        two = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for i in range(reps):
            a, b = plans[(2 * i) % copies], plans[(2 * i + 1) % copies]
            prepare(a)
            prepare(b)
            one[i][0].record()
            launch(a)
            one[i][1].record()
            two[i][0].record()
            launch(b)
            launch(a)
            two[i][1].record()
        torch.cuda.synchronize()
        one_ms = sum(e0.elapsed_time(e1) for e0, e1 in one) / reps
        two_ms = sum(e0.elapsed_time(e1) for e0, e1 in two) / reps
        return two_ms - one_ms, one_ms

    verify_launch = (lambda pl: pl.verify_and_walk(stream)) if fused else (lambda pl: pl.verify(stream))
    kernel_ms, one_ms = differential(lambda pl: pl.draft(stream), verify_launch)
    event_overhead_ms = one_ms - kernel_ms
    achieved = alg_bytes / (kernel_ms * 1e-3) / 1e9
    draft_ms, _ = differential(lambda pl: None, lambda pl: pl.draft(stream))
    # the other placement of the walk, measured beside the one the step uses: the same verify
    # kernel without (or with) the walk in it, and the step with three (or two) launches
    other_launch = (lambda pl: pl.verify(stream)) if fused else (lambda pl: pl.verify_and_walk(stream))
    other_kernel_ms, _ = differential(lambda pl: pl.draft(stream), other_launch)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for i in range(args.steps):
        pl = plans[i % copies]
        pl.draft(stream)
        other_launch(pl)
        if fused:
            pl.walk(stream)
    torch.cuda.synchronize()
    other_step_ms = 1e3 * (time.perf_counter() - t1) / args.steps
    es = 2 if wl0.dtype == "bf16" else 4
    draft_bytes = Bn * wl0.n_internal * wl0.V * es
    # Reference line: a plain device copy of the same target rows (the library's copy kernel,
    # nothing of the method), timed the same way on the rotating copies: what a kernel that only
    # moves bytes reaches on a buffer of this size (it reads and writes, so twice the bytes).
    srcs = [w.target for w in wls]
    dst = torch.empty_like(srcs[0])
    for v in srcs:
        dst.copy_(v)
    r_one = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    r_two = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for i in range(reps):
        a, b = srcs[(2 * i) % copies], srcs[(2 * i + 1) % copies]
        r_one[i][0].record()
        dst.copy_(a)
        r_one[i][1].record()
        r_two[i][0].record()
        dst.copy_(b)
        dst.copy_(a)
        r_two[i][1].record()
    torch.cuda.synchronize()
    copy_ms = (sum(e0.elapsed_time(e1) for e0, e1 in r_two) - sum(e0.elapsed_time(e1) for e0, e1 in r_one)) / reps
    copy_bytes = 2 * srcs[0].numel() * srcs[0].element_size()
    plain_copy_gbs = copy_bytes / (copy_ms * 1e-3) / 1e9 if copy_ms > 0 else None
    del dst
    tps = float(ad.float().mean().item()) + 1.0
    kernel_key = "%s_verify:%s" % (args.method, wl0.name)
    traffic = read_traffic(kernel_key)
    draft_traffic = read_traffic("%s_draft:%s" % (args.method, wl0.name))

    if toy:
        headline = {"metric": "toy-experiment (p, q) pairs drafted and verified per second at V=50 (App. D)",
                    "value": Bn * args.steps / dt, "unit": "pairs/s", "nodes_per_s": nodes_per_s}
    else:
        headline = {"metric": metric_name(wl0), "value": nodes_per_s, "unit": "nodes/s"}
    out = {
        **headline, "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl0.name, "method": args.method, "B": Bn, "nodes_per_tree": N, "V": wl0.V,
                   "k": k, "storage": wl0.dtype, "temperature": wl0.temp_target,
                   "step": "draft+verify+walk",
                   "launch": "hip graph replay" if graphs else
                             ("two launches (walk inside the verify kernel)" if fused else "three launches"),
                   "input_copies_rotated": copies,
                   "settle_s_before_warmup": SETTLE_S,
                   "early_exit": True,
                   "draft_stats_handed_to_verify": not args.no_stats,
                   "tokens_per_step_last_batch": tps},
        # achieved = ALGORITHMIC bytes (every needed row once: the target row of every node, the draft
        # row of every internal node) / kernel time.  With the draft call's records and early exit
        # the kernel skips the draft rows of nodes decided by their first test, so it moves fewer
        # bytes than that: `traffic` (rocprofv3 counters, offline) and `frac_of_bytes_moved` say
        # what the memory system really did.
        "roofline": {"bound": "hbm", "kernel": "%s_verify" % args.method, "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "achieved_is": "algorithmic bytes (includes rows an early exit skips) / kernel time",
                     "algorithmic_bytes_per_launch": alg_bytes, "kernel_ms": kernel_ms,
                     "kernel_reps": reps,
                     "event_bracket_ms": bracket_ms, "event_overhead_ms": event_overhead_ms,
                     "traffic": traffic,
                     "traffic_source": None if traffic is None else
                                       "offline: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this command, profiles/hbm_traffic.txt",
                     "hbm_measured_gbs": None if traffic is None else traffic / (kernel_ms * 1e-3) / 1e9,
                     "frac_of_bytes_moved": None if traffic is None else traffic / (kernel_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "plain_copy_reference": {"gbs": plain_copy_gbs, "bytes": copy_bytes,
                                              "what": "device copy of the target rows of one input copy, "
                                                      "bytes read + written"}},
        "other_walk_placement": {
            "launch": "three launches (walk as a launch of its own)" if fused else "two launches (walk inside the verify kernel)",
            "ms_per_step": other_step_ms, "nodes_per_s": Bn * N / (other_step_ms * 1e-3),
            "verify_kernel_ms": other_kernel_ms,
            "verify_frac": alg_bytes / (other_kernel_ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "other_kernels": {"%s_draft" % args.method: {
            "kernel_ms": draft_ms, "algorithmic_bytes_per_launch": draft_bytes,
            "achieved": draft_bytes / (draft_ms * 1e-3) / 1e9 if draft_ms > 0 else None,
            "frac": draft_bytes / (draft_ms * 1e-3) / 1e9 / HBM_PEAK_GBS if draft_ms > 0 else None,
            "traffic": draft_traffic}},
        "whole_step": {"algorithmic_bytes": alg_bytes, "gbs": alg_bytes / (ms_per_step * 1e-3) / 1e9,
                       "frac": alg_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                       "what": "the verify call's algorithmic bytes over the whole step's time "
                               "(the draft call re-reads the draft rows: not counted twice)"},
    }
    if not args.no_path_only:
        # the same step with verification restricted to the nodes the walk visits (the walk is
        # inside that kernel); reported beside the headline, never as it
        psteps = KERNEL_REPS
        for i in range(min(args.warmup, 10)):
            plans[i % copies].draft(stream)
            plans[i % copies].verify_path(stream)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(psteps):
            pl = plans[i % copies]
            pl.draft(stream)
            pl.verify_path(stream)
        torch.cuda.synchronize()
        pdt = time.perf_counter() - t0
        visited = int((plans[(psteps - 1) % copies].out["outcome"] != B.UNVISITED).sum().item())
        out["path_only"] = {"step": "draft+verify_path", "steps": psteps, "ms_per_step": 1e3 * pdt / psteps,
                            "trees_per_s": Bn * psteps / pdt,
                            "visited_nodes_per_s": visited * psteps / pdt,
                            "visited_nodes_last_batch": visited,
                            "full_step_trees_per_s": Bn * args.steps / dt}
    if not args.no_cpu_baseline:
        threads = min(16, os.cpu_count() or 1)
        sample_B = min(Bn, max(1, (64 * 32000) // wl0.V))     # about 2000 config-3-sized node rows
        rows = (W.rows_as_numpy(wl0.target[:sample_B]), W.rows_as_numpy(wl0.draft[:sample_B]))
        method_id = {"spechub": 0, "rrs": 1, "rrsw": 2}[args.method]
        repeats = 24
        v, secs = cpu_baseline(rows, k, wl0.depth, (wl0.temp_target, wl0.temp_draft), method_id, repeats, threads)
        out["cpu_baseline"] = {"value": v, "unit": "nodes/s", "cores": threads, "kind": "oracle",
                               "sample": "%d trees (%d nodes) of the same batch x %d repeats, %.1f s wall"
                                         % (sample_B, sample_B * N, repeats, secs)}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
