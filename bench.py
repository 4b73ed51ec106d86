#!/usr/bin/env python3
"""Benchmark of the repetend-candidate evaluator on one MI355X.

One step = the whole hot path over one batch: score every candidate of the workload
(decode, build, memory, period), reduce to the best (period, index), read it back and
complete the schedule from it.  Workload: the 8-simulated-device folded ("V") placement
with 16 stages, N_R = 8, 2^28 seeded candidates, completion to 64 micro-batches.
Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_INT32_OPS = 256 * 64 * 2.4e9 / 1e12      # T int32 lane-ops/s: 256 CUs x 64 lanes x 2.4 GHz, full-rate VALU ops
PEAK_LDS_OPS = 256 * 32 * 2.4e9 / 1e12        # T 32-bit LDS lane accesses/s: 256 CUs x 32 banks x 2.4 GHz
COUNTERS_MD = os.path.join(ROOT, "profiles", "eval_fast_kernel_cfg5_counters.md")


def profiled_traffic():
    """HBM bytes of one launch of 2^26 candidates of the headline workload: the copy-calibrated FETCH_SIZE + WRITE_SIZE
    of the committed rocprofv3 counter summary, and the commit the kernel was at when they were taken.  The line
    `traffic_bytes_per_2p26_launch: <bytes> (kernel at <commit>)` of that file."""
    try:
        for line in open(COUNTERS_MD):
            if line.startswith("traffic_bytes_per_2p26_launch:"):
                parts = line.split()
                return int(parts[1]), parts[-1].rstrip(")")
    except OSError:
        pass
    return None, None


DECODE_OPS, BUILD_OPS, SWEEP_OPS = 17, 34, 2   # per block: see algorithmic_ops


def algorithmic_ops(prob, n_candidates, n_blocks_placed, n_sweeps):
    """Integer operations of a straight-line statement of the method (not what the kernel happens to issue):
    decode 17 per block of the window (half a hash word, digit, pick) for every candidate, build 34 per block
    placed (select, union of runnable entries, remove, new head, counters, masks, memory add + max, emit), and 2
    (one max, one add) per block and executed window sweep."""
    n = prob["K"] * prob["NR"]
    return n_candidates * n * DECODE_OPS + n_blocks_placed * BUILD_OPS + n_sweeps * n * SWEEP_OPS


def host_threads():
    """threads the oracle gets: the cores this process may run on"""
    try:
        return max(1, len(os.sched_getaffinity(0)))
    except AttributeError:
        return os.cpu_count() or 1


def oracle_baseline(prob, sample):
    """The CPU oracle as it stands on the first `sample` ordinals of the workload: all host cores, then one thread on
    a sixteenth of the sample."""
    from oracle import Oracle
    cores = host_threads()
    orc = Oracle(prob)
    t1 = time.perf_counter()
    ref = orc.sweep(0, sample, threads=cores)
    cdt = time.perf_counter() - t1
    single = max(1, sample // 16)
    t1 = time.perf_counter()
    orc.sweep(0, single, threads=1)
    sdt = time.perf_counter() - t1
    return {"value": sample / cdt, "unit": "candidates/s", "cores": cores, "kind": "oracle",
            "sample": "first 2^%d ordinals of the same workload, %d threads, %.1f s; one thread on the first %d: %.1f s"
                      % (sample.bit_length() - 1, cores, cdt, single, sdt),
            "single_thread_value": single / sdt,
            "oracle_ops_per_candidate": ref["ops"] / sample}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--log2-candidates", type=int, default=28, help="candidates per step = 2^this (28 = the workload)")
    ap.add_argument("--log2-chunk", type=int, default=26, help="candidates per call of the entry point (one launch)")
    ap.add_argument("--cpu-sample-log2", type=int, default=20, help="oracle baseline sample size")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--search", action="store_true",
                    help="time the whole search of Alg. 1 (window sizes 1..4, early exit) on the sequential 4-stage "
                         "placement instead of the headline workload; prints its own JSON line")
    ap.add_argument("--completions", action="store_true",
                    help="time the searched completion (perturbed greedy warm-up / cool-down orders around the best window "
                         "of the first 2^24 candidates, 64 micro-batches) instead of the headline workload")
    ap.add_argument("--log2-completions", type=int, default=20, help="completion candidates per step = 2^this")
    ap.add_argument("--jitter", type=int, default=2)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run one plain device copy of 1 GiB instead (reference for the FETCH_SIZE/WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; the problem's 8 'devices' are simulated "
              "entities of the schedule, not GPUs. Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    if args.calibrate_copy:
        src = torch.ones(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes": 1 << 30}))
        return
    from paper_2311_15269_amd import workloads
    from paper_2311_15269_amd.binding import Problem

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    if args.search:
        from paper_2311_15269_amd.binding import search
        prob = workloads.config2()
        for _ in range(args.warmup):
            search(prob, 8, 1 << 62)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            got, best = search(prob, 8, 1 << 62)
            sched = best.complete_schedule(16)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / args.steps
        print(json.dumps({"metric": "wall time of the whole schedule search (Alg. 1: window sizes, early exit, completion)",
                          "value": dt, "unit": "s", "higher_is_better": False, "n_gpus": 1, "steps": args.steps,
                          "warmup": args.warmup, "dtype": "int32", "data": "synthetic", "vs_baseline": None,
                          "config": {"workload": "sequential 4-stage placement, tf=1, tb=2, M=4, exhaustive canonical "
                                                 "spaces of N_R=1..4, completion to 16 micro-batches"},
                          "result": dict(got, makespan_16_microbatches=sched["makespan"]),
                          "candidates_scored": sum(got["evaluated_nr"]),
                          "candidates_per_s": sum(got["evaluated_nr"]) / dt}))
        return
    if args.completions:
        prob = workloads.config5()
        N = prob["num_microbatches"]
        gpu = Problem(prob)
        gpu.eval_candidates(0, 1 << 24)
        best = gpu.best()
        greedy = gpu.complete_schedule(N)
        n = 1 << args.log2_completions
        for _ in range(args.warmup):
            gpu.search_completions(N, args.jitter, 0, n)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(args.steps):
            gpu.search_completions(N, args.jitter, k * n, n)
        found = gpu.best_completion(N)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        blocks = prob["K"] * N
        # Straight-line operations of one completion candidate, the work the kernel does: a block of the two greedy
        # phases recomputes the offers of the types it can change (those on its device and its consumer: 8 operations
        # each: token/device maximum, jitter add, three eligibility tests, key packing), takes the minimum over the K
        # offers, commits (6) and draws the next jitter (7).  The replayed windows are not counted: the kernel applies
        # them as one (max, +) matrix (at most 32 x 16 terms), not block by block (one max and one add a block).
        cand = gpu.best_candidate()
        affected = max(sum(1 for j in range(prob["K"]) if (prob["dev_mask"][j] & prob["dev_mask"][i]) or (j, i) in
                           [(b, a) for a, b in prob["deps"]]) for i in range(prob["K"]))
        greedy_blocks = blocks - found["num_windows"] * prob["K"] * prob["NR"]
        ops = greedy_blocks * (8 * affected + (prob["K"] - 1) + 6 + 7)
        rate = n * args.steps / dt
        out = {"metric": "completion candidates (whole schedules of 64 micro-batches) scored/s", "value": rate,
               "unit": "candidates/s", "higher_is_better": True, "n_gpus": 1, "steps": args.steps,
               "warmup": args.warmup, "ms_per_step": dt / args.steps * 1e3, "dtype": "int32", "data": "synthetic",
               "vs_baseline": None,
               "config": {"workload": "cfg5 best window of the first 2^24 candidates, N=%d micro-batches (%d blocks), "
                                      "jitter %d, 2^%d completion candidates per step" % (N, blocks, args.jitter, args.log2_completions)},
               "result": {"window_period": best["period"], "windows": found["num_windows"],
                          "greedy_makespan": greedy["makespan"], "best_makespan": found["makespan"],
                          "best_ordinal": found["ordinal"]},
               "blocks_scheduled_per_s": rate * blocks,
               "roofline": {"bound": "alu", "achieved": ops * rate / 1e12, "peak": PEAK_INT32_OPS, "unit": "Tint32op/s",
                            "frac": ops * rate / 1e12 / PEAK_INT32_OPS, "traffic": None, "kernel": "complete_kernel",
                            "algorithmic_ops_per_candidate": ops,
                            "limited_by": "latency: every scheduled block of the greedy phases is a chain of dependent per-lane "
                                          "decisions through LDS, at two waves per SIMD "
                                          "(profiles/complete_kernel_cfg5_kernel_trace_counters.md)"}}
        if not args.no_cpu_baseline:
            from oracle import Oracle
            orc = Oracle(prob)
            sample = 1 << 16
            t1 = time.perf_counter()
            orc.completion_scores(cand["leads"], cand["orders"], N, 0, sample, args.jitter)
            cdt = time.perf_counter() - t1
            out["cpu_baseline"] = {"value": sample / cdt, "unit": "candidates/s", "cores": 1, "kind": "oracle",
                                   "sample": "completion candidates 0..%d of the same window, one thread, %.1f s" % (sample - 1, cdt)}
        print(json.dumps(out))
        return
    prob = workloads.config5()
    n_cand = 1 << args.log2_candidates
    chunk = min(1 << args.log2_chunk, n_cand)
    N = prob["num_microbatches"]
    gpu = Problem(prob)

    def step(events=None):
        gpu.reset()
        for first in range(0, n_cand, chunk):
            if events is not None:
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
            gpu.eval_candidates(first, chunk)
            if events is not None:
                b.record()
                events.append((a, b))
        best = gpu.best()
        sched = gpu.complete_schedule(N)
        return best, sched

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        best, sched = step(events)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    launch_ms = [a.elapsed_time(b) for a, b in events]
    avg_launch_s = sum(launch_ms) / len(launch_ms) / 1e3
    sweeps_per_cand = best["n_window_sweeps"] / best["n_evaluated"]
    blocks_per_cand = best["n_blocks_placed"] / best["n_evaluated"]
    total_blocks = prob["K"] * prob["NR"]
    # Work done: the kernel stops building a candidate that is over the memory cap at the end of its first build phase,
    # so only the blocks it placed (counted by the kernel) are priced.  The second figure prices every candidate at
    # the whole window, as the method is stated and as the per-candidate entry point computes it.
    ops_per_launch = algorithmic_ops(prob, chunk, blocks_per_cand * chunk, sweeps_per_cand * chunk)
    ops_whole_window = algorithmic_ops(prob, chunk, total_blocks * chunk, sweeps_per_cand * chunk)
    achieved = ops_per_launch / avg_launch_s / 1e12

    # practical ceiling: independent full-rate integer adds/maxes on every lane of the chip
    from paper_2311_15269_amd.binding import alu_probe
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    probe_ops, probe_out = alu_probe(n_cu * 16, 256)
    torch.cuda.synchronize()
    pa, pb = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    pa.record()
    probe_ops, _ = alu_probe(n_cu * 16, 20000, probe_out)
    pb.record()
    torch.cuda.synchronize()
    peak_measured = probe_ops / (pa.elapsed_time(pb) / 1e3) / 1e12
    traffic, traffic_commit = profiled_traffic()

    out = {
        "metric": "repetend candidates evaluated/sec + % peak VALU int ops, 8-dev V-shape",
        "value": n_cand * args.steps / dt,
        "unit": "candidates/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32", "data": "synthetic",
        "config": {"workload": "cfg5: 8 simulated devices, 16 folded stages, N_R=8, 256 blocks/window, "
                               "2^%d seeded candidates (sampled_repair), completion to %d micro-batches" % (args.log2_candidates, N),
                   "candidates_per_step": n_cand, "candidates_per_launch": chunk, "mem_cap": prob["M"]},
        "result": {"best_period": best["period"], "best_index": best["index"], "lower_bound": best["lower_bound"],
                   "peak_mem": best["peak"], "n_feasible": best["n_feasible"], "n_reject": best["n_reject"],
                   "makespan_%d_microbatches" % N: sched["makespan"], "windows": sched["num_windows"]},
        "roofline": {"bound": "alu", "achieved": achieved, "peak": PEAK_INT32_OPS, "unit": "Tint32op/s",
                     "frac": achieved / PEAK_INT32_OPS,
                     "peak_measured": peak_measured, "frac_of_measured": achieved / peak_measured,
                     "traffic": traffic if chunk == 1 << 26 else None, "traffic_measured_at_commit": traffic_commit,
                     "kernel": "eval_fast_kernel<8, 16, 2, false>", "avg_launch_ms": avg_launch_s * 1e3,
                     "algorithmic_ops_per_candidate": ops_per_launch / chunk,
                     "blocks_placed_per_candidate": blocks_per_cand,
                     "window_sweeps_per_candidate": sweeps_per_cand,
                     "frac_if_every_candidate_priced_at_the_whole_window": ops_whole_window / avg_launch_s / 1e12 / PEAK_INT32_OPS},
    }

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = oracle_baseline(prob, 1 << args.cpu_sample_log2)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
