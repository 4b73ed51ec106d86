"""Writes the stored brute-force results of the CPU oracle that the full-size GPU tests compare with.
Calls only oracle/ (and the shared problem descriptions).

    python tests/golden/make_exhaustive_golden.py 2 [threads]    -> config2_exhaustive.json
    python tests/golden/make_exhaustive_golden.py 3 [threads]    -> config3_full.json   (2^24 ordinals)
    python tests/golden/make_exhaustive_golden.py 4 [threads]    -> config4_full.json   (2^26 ordinals)
    python tests/golden/make_exhaustive_golden.py 5 [threads]    -> config5_full.json   (2^28 ordinals)

Config 2 is the whole canonical space of the 4-device linear problem (2,881,200,000 candidates, minutes
on 8 cores).  Configs 3-5 are the sampled spaces at the benchmark's sizes; their files also hold one
record per piece of 2^26 ordinals (the launch size of the benchmark), so that every launch of the GPU
sweep is compared on its own.  Config 5 takes about five hours on 6 cores; the file is rewritten after
every finished piece ("complete": false until the last one)."""
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import Oracle  # noqa: E402
from paper_2311_15269_amd import workloads  # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))
PIECE = 1 << 26


def merge(acc, r):
    """fold the sweep result r into acc: counters add up, the least (period, index) stays"""
    acc["n_evaluated"] += r["n_evaluated"]
    acc["n_feasible"] += r["n_feasible"]
    acc["n_reject"] = [a + b for a, b in zip(acc["n_reject"], r["n_reject"])]
    if r["n_feasible"] and (acc.get("period") is None or (r["period"], r["index"]) < (acc["period"], acc["index"])):
        acc["period"], acc["index"], acc["peak"] = r["period"], r["index"], r["peak"]


def empty():
    return {"n_evaluated": 0, "n_feasible": 0, "n_reject": [0] * 6, "period": None, "index": None, "peak": None}


def config2(threads):
    prob = workloads.config2()
    orc = Oracle(prob)
    total = orc.count
    t0 = time.time()
    out = empty()
    step = 1 << 27
    for first in range(0, total, step):
        n = min(step, total - first)
        merge(out, orc.sweep(first, n, threads=threads))
        print("%d / %d  %.0fs" % (first + n, total, time.time() - t0), flush=True)
    out["count"] = total
    out["lower_bound"] = orc.lower_bound
    out["workload"] = prob["name"]
    with open(os.path.join(HERE, "config2_exhaustive.json"), "w") as f:
        json.dump(out, f, indent=1)
    print(out)


def sampled(cfg, threads):
    prob = workloads.CONFIGS[cfg]()
    orc = Oracle(prob)
    total = prob["n_candidates"]
    path = os.path.join(HERE, "config%d_full.json" % cfg)
    t0 = time.time()
    out = empty()
    pieces = []
    step = 1 << 22                       # slices for visible progress
    for p0 in range(0, total, PIECE):
        pn = min(PIECE, total - p0)
        piece = empty()
        for first in range(p0, p0 + pn, step):
            n = min(step, p0 + pn - first)
            merge(piece, orc.sweep(first, n, threads=threads))
            print("cfg%d %d / %d  %.0fs" % (cfg, first + n, total, time.time() - t0), flush=True)
        merge(out, piece)
        piece["first"], piece["count"] = p0, pn
        pieces.append(piece)
        doc = dict(out, count=total, lower_bound=orc.lower_bound, workload=prob["name"], seed=prob["seed"],
                   pieces=pieces, complete=(p0 + pn == total))
        with open(path + ".tmp", "w") as f:
            json.dump(doc, f, indent=1)
        os.replace(path + ".tmp", path)
    print(doc)


def main():
    cfg = int(sys.argv[1]) if len(sys.argv) > 1 else 2
    threads = int(sys.argv[2]) if len(sys.argv) > 2 else (os.cpu_count() or 1)
    if cfg == 2:
        config2(threads)
    else:
        sampled(cfg, threads)


if __name__ == "__main__":
    main()
