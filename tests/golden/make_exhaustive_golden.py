"""Writes tests/golden/config2_exhaustive.json: the CPU oracle's brute-force result over the whole
canonical space of the 4-device linear problem (2,881,200,000 candidates).  Calls only oracle/.
Takes several minutes on 8 cores:  python tests/golden/make_exhaustive_golden.py [threads]"""
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import Oracle  # noqa: E402
from paper_2311_15269_amd import workloads  # noqa: E402


def main():
    threads = int(sys.argv[1]) if len(sys.argv) > 1 else (os.cpu_count() or 1)
    prob = workloads.config2()
    orc = Oracle(prob)
    total = orc.count
    t0 = time.time()
    # in slices, so that progress is visible; merging keeps the lowest index among equal periods
    best = None
    out = {"n_evaluated": 0, "n_feasible": 0, "n_reject": [0] * 6}
    step = 1 << 27
    for first in range(0, total, step):
        n = min(step, total - first)
        r = orc.sweep(first, n, threads=threads)
        out["n_evaluated"] += r["n_evaluated"]
        out["n_feasible"] += r["n_feasible"]
        out["n_reject"] = [a + b for a, b in zip(out["n_reject"], r["n_reject"])]
        if r["n_feasible"] and (best is None or r["period"] < best["period"]):
            best = {"period": r["period"], "index": r["index"], "peak": r["peak"]}
        print("%d / %d  %.0fs" % (first + n, total, time.time() - t0), flush=True)
    out.update(best)
    out["count"] = total
    out["lower_bound"] = orc.lower_bound
    out["workload"] = prob["name"]
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "config2_exhaustive.json"), "w") as f:
        json.dump(out, f, indent=1)
    print(out)


if __name__ == "__main__":
    main()
