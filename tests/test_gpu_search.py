"""The whole search of Alg. 1 (all window sizes, early exit at the lower bound) on the GPU
against the oracle's candidate-by-candidate version, through the C ABI."""
import json
import os

import pytest

from paper_2311_15269_amd import workloads as W
from tests import schedule_checks as SC

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: the HIP path has no CPU fallback")
    from paper_2311_15269_amd import binding
    binding.load_library()
    return binding


def linear(p, tf, tb, M, space="canonical"):
    return W.pipeline_problem(W.linear_placement(p), [tf] * p, [tb] * p, p, 1, M, space)


CASES = [
    ("cfg1-factorial", W.config1(), 4, 1 << 30, 0, True),
    ("cfg1-factorial-small-launches", W.config1(), 4, 1 << 30, 7, True),
    ("cfg1-canonical", dict(W.config1(), space="canonical"), 2, 1 << 30, 0, True),
    ("3dev", linear(3, 1, 2, 3), 8, 1 << 30, 4096, True),
    ("3dev-tight", linear(3, 1, 2, 2), 4, 1 << 30, 0, True),
    ("3dev-tight-no-bound", linear(3, 1, 2, 2), 3, 1 << 30, 1000, False),
    ("3dev-times-2-3", linear(3, 2, 3, 3), 8, 1 << 30, 0, True),
    ("1dev", W.pipeline_problem([0], [3], [5], 1, 1, 1, "canonical"), 4, 1 << 20, 0, True),
    ("inference-4", {"name": "inference-4", "D": 4, "K": 4, "NR": 1, "M": 1, "t": [2, 1, 3, 2], "m": [0] * 4,
                     "dev_mask": [1, 2, 4, 8], "deps": [(0, 1), (1, 2), (2, 3)], "space": "canonical", "seed": 0,
                     "lead_step_q16": 0}, 5, 1 << 20, 0, True),
    ("cfg3-repair", W.config3(), 4, 20000, 4096, True),
    ("cfg3-strict", dict(W.config3(), space="sampled_strict"), 3, 5000, 0, True),
    ("cfg4-tp", dict(W.config4(), M=9), 4, 6000, 2048, True),
    ("cfg5-repair", W.config5(), 8, 3000, 1024, True),
    ("cfg5-repair-no-bound", W.config5(), 6, 1000, 0, False),
    ("xshape-two-chains", W.xshape_problem(4, 1, 2, 1, 4), 3, 4000, 1024, False),
    # graphs with fan-in and fan-out, a pipeline on 12 devices, six block types per device
    ("kshape-canonical", W.kshape_problem(1, 3, space="canonical"), 3, 1 << 30, 0, True),
    ("diamond-repair", W.diamond_problem(1, 4), 4, 6000, 1024, True),
    ("12-devices", W.pipeline_problem(W.linear_placement(12), [1 + (i % 2) for i in range(12)], [2] * 12, 12, 1, 3,
                                      "sampled_repair", seed=5, lead_step_q16=20000), 3, 3000, 0, True),
    ("six-types-a-device", W.pipeline_problem([0, 1, 0, 1, 0, 1], [1, 2, 1, 1, 2, 1], [2, 1, 2, 2, 1, 2], 2, 1, 9,
                                              "sampled_repair", seed=6, lead_step_q16=30000), 4, 4000, 512, True),
    # window sizes beyond 8 (sampled spaces)
    ("10-devices-to-nr-11", W.pipeline_problem(list(range(10)), [1] * 10, [2] * 10, 10, 1, 14, "sampled_repair", seed=9,
                                               lead_step_q16=20000), 11, 150, 0, False),
    ("4-devices-cap-1-to-nr-12", W.pipeline_problem(list(range(4)), [1] * 4, [2] * 4, 4, 1, 1, "sampled_repair", seed=9,
                                                    lead_step_q16=20000), 12, 150, 64, False),
]


@pytest.mark.parametrize("name,problem,max_nr,budget,launch,bound", CASES, ids=[c[0] for c in CASES])
def test_search_matches_the_oracle(gpu, name, problem, max_nr, budget, launch, bound):
    from oracle import oracle as O
    want = O.search(problem, max_nr, budget, use_inflight_bound=bound)
    got, best = gpu.search(problem, max_nr, budget, launch_candidates=launch, use_inflight_bound=bound)
    for key in ("inflights", "lower_bound", "nr_tried", "best_nr", "best_period", "best_index", "early_exit",
                "period_nr", "index_nr"):
        assert got[key] == want[key], (name, key, got, want)
    # the GPU scores whole launches: at least what the candidate-by-candidate scan saw, same for full windows
    step = launch if launch else 1 << 24
    for nr, (g, w) in enumerate(zip(got["evaluated_nr"], want["evaluated_nr"]), start=1):
        last = want["early_exit"] and nr == want["nr_tried"]
        if last:
            assert w <= g < w + step
        else:
            assert g == w
    if want["best_nr"] == 0:
        assert best is None
        return
    # the returned handle holds the incumbent: its decoded form is what the oracle decodes, and it completes
    o = O.Oracle(dict(problem, NR=want["best_nr"]))
    b = best.best()
    sc = o.eval_index(want["best_index"])
    assert (b["period"], b["index"], b["peak"]) == (sc["period"], want["best_index"], sc["peak"])
    cand = best.best_candidate()
    status, leads, orders = o.decode(want["best_index"])
    assert status == 0 and cand["leads"] == leads and cand["orders"] == orders
    N = 3 * want["best_nr"] + 2
    sched = best.complete_schedule(N)
    ok, makespan, peaks = SC.check_flat_schedule(problem, N, sched["start"].tolist(), sched["dev_order"])
    assert ok and makespan == sched["makespan"] and max(peaks) <= problem["M"]


def test_four_stage_pipeline_exits_at_the_stored_exhaustive_best(gpu):
    """Sequential 4-stage placement, M = 4: windows of 1, 2, 3 micro-batches (16 + 10,368 + 5,760,000
    candidates, compared with oracle sweeps) only reach the round trip time 12; the window of 4
    reaches the bound 12 = 4 * 3 at the index the stored exhaustive oracle result names, and the
    search stops in that launch."""
    from oracle import oracle as O
    want4 = json.load(open(os.path.join(GOLDEN, "config2_exhaustive.json")))
    prob = W.config2()
    got, best = gpu.search(prob, 8, 1 << 62)
    assert got["inflights"] == 4 and got["lower_bound"] == 3 and got["nr_tried"] == 4 and got["early_exit"]
    for nr in (1, 2, 3):
        o = O.Oracle(dict(prob, NR=nr))
        r = o.sweep(0, o.count, threads=8)
        assert (got["period_nr"][nr - 1], got["index_nr"][nr - 1], got["evaluated_nr"][nr - 1]) == \
               (r["period"], r["index"], o.count)
    assert (got["best_nr"], got["best_period"], got["best_index"]) == (4, want4["period"], want4["index"])
    assert got["evaluated_nr"][3] == ((want4["index"] >> 24) + 1) << 24
    assert best.best()["peak"] == want4["peak"]


def test_xshape_window_of_two_reaches_the_bubble_of_the_direct_bidirectional_schedule(gpu):
    """Bidirectional pipelines on 4 devices, tf = 1, tb = 2 (lower bound 6 per micro-batch): the window of one
    micro-batch repeats every 12 (bubble 1/2); with two micro-batches the sampled search finds period 15, bubble 1/5,
    the figure Table II lists for the direct bidirectional schedule; the oracle confirms both candidates."""
    from oracle import oracle as O
    prob = W.xshape_problem(4, 1, 2, 1, 4, seed=77)
    got, best = gpu.search(prob, 2, 1 << 24, use_inflight_bound=False)
    assert got["lower_bound"] == 6 and got["period_nr"] == [12, 15] and got["best_nr"] == 2
    for nr in (1, 2):
        sc = O.Oracle(dict(prob, NR=nr)).eval_index(got["index_nr"][nr - 1])
        assert sc["status"] == 0 and sc["period"] == got["period_nr"][nr - 1] and sc["peak_max"] <= 4
