"""Searched completion on the GPU (warm-up / cool-down orders as perturbed greedy schedules around the best
window, Sec. IV-C) against the oracle: every candidate's makespan, the best (makespan, ordinal) and the
schedule that is handed back, through the C ABI."""
import numpy as np
import pytest

from paper_2311_15269_amd import workloads as W
from tests import schedule_checks as SC

pytestmark = pytest.mark.gpu
INT32_MAX = 2 ** 31 - 1


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: the HIP path has no CPU fallback")
    from paper_2311_15269_amd import binding
    binding.load_library()
    return binding


CASES = [
    ("cfg1", W.config1(), 576, 9, 2, 700),
    ("cfg2-slice", W.config2(), 1 << 21, 16, 2, 1000),
    ("cfg3", W.config3(), 4096, 20, 3, 1500),
    ("cfg3-long", W.config3(), 4096, 64, 1, 300),
    ("cfg4-tp", dict(W.config4(), M=9), 6000, 14, 2, 1000),
    ("cfg5", W.config5(), 2048, 24, 4, 600),
    ("cfg5-64", W.config5(), 2048, 64, 2, 200),
    ("lin3", W.pipeline_problem(W.linear_placement(3), [1, 2, 1], [2, 3, 1], 3, 3, 3, "canonical"), 1 << 30, 10, 5, 333),
    # micro-batch graphs with fan-in and fan-out (Sec. III-A, Eq. 1 [3]): two encoders into a joint stage, a diamond
    ("kshape", W.kshape_problem(2, 4), 4000, 12, 3, 700),
    ("kshape-nr4", W.kshape_problem(4, 5), 4000, 21, 6, 500),
    ("diamond", W.diamond_problem(3, 5), 4000, 12, 3, 700),
    ("diamond-tight", W.diamond_problem(2, 3), 4000, 17, 8, 500),
]


@pytest.mark.parametrize("name,prob,budget,N,J,ncand", CASES, ids=[c[0] for c in CASES])
def test_completion_candidates_match_the_oracle(gpu, name, prob, budget, N, J, ncand):
    from oracle import Oracle
    g = gpu.Problem(prob)
    n = min(budget, g.candidate_count())
    g.eval_candidates(0, n)
    best = g.best()
    assert best["feasible"]
    o = Oracle(prob)
    status, leads, orders = o.decode(best["index"])
    cand = g.best_candidate()
    assert cand["leads"] == leads and cand["orders"] == orders
    # per candidate, a range that does not start at 0 and is no multiple of the wave size
    want, want_best, want_ord = o.completion_scores(leads, orders, N, 0, ncand, J)
    got = g.score_completions(N, J, 0, ncand).cpu().numpy()
    bad = np.nonzero(got != want)[0]
    assert bad.size == 0, (name, "first mismatch at ordinal", int(bad[0]), int(got[bad[0]]), int(want[bad[0]]))
    got2 = g.score_completions(N, J, 37, 101).cpu().numpy()
    assert np.array_equal(got2, want[37:138])
    # the search, in two pieces submitted out of order, and the schedule it hands back
    g.search_completions(N, J, ncand // 2, ncand - ncand // 2)
    g.search_completions(N, J, 0, ncand // 2)
    g.search_completions(N, J, 5, 0)                       # empty range
    sched = g.best_completion(N)
    assert (sched["makespan"], sched["ordinal"]) == (want_best, want_ord)
    ref = o.complete_jitter(leads, orders, N, want_ord, J)
    assert sched["start"].tolist() == ref["start"].tolist() and sched["dev_order"] == ref["dev_order"]
    ok, makespan, peaks = SC.check_flat_schedule(prob, N, sched["start"].tolist(), sched["dev_order"])
    assert ok and makespan == sched["makespan"] and max(peaks) <= prob["M"]
    greedy = g.complete_schedule(N)
    assert greedy["makespan"] == want[0] >= sched["makespan"]


def test_the_windows_block_by_block_equal_their_matrix(gpu, monkeypatch):
    """The kernel applies the R replayed windows as one (max, +) matrix; TESSEL_REPLAY_BLOCKS=1 makes it run them
    block by block instead (the path of windows with too many crossing values): both equal the oracle."""
    from oracle import Oracle
    for prob, budget, N, J, ncand in ((W.config5(), 2048, 40, 3, 400), (W.config3(), 4096, 33, 2, 500),
                                      (W.xshape_problem(4, 1, 2, 2, 4), 4096, 11, 1, 300)):
        o = Oracle(prob)
        scores = []
        for replay in ("0", "1"):
            monkeypatch.setenv("TESSEL_REPLAY_BLOCKS", replay)
            g = gpu.Problem(prob)
            g.eval_candidates(0, budget)
            status, leads, orders = o.decode(g.best()["index"])
            scores.append(g.score_completions(N, J, 3, ncand).cpu().numpy())
        monkeypatch.delenv("TESSEL_REPLAY_BLOCKS")
        want, _, _ = o.completion_scores(leads, orders, N, 3, ncand, J)
        assert np.array_equal(scores[0], want) and np.array_equal(scores[1], want), prob["name"]


@pytest.mark.parametrize("seed", [51, 52, 53])
def test_completion_candidates_on_random_graphs(gpu, seed):
    """seeded random micro-batch graphs on 2-5 devices: every completion candidate's makespan, the best and its schedule"""
    from oracle import Oracle
    from tests.test_gpu_dag import random_graph_problem
    rng = np.random.default_rng(seed)
    ran = 0
    for case in range(10):
        prob = dict(random_graph_problem(rng), space="sampled_repair")
        prob["M"] = max(prob["M"], prob["NR"])
        g, o = gpu.Problem(prob), Oracle(prob)
        g.eval_candidates(int(rng.integers(0, 1 << 30)), 4096)
        best = g.best()
        if not best["feasible"]:
            continue
        status, leads, orders = o.decode(best["index"])
        N = int(rng.integers(prob["NR"] + max(leads), 50))
        J, first, ncand = int(rng.integers(1, 9)), int(rng.integers(0, 40)), int(rng.integers(100, 400))
        want, want_best, want_ord = o.completion_scores(leads, orders, N, first, ncand, J)
        got = g.score_completions(N, J, first, ncand).cpu().numpy()
        assert np.array_equal(got, want), (seed, case, prob)
        g.search_completions(N, J, first, ncand)
        if want_best is None:
            with pytest.raises(gpu.TesselError) as e:
                g.best_completion(N)
            assert e.value.code == -10
            continue
        sched = g.best_completion(N)
        assert (sched["makespan"], sched["ordinal"]) == (want_best, want_ord), (seed, case)
        ok, makespan, peaks = SC.check_flat_schedule(prob, N, sched["start"].tolist(), sched["dev_order"])
        assert ok and makespan == sched["makespan"] and max(peaks) <= prob["M"]
        ran += 1
    assert ran >= 5


def test_greedy_completion_matches_the_worked_example(gpu):
    """The hand-worked tie-order example of the oracle's pins (one device, types of 1, 2, 3 time units, leads 2, 1, 0,
    five micro-batches): whatever order the best window has, the device never idles, so warm-up and cool-down start
    where the derivation puts them."""
    prob = {"name": "one-device", "D": 1, "K": 3, "NR": 3, "M": 0, "t": [1, 2, 3], "m": [0, 0, 0], "dev_mask": [1, 1, 1],
            "deps": [], "space": "sampled_repair", "seed": 1, "lead_step_q16": 0, "fixed_leads": [2, 1, 0]}
    g = gpu.Problem(prob)
    g.eval_candidates(0, 64)
    assert g.best()["period"] == 18
    sched = g.complete_schedule(5)
    start = sched["start"].tolist()
    assert sched["makespan"] == 30
    assert (start[0][0], start[1][0], start[0][1]) == (0, 1, 3)            # warm-up: A0, B0, A1
    assert (start[2][3], start[1][4], start[2][4]) == (22, 25, 27)         # cool-down: C3, B4, C4
    assert int(g.score_completions(5, 0, 0, 4).cpu().numpy()[0]) == 30


def test_completion_argument_checks(gpu):
    g = gpu.Problem(W.config3())
    with pytest.raises(gpu.TesselError) as e:
        g.search_completions(20, 2, 0, 10)                 # nothing scored yet
    assert e.value.code == -7
    g.eval_candidates(0, 4096)
    with pytest.raises(gpu.TesselError) as e:
        g.search_completions(3, 2, 0, 10)                  # fewer micro-batches than one window
    assert e.value.code == -8
    with pytest.raises(gpu.TesselError) as e:
        g.search_completions(1100, 2, 0, 10)               # micro-batch numbers are kept in 10 bits, times in 16
    assert e.value.code == -4
    with pytest.raises(gpu.TesselError) as e:
        g.search_completions(20, 64, 0, 10)                # the jitter in 6 bits
    assert e.value.code == -4
    with pytest.raises(gpu.TesselError) as e:
        g.search_completions(20, -1, 0, 10)
    assert e.value.code == -1
    g.search_completions(20, 2, 0, 10)
    with pytest.raises(gpu.TesselError) as e:
        g.best_completion(21)                              # not the number of micro-batches that was searched
    assert e.value.code == -1


def test_a_new_best_window_restarts_the_completion_search(gpu):
    from oracle import Oracle
    prob = W.config3()
    g = gpu.Problem(prob)
    o = Oracle(prob)
    g.eval_candidates(0, 64)
    first = g.best()
    g.search_completions(20, 3, 0, 200)
    a = g.best_completion(20)
    g.eval_candidates(64, 8192)
    second = g.best()
    assert second["index"] != first["index"]
    g.search_completions(20, 3, 0, 200)
    b = g.best_completion(20)
    status, leads, orders = o.decode(second["index"])
    want, want_best, want_ord = o.completion_scores(leads, orders, 20, 0, 200, 3)
    assert (b["makespan"], b["ordinal"]) == (want_best, want_ord)
    assert a["period"] == first["period"] and b["period"] == second["period"]
