"""Pins of the oracle's searched completion (warm-up / cool-down orders as perturbed greedy schedules,
Sec. IV-C): candidate 0 is the pinned greedy completion, every candidate is a valid schedule of Eq. 1 that
keeps the window orders, no candidate undercuts what the windows alone take, and the search never
loses against the greedy completion."""
import numpy as np
import pytest

from oracle import oracle as O
from paper_2311_15269_amd import workloads as W
from tests import schedule_checks as SC

INT32_MAX = 2 ** 31 - 1


def best_window(prob, budget):
    o = O.Oracle(prob)
    r = o.sweep(0, min(o.count, budget), threads=4)
    status, leads, orders = o.decode(r["index"])
    return o, r, leads, orders


CASES = [
    ("cfg1", W.config1(), 576, 9, 2),
    ("cfg2", W.config2(), 2000000, 16, 2),
    ("cfg3", W.config3(), 2000, 20, 3),
    ("cfg4-tp", dict(W.config4(), M=9), 3000, 14, 2),
    ("cfg5", W.config5(), 300, 24, 4),
]


@pytest.mark.parametrize("name,prob,budget,N,J", CASES, ids=[c[0] for c in CASES])
def test_candidate_zero_is_the_greedy_completion(name, prob, budget, N, J):
    o, r, leads, orders = best_window(prob, budget)
    ref = o.complete(leads, orders, N)
    for ordinal, amp in ((0, J), (5, 0), (0, 0)):
        got = o.complete_jitter(leads, orders, N, ordinal, amp)
        assert got["makespan"] == ref["makespan"]
        assert got["start"].tolist() == ref["start"].tolist() and got["dev_order"] == ref["dev_order"]


@pytest.mark.parametrize("name,prob,budget,N,J", CASES, ids=[c[0] for c in CASES])
def test_every_candidate_is_a_valid_schedule_around_the_same_windows(name, prob, budget, N, J):
    o, r, leads, orders = best_window(prob, budget)
    NR = prob["NR"]
    R = (N - max(leads)) // NR
    scores, best, best_ord = o.completion_scores(leads, orders, N, 0, 40, J)
    assert best == scores.min() and scores[best_ord] == best and best_ord == int(np.argmin(scores))
    assert best <= scores[0]                                   # the search never loses against the greedy schedule
    for ordinal in range(0, 40, 3):
        if scores[ordinal] == INT32_MAX:
            continue
        s = o.complete_jitter(leads, orders, N, ordinal, J)
        assert s["makespan"] == scores[ordinal]
        ok, makespan, peaks = SC.check_flat_schedule(prob, N, s["start"].tolist(), s["dev_order"])
        assert ok and makespan == s["makespan"] and max(peaks) <= prob["M"]
        assert s["makespan"] >= R * r["period"]                # R windows alone take R periods
        # blocks of one type run in micro-batch order on every device, and the windows keep the candidate's order
        for d, row in enumerate(s["dev_order"]):
            by_type = {}
            for blk in row:
                by_type.setdefault(blk // N, []).append(blk % N)
            assert all(v == sorted(v) for v in by_type.values())
            steady = [blk // N for blk in row if leads[blk // N] <= blk % N < leads[blk // N] + NR * R]
            assert steady == orders[d] * R


def test_uniform_pipeline_keeps_the_known_optimum():
    """1F1B on a uniform pipeline: the greedy completion already reaches (N + p - 1)(tf + tb); no candidate beats it."""
    p, tf, tb, N = 3, 1, 2, 9
    prob = W.pipeline_problem(W.linear_placement(p), [tf] * p, [tb] * p, p, p, p, "canonical")
    o, r, leads, orders = best_window(prob, 1 << 30)
    assert r["period"] == p * (tf + tb)
    scores, best, best_ord = o.completion_scores(leads, orders, N, 0, 200, 2)
    assert best >= (N + p - 1) * (tf + tb) - 0 and scores[0] >= best


def test_jitter_finds_shorter_schedules_on_the_large_problem():
    o, r, leads, orders = best_window(W.config5(), 300)
    scores, best, best_ord = o.completion_scores(leads, orders, 32, 0, 300, 2)
    assert best < scores[0] and best_ord > 0
