"""Pins of the oracle's whole-search routine (Alg. 1, Sec. IV-C) against facts that do not come
from it: closed forms of the sequential pipeline (Sec. VI ablation: no bubble once the window
holds as many micro-batches as there are stages and the memory allows them), the hand-checked
2-device golden row, a re-derivation from the separately pinned per-window argmin with exact
fractions, and monotonicity in the memory cap."""
from fractions import Fraction

import pytest

from oracle import oracle as O
from paper_2311_15269_amd import workloads as W


def linear(p, tf, tb, M, space="canonical"):
    return W.pipeline_problem(W.linear_placement(p), [tf] * p, [tb] * p, p, 1, M, space)


def per_window_argmin(problem, max_nr, max_candidates, use_bound=True):
    """Alg. 1 re-derived from Oracle.sweep (pinned elsewhere): per window size the lowest index of
    the least period; window sizes compared as exact fractions; stop after the first size that
    meets the bound."""
    lb = O.Oracle(dict(problem, NR=1)).lower_bound
    limit = min(max_nr, O.Oracle(dict(problem, NR=1)).max_inflight()) if use_bound else max_nr
    best = None
    rows = []
    for nr in range(1, limit + 1):
        o = O.Oracle(dict(problem, NR=nr))
        r = o.sweep(0, min(o.count, max_candidates), threads=4)
        rows.append((r["period"], r["index"]))
        if r["period"] > 0 and (best is None or Fraction(r["period"], nr) < Fraction(best[1], best[0])):
            best = (nr, r["period"], r["index"])
        if r["period"] == nr * lb:
            return best, rows, True
    return best, rows, False


@pytest.mark.parametrize("p,tf,tb", [(2, 1, 2), (3, 1, 2), (2, 2, 3), (3, 2, 3)])
def test_sequential_pipeline_reaches_the_bound_at_nr_equal_stages(p, tf, tb):
    """1F1B: with M = p the p-stage pipeline has a bubble-free window of p micro-batches
    (T* = p (tf + tb)) and none smaller: fewer micro-batches in the window cannot keep the
    first stage busy across the round trip of p (tf + tb)."""
    r = O.search(linear(p, tf, tb, p), 8, 1 << 40)
    assert r["inflights"] == p and r["lower_bound"] == tf + tb
    assert r["early_exit"] and r["best_nr"] == p and r["best_period"] == p * (tf + tb)
    assert r["nr_tried"] == p
    # every smaller window only reaches the round trip time of one micro-batch: p (tf + tb)
    assert r["period_nr"][:p - 1] == [p * (tf + tb)] * (p - 1)


def test_single_device_is_optimal_serially():
    prob = W.pipeline_problem([0], [3], [5], 1, 1, 1, "canonical")
    r = O.search(prob, 4, 1 << 20)
    assert r["early_exit"] and r["best_nr"] == 1 and r["best_period"] == 8 and r["best_index"] == 0
    assert r["evaluated_nr"] == [1]


def test_two_device_golden_row():
    """Config 1 by hand: T* = 6 = 2 * LB at N_R = 2; the serial window of N_R = 1 takes 6 per micro-batch."""
    r = O.search(W.config1(), 2, 1 << 20)
    assert r["period_nr"] == [6, 6] and r["best_nr"] == 2 and r["lower_bound"] == 3 and r["early_exit"]
    o = O.Oracle(W.config1())
    assert o.sweep(0, o.count)["index"] == r["best_index"]


@pytest.mark.parametrize("name,problem,max_nr,budget,bound", [
    ("cfg1", W.config1(), 4, 1 << 30, True),
    ("3dev", linear(3, 1, 2, 3), 4, 1 << 30, True),
    ("3dev-tight", linear(3, 1, 2, 2), 4, 1 << 30, True),
    ("3dev-tight-unbounded", linear(3, 1, 2, 2), 3, 1 << 30, False),
    ("cfg3-sampled", W.config3(), 4, 3000, True),
    ("cfg4-sampled-tp", dict(W.config4(), M=9), 3, 1500, True),
    ("cfg5-sampled", W.config5(), 3, 300, True),
])
def test_search_equals_per_window_argmin(name, problem, max_nr, budget, bound):
    r = O.search(problem, max_nr, budget, use_inflight_bound=bound)
    best, rows, early = per_window_argmin(problem, max_nr, budget, bound)
    assert r["early_exit"] == early
    assert r["nr_tried"] == len(rows)
    got_rows = [(pr if pr >= 0 else -1, ix if pr >= 0 else 0) for pr, ix in zip(r["period_nr"], r["index_nr"])]
    want_rows = [(pr if pr > 0 else -1, ix if pr > 0 else 0) for pr, ix in rows]
    if early:      # the last window stops at the first candidate that meets the bound: same period, same index
        assert got_rows[-1] == want_rows[-1]
    assert got_rows == want_rows
    if best is None:
        assert r["best_nr"] == 0 and r["best_period"] == -1
    else:
        assert (r["best_nr"], r["best_period"], r["best_index"]) == best


def test_early_exit_stops_at_the_first_candidate_that_meets_the_bound():
    r = O.search(W.config1(), 2, 1 << 20)
    assert r["evaluated_nr"][1] == r["best_index"] + 1


def test_best_time_per_microbatch_never_grows_with_the_cap():
    prev = None
    for M in (1, 2, 3, 4):
        r = O.search(linear(3, 1, 2, M), 4, 1 << 30)
        assert r["inflights"] == min(M, 16)
        cur = Fraction(r["best_period"], r["best_nr"])
        assert prev is None or cur <= prev
        prev = cur
    assert prev == 3      # M >= 3: the bound


def test_inflight_bound_of_the_benchmark_problems():
    # folded placements hold two activations per micro-batch on a device at most
    assert O.Oracle(W.config2()).max_inflight() == 4
    assert O.Oracle(W.config3()).max_inflight() == 3
    assert O.Oracle(W.config5()).max_inflight() == 5
    # the tensor-parallel embedding (+2) and a stage (+1) share every device of config 4
    assert O.Oracle(W.config4()).max_inflight() == 2


@pytest.mark.parametrize("p,tf,tb", [(2, 1, 2), (2, 1, 3), (3, 1, 2), (3, 1, 3)])
def test_bubble_rate_against_window_size_without_memory_limit(p, tf, tb):
    """Sec. VI-C, bubble rate and N_R for the sequential placement: a window of N_R micro-batches
    keeps at most N_R of them in flight, one round trip takes p (tf + tb), so
    T*(N_R) = max(N_R (tf + tb), p (tf + tb)): the bubble 1 - N_R/p vanishes first at N_R = p."""
    prob = W.pipeline_problem(W.linear_placement(p), [tf] * p, [tb] * p, p, 1, 64, "canonical")
    r = O.search(prob, p + 1 if p < 3 else p, 1 << 40, use_inflight_bound=False)
    want = [max(nr, p) * (tf + tb) for nr in range(1, p + 1)]
    assert r["period_nr"][:p] == want
    assert r["best_nr"] == p and r["early_exit"]


def inference_pipeline(p, tf):
    """forward blocks only, nothing held (Sec. VI: schedules for inference drop the backward blocks)"""
    return {"name": "inference-%d" % p, "D": p, "K": p, "NR": 1, "M": 1, "t": [tf] * p, "m": [0] * p,
            "dev_mask": [1 << s for s in range(p)], "deps": [(s, s + 1) for s in range(p - 1)],
            "space": "canonical", "seed": 0, "lead_step_q16": 0}


@pytest.mark.parametrize("p", [2, 3, 4])
def test_inference_pipeline_needs_one_micro_batch_per_window(p):
    """Without backward blocks neighbouring windows overlap freely (negative W_R of Eq. 4): the window of one
    micro-batch already repeats every tf, the bound; memory does not limit the window size."""
    r = O.search(inference_pipeline(p, 2), 5, 1 << 20)
    assert r["inflights"] == 5
    assert (r["best_nr"], r["best_period"], r["best_index"], r["early_exit"]) == (1, 2, 0, True)
