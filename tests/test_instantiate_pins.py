"""Pins of the oracle's runtime instantiation (Sec. IV-D: one global sequence of blocks and send/receive
pairs) against a sequence written out by hand and against the properties the section asks for, checked
by code that shares nothing with the oracle (tests/schedule_checks.py)."""
import os

import numpy as np
import pytest

from oracle import oracle as O
from paper_2311_15269_amd import workloads as W
from tests import schedule_checks as SC

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_hand_written_sequence():
    want = [tuple(int(v) for v in line.split()) for line in open(os.path.join(GOLDEN, "instantiate_hand.txt"))
            if line.strip() and not line.startswith("#")]
    prob = W.config1()
    N = 2
    start = [[0, 1], [1, 4], [2, 5], [4, 7]]
    dev_order = [[0, 1, 6, 7], [2, 4, 3, 5]]
    ok, _, _ = SC.check_flat_schedule(dict(prob, M=2), N, start, dev_order)
    assert ok
    got = O.Oracle(prob).instantiate(N, start, dev_order)
    assert got == want
    assert SC.check_instantiation(prob, N, start, got) == (True, "")


def _best_schedule(prob, budget, N):
    o = O.Oracle(prob)
    r = o.sweep(0, min(o.count, budget), threads=4)
    assert r["period"] > 0
    status, leads, orders = o.decode(r["index"])
    return o, o.complete(leads, orders, N)


@pytest.mark.parametrize("name,prob,budget,N", [
    ("cfg1", W.config1(), 576, 7),
    ("cfg3", W.config3(), 2000, 14),
    ("cfg4-tp", dict(W.config4(), M=9), 3000, 13),
    ("cfg5", W.config5(), 300, 20),
    ("lin3", W.pipeline_problem(W.linear_placement(3), [1, 2, 1], [2, 3, 1], 3, 3, 3, "canonical"), 1 << 30, 10),
])
def test_sequences_of_completed_schedules_have_the_required_properties(name, prob, budget, N):
    o, sched = _best_schedule(prob, budget, N)
    ops = o.instantiate(N, sched["start"], sched["dev_order"])
    ok, why = SC.check_instantiation(prob, N, sched["start"].tolist(), ops)
    assert ok, (name, why)
    # pairs sit right after the time slot of their producer: no block that starts later precedes them
    start = sched["start"]
    last_block_start = -1
    for kind, blk, src, dst, aux in ops:
        if kind == 0:
            last_block_start = dst
        else:
            assert start[blk // N][blk % N] == last_block_start


def test_the_checker_rejects_a_swapped_pair_order():
    """Two devices exchange tensors in both directions; receiving before sending on both sides deadlocks."""
    prob = W.config1()
    N = 2
    start = [[0, 1], [1, 4], [2, 5], [4, 7]]
    dev_order = [[0, 1, 6, 7], [2, 4, 3, 5]]
    ops = O.Oracle(prob).instantiate(N, start, dev_order)
    assert SC.check_instantiation(prob, N, start, ops)[0]
    bad = list(ops)
    k = next(i for i, o in enumerate(bad) if o[0] == 1)
    del bad[k]
    assert SC.check_instantiation(prob, N, start, bad) == (False, "missing pairs")
    # a pair moved behind its consumer
    bad = list(ops)
    pair = bad.pop(k)
    bad.append(pair)
    assert not SC.check_instantiation(prob, N, start, bad)[0]


# ---- the library's host-side tessel_instantiate against the oracle (no GPU involved) ----------------
@pytest.mark.parametrize("name,prob,budget,N", [
    ("cfg1", W.config1(), 576, 7),
    ("cfg3", W.config3(), 2000, 14),
    ("cfg4-tp", dict(W.config4(), M=9), 3000, 13),
    ("cfg5", W.config5(), 300, 20),
])
def test_library_sequence_equals_the_oracle(name, prob, budget, N):
    from paper_2311_15269_amd import binding
    o, sched = _best_schedule(prob, budget, N)
    want = o.instantiate(N, sched["start"], sched["dev_order"])
    got = binding.Problem(prob).instantiate(N, sched["start"])
    assert got == want


def test_library_instantiate_reports_bad_arguments():
    import ctypes as C
    from paper_2311_15269_amd import binding
    lib = binding.load_library()
    p = binding.Problem(W.config1())
    start = np.array([0, 1, 1, 4, 2, 5, 4, -1], dtype=np.int32)          # one block without a start time
    s = binding.Schedule(2, 8, start.ctypes.data, None, None, 0, 0, 0)
    n = C.c_int32(0)
    assert lib.tessel_instantiate(p._h, C.byref(s), None, 0, C.byref(n)) == -1
    start[7] = 7
    assert lib.tessel_instantiate(p._h, C.byref(s), None, 0, C.byref(n)) == -8 and n.value == 12
    assert lib.tessel_instantiate(p._h, None, None, 0, C.byref(n)) == -1
