"""Pins of the CPU oracle against things other than itself: brute force over start vectors,
closed forms (1F1B, GPipe), hand-verified 2-device schedules, invariants, an independent
Eq. 1 checker.  No GPU."""
import collections
import itertools
import os
import random

import numpy as np
import pytest

from oracle import Oracle
from oracle.oracle import OracleError, draw16
from paper_2311_15269_amd import workloads as W
from tests import schedule_checks as SC

OK, DUP, TP_MISMATCH, PROP2, DEADLOCK, MEM = range(6)
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def linear(p, tf, tb, nr, cap, space="sampled_strict", **kw):
    return W.pipeline_problem(W.linear_placement(p), [tf] * p, [tb] * p, p, nr, cap, space, **kw)


def one_f_one_b(p):
    """1F1B steady state on p linear stages as a window of N_R = p micro-batches: stage s
    alternates F, B and is p-1-s micro-batches ahead in its forward pass."""
    leads = [p - 1 - s for s in range(p)] + [0] * p
    orders = [[s, 2 * p - 1 - s] * p for s in range(p)]
    return leads, orders


def gpipe(p, nr):
    leads = [0] * (2 * p)
    orders = [[s] * nr + [2 * p - 1 - s] * nr for s in range(p)]
    return leads, orders


# ---------------------------------------------------------------- closed forms
@pytest.mark.parametrize("p", [2, 3, 4, 6, 9, 12, 16])             # windows of up to 16 micro-batches
@pytest.mark.parametrize("tf,tb", [(1, 2), (2, 3), (3, 3)])
def test_1f1b_period_is_device_busy_time(p, tf, tb):
    """Zero-bubble 1F1B (Table II; Sec. III-C): the steady-state period of N_R = p
    micro-batches is N_R * (tf + tb) and stage s keeps p - s micro-batches in flight."""
    orc = Oracle(linear(p, tf, tb, p, p))
    leads, orders = one_f_one_b(p)
    r = orc.eval_explicit(leads, orders, want_starts=True)
    assert r["status"] == OK
    assert r["period"] == p * (tf + tb) == orc.lower_bound
    assert r["peak"] == [p - s for s in range(p)]
    assert SC.check_periodic(orc.problem, leads, orders, r["starts"].tolist(), r["period"])
    assert not SC.check_periodic(orc.problem, leads, orders, r["starts"].tolist(), r["period"] - 1)


@pytest.mark.parametrize("p", [2, 3, 4])
@pytest.mark.parametrize("nr", [1, 2, 4, 5, 9, 13, 16])
@pytest.mark.parametrize("tf,tb", [(1, 2), (2, 3)])
def test_gpipe_window_period_is_gpipe_makespan(p, nr, tf, tb):
    """All forwards then all backwards on every device cannot overlap with the next window,
    so the period is the GPipe makespan (m + p - 1)(tf + tb) with m = N_R."""
    orc = Oracle(linear(p, tf, tb, nr, nr))
    leads, orders = gpipe(p, nr)
    r = orc.eval_explicit(leads, orders)
    assert r["status"] == OK
    assert r["period"] == (nr + p - 1) * (tf + tb)
    assert r["peak"] == [nr] * p


def test_1f1b_rejected_when_cap_below_pipeline_depth():
    p = 4
    orc = Oracle(linear(p, 1, 2, p, p - 1))
    leads, orders = one_f_one_b(p)
    r = orc.eval_explicit(leads, orders)
    assert r["status"] == MEM and r["peak_max"] == p


# ---------------------------------------------------------------- brute force on tiny inputs
def _tiny_cases():
    """Small problems (4..8 blocks per window).  Orders come half from plain shuffles (mostly
    deadlocked) and half from the repaired sampled space, so that runnable ones dominate."""
    rng = random.Random(20231115)
    cases = []
    for k in range(60):
        p = rng.choice([2, 2, 3])
        nr = rng.choice([1, 2]) if p == 2 else 1
        folded = rng.random() < 0.3 and p == 2 and nr == 1
        place = W.folded_placement(p) if folded else W.linear_placement(p)
        S = len(place)
        tf = [rng.randint(1, 2) for _ in range(S)]
        tb = [rng.randint(1, 3) for _ in range(S)]
        prob = W.pipeline_problem(place, tf, tb, p, nr, 99, "sampled_repair", seed=k, lead_step_q16=40000)
        K = prob["K"]
        if k % 4 == 0:
            leads = [0] * K
            for i in reversed(range(K - 1)):
                leads[i] = min(nr - 1, leads[i + 1] + (rng.random() < 0.5))
            orders = []
            for d in range(p):
                seq = [g for g in range(K) if prob["dev_mask"][g] >> d & 1 for _ in range(nr)]
                rng.shuffle(seq)
                orders.append(seq)
        else:
            _, leads, orders = Oracle(prob).decode(rng.randrange(1 << 30))
        cases.append((prob, leads, orders))
    return cases


def test_period_equals_brute_force_over_start_vectors():
    """T* is the smallest T for which *some* integer start vector makes the repeated window a
    valid schedule.  Enumerate T upward and start vectors in a box, literally."""
    checked = 0
    for prob, leads, orders in _tiny_cases():
        orc = Oracle(prob)
        r = orc.eval_explicit(leads, orders, want_starts=True)
        box = orc.upper_bound
        if r["status"] == DEADLOCK:
            # no period works, not even the serial one (much larger box would not help either:
            # a lag-0 cycle is independent of T)
            assert not SC.exists_periodic_schedule(prob, leads, orders, 2 * orc.upper_bound, box)
            continue
        assert r["status"] == OK
        T = r["period"]
        assert orc.lower_bound <= T <= orc.upper_bound
        assert SC.check_periodic(prob, leads, orders, r["starts"].tolist(), T)
        assert SC.exists_periodic_schedule(prob, leads, orders, T, box)
        if T > 1:
            assert not SC.exists_periodic_schedule(prob, leads, orders, T - 1, box)
        checked += 1
    assert checked >= 30


def test_feasibility_is_monotone_in_period():
    prob = W.config1()
    orc = Oracle(prob)
    leads, orders = [1, 0, 0, 0], [[0, 3, 0, 3], [1, 2, 1, 2]]
    flags = [orc.feasible_explicit(leads, orders, T) for T in range(1, 14)]
    assert flags == [0] * 5 + [1] * 8


# ---------------------------------------------------------------- config 1, by hand
def test_config1_hand_verified_rows():
    """Rows worked out on paper for the 2-device problem (tf=1, tb=2, cap 2, N_R=2); the
    derivations are in tests/golden/config1_hand.txt."""
    orc = Oracle(W.config1())
    rows = []
    with open(os.path.join(GOLDEN, "config1_hand.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                rows.append(line.split())
    assert len(rows) >= 5
    names = {"F0": 0, "F1": 1, "B1": 2, "B0": 3}
    for leads_s, d0, d1, status, period, peaks in rows:
        leads = [int(x) for x in leads_s.split(",")]
        orders = [[names[x] for x in d0.split(",")], [names[x] for x in d1.split(",")]]
        r = orc.eval_explicit(leads, orders, want_starts=True)
        assert r["status"] == ("OK", "DUP", "TP_MISMATCH", "PROP2", "DEADLOCK", "MEM").index(status), (leads, orders)
        if status == "OK":
            assert r["period"] == int(period)
        if status in ("OK", "MEM"):
            assert r["peak"] == [int(x) for x in peaks.split(",")]
    # the zero-bubble row also pins the least start times
    r = orc.eval_explicit([1, 0, 0, 0], [[0, 3, 0, 3], [1, 2, 1, 2]], want_starts=True)
    assert r["starts"].tolist() == [[2, 5], [0, 3], [1, 4], [3, 6]]


def test_config1_exhaustive_summary():
    orc = Oracle(W.config1())
    assert orc.count == 576 and orc.lower_bound == 6
    res = orc.sweep(0, 576)
    code, _ = orc.score_range(0, 576)
    hist = collections.Counter(code.tolist())
    assert res["n_evaluated"] == 576
    assert res["period"] == 6 == orc.lower_bound          # a zero-bubble repetend exists
    assert res["n_feasible"] == sum(v for k, v in hist.items() if k > 0)
    # the census of the whole space: 27 of the 576 candidates are feasible, 3 at the bound, 18 at period 9, 6 at 12
    # (worked out apart from this oracle when the problem was stated)
    assert res["n_feasible"] == 27
    assert {k: v for k, v in hist.items() if k > 0} == {6: 3, 9: 18, 12: 6}
    # 16 lead vectors x 36 interleavings, every label order cyclic when N_R = 2
    assert hist[-DUP] == 0 and hist[-TP_MISMATCH] == 0
    # lowest index wins among equal periods (Alg. 1 compares with strict <)
    assert res["index"] == min(i for i, c in enumerate(code.tolist()) if c == 6)
    # every feasible candidate: valid by the independent checker, invalid one period lower
    for idx in range(576):
        if code[idx] > 0:
            _, leads, orders = orc.decode(idx)
            r = orc.eval_index(idx, want_starts=True)
            assert SC.check_periodic(orc.problem, leads, orders, r["starts"].tolist(), r["period"])
            assert not SC.exists_periodic_schedule(orc.problem, leads, orders, r["period"] - 1, orc.upper_bound)
            assert max(r["peak"]) <= 2


def test_factorial_space_is_a_bijection_onto_lead_and_interleaving_pairs():
    orc = Oracle(W.config1())
    seen = set()
    for idx in range(576):
        st, leads, orders = orc.decode(idx)
        seen.add((tuple(leads), tuple(map(tuple, orders))))
    assert len(seen) == 576          # 2^4 lead vectors x C(4,2)^2 interleavings


def test_factorial_dup_detection_nr3():
    """With N_R = 3 a label order like 0,2,1 is not cyclic: a Property-1 duplicate."""
    prob = W.pipeline_problem([0], [1], [1], 1, 3, 9, "factorial")
    orc = Oracle(prob)
    assert orc.count == 720
    code, _ = orc.score_range(0, 720)
    hist = collections.Counter((c if c < 0 else 0) for c in code.tolist())
    # per type 3 cyclic label orders of 3! -> (3/6)^2 of all; interleavings C(6,3) = 20
    assert hist[-DUP] == 720 - 20 * 3 * 3
    assert 720 - hist[-DUP] == 180


# ---------------------------------------------------------------- invariants
def test_period_invariant_under_common_lead_shift_and_bounds():
    rng = random.Random(5)
    prob = W.pipeline_problem(W.folded_placement(3), [1, 2, 3, 1, 2, 3], [2, 2, 4, 3, 1, 5], 3, 4, 99, "sampled_repair",
                              seed=11, lead_step_q16=20000)
    orc = Oracle(prob)
    n_ok = 0
    for idx in range(300):
        st, leads, orders = orc.decode(idx)
        r = orc.eval_explicit(leads, orders)
        assert r["status"] == OK                      # repaired, no cap
        assert orc.lower_bound <= r["period"] <= orc.upper_bound
        room = prob["NR"] - 1 - max(leads)
        if room > 0:
            shifted = [x + room for x in leads]
            r2 = orc.eval_explicit(shifted, orders)
            assert r2["period"] == r["period"] and r2["peak"] == r["peak"]
            n_ok += 1
    assert n_ok > 50


def test_best_period_is_monotone_in_memory_cap():
    """Less memory can only make the best repetend slower (Sec. VI-C, memory ablation)."""
    best = []
    for cap in (1, 2, 3, 4):
        prob = W.config1()
        prob["M"] = cap
        res = Oracle(prob).sweep(0, 576)
        best.append(res["period"] if res["n_feasible"] else 10 ** 9)
    assert best == sorted(best, reverse=True)
    assert best[1] == 6


def test_linear_placement_needs_nr_equal_devices_for_zero_bubble():
    """Sec. VI-C: the sequential placement reaches zero bubble only from N_R = #devices on."""
    p = 3
    for nr, expect_zero in ((1, False), (2, False), (3, True)):
        prob = W.pipeline_problem(W.linear_placement(p), [1] * p, [2] * p, p, nr, 99, "canonical")
        orc = Oracle(prob)
        res = orc.sweep(0, orc.count)
        assert (res["period"] == orc.lower_bound) == expect_zero, (nr, res)


# ---------------------------------------------------------------- spaces and sampler
def test_canonical_count_config2():
    orc = Oracle(W.config2())
    assert orc.num_lead_vectors == 120            # non-increasing 8-sequences over {0..3} ending in 0
    assert orc.count == 120 * 70 ** 4
    # the 1F1B candidate is in the space and reaches the lower bound with peaks [4,3,2,1]
    leads, orders = one_f_one_b(4)
    r = orc.eval_explicit(leads, orders)
    assert (r["status"], r["period"], r["peak"]) == (OK, 12, [4, 3, 2, 1])


def test_canonical_space_enumerates_distinct_candidates():
    prob = W.pipeline_problem(W.linear_placement(2), [1, 1], [2, 2], 2, 2, 2, "canonical")
    orc = Oracle(prob)
    assert orc.count == 4 * 36                    # leads (a,b,c,0) non-increasing over {0,1}: 000,100,110,111
    seen = set()
    for idx in range(orc.count):
        st, leads, orders = orc.decode(idx)
        assert st == OK and min(leads) == 0
        assert all(leads[a] >= leads[b] for a, b in prob["deps"])
        seen.add((tuple(leads), tuple(map(tuple, orders))))
    assert len(seen) == orc.count


def test_canonical_and_factorial_agree_on_config1():
    """Every canonical candidate is a FACTORIAL candidate with the same score."""
    fac = Oracle(W.config1())
    prob = W.config1()
    prob["space"] = "canonical"
    can = Oracle(prob)
    by_key = {}
    for idx in range(576):
        st, leads, orders = fac.decode(idx)
        code = fac.score_range(idx, 1)[0][0]
        by_key[(tuple(leads), tuple(map(tuple, orders)))] = code
    for idx in range(can.count):
        st, leads, orders = can.decode(idx)
        code = can.score_range(idx, 1)[0][0]
        assert by_key[(tuple(leads), tuple(map(tuple, orders)))] == code


def test_sampler_digits_look_uniform_and_depend_on_every_input():
    n = 20000
    draws = np.array([draw16(123, o, 128 + 5) for o in range(n)])
    hist = np.bincount((draws * 16) >> 16, minlength=16)
    chi2 = float(((hist - n / 16) ** 2 / (n / 16)).sum())
    assert chi2 < 50                                   # 15 dof, p ~ 1e-5
    assert draw16(1, 2, 3) != draw16(2, 2, 3) or draw16(1, 2, 4) != draw16(2, 2, 4)
    assert len({draw16(9, o, j) for o in range(50) for j in range(50)}) > 2300
    # adjacent halves of one word are different draws
    assert [draw16(7, 7, j) for j in range(8)] != [draw16(7, 7, j ^ 1) for j in range(8)]


def test_sampled_orders_are_uniform_over_types():
    prob = W.config3("sampled_strict")
    orc = Oracle(prob)
    first = collections.Counter()
    for idx in range(4000):
        _, leads, orders = orc.decode(idx)
        for d, seq in enumerate(orders):
            assert sorted(seq) == sorted(g for g in range(16) if prob["dev_mask"][g] >> d & 1 for _ in range(4))
        first[orders[0][0]] += 1
        assert all(leads[a] >= leads[b] for a, b in prob["deps"]) and max(leads) <= 3 and leads[-1] == 0
    assert all(800 < v < 1200 for v in first.values()) and len(first) == 4


# ---------------------------------------------------------------- repair convention
def test_repair_keeps_valid_orders_and_always_yields_runnable_ones():
    prob = W.config3("sampled_repair")
    strict = dict(prob, space="sampled_strict")
    rep, stc = Oracle(prob), Oracle(strict)
    unchanged = 0
    for idx in range(1500):
        _, leads_r, orders_r = rep.decode(idx)
        _, leads_s, orders_s = stc.decode(idx)
        assert leads_r == leads_s
        for a, b in zip(orders_r, orders_s):
            assert sorted(a) == sorted(b)
        r = rep.eval_index(idx)
        assert r["status"] in (OK, MEM)
        s = stc.eval_index(idx)
        if s["status"] != DEADLOCK:
            assert orders_r == orders_s and (s["status"], s["period"]) == (r["status"], r["period"])
            unchanged += 1
    # a runnable order handed to the repair comes back as it was
    p = 4
    prob = linear(p, 1, 2, p, p, space="sampled_repair", fixed_leads=one_f_one_b(p)[0])
    orc = Oracle(prob)
    r = orc.eval_explicit(*one_f_one_b(p))
    assert r["period"] == 12


# ---------------------------------------------------------------- completion
@pytest.mark.parametrize("p,N", [(2, 6), (4, 16), (4, 17), (3, 10)])
def test_completion_of_1f1b_reaches_textbook_makespan(p, N):
    """1F1B on uniform stages finishes N micro-batches in (N + p - 1)(tf + tb)."""
    tf, tb = 1, 2
    prob = linear(p, tf, tb, p, p)
    orc = Oracle(prob)
    leads, orders = one_f_one_b(p)
    out = orc.complete(leads, orders, N)
    ok, makespan, peaks = SC.check_flat_schedule(prob, N, out["start"].tolist(), out["dev_order"])
    assert ok and makespan == out["makespan"]
    assert makespan == (N + p - 1) * (tf + tb)
    assert max(peaks) <= p


@pytest.mark.parametrize("prob", [W.config3(), dict(W.config4(), M=12), W.kshape_problem(3, 5), W.diamond_problem(2, 4)],
                         ids=["folded", "shared-block", "k-shape", "diamond"])
def test_completion_is_valid_on_sampled_candidates(prob):
    orc = Oracle(prob)
    done = 0
    for idx in range(400):
        r = orc.eval_index(idx)
        if r["status"] != OK:
            continue
        _, leads, orders = orc.decode(idx)
        for N in (8, 13):
            out = orc.complete(leads, orders, N)
            ok, makespan, peaks = SC.check_flat_schedule(prob, N, out["start"].tolist(), out["dev_order"])
            assert ok and makespan == out["makespan"] and max(peaks) <= prob["M"]
            # the steady part cannot beat its own period
            R = (N - max(leads)) // prob["NR"]
            assert makespan >= R * r["period"] - 0 if R > 1 else True
        done += 1
        if done >= 25:
            break
    assert done >= 5


def test_lead_law_at_its_deterministic_ends():
    """The leads of a sampled candidate: consumers before producers, a type's lead is the largest (consumer's lead +
    step) over its dependencies, capped at N_R - 1; the step is drawn only where the two blocks sit on different
    device sets.  With the probability of a step at 1 or at 0 no draw matters and the vector can be written down."""
    lin = W.pipeline_problem(W.linear_placement(3), [1] * 3, [2] * 3, 3, 4, 4, "sampled_repair", seed=5, lead_step_q16=65536)
    cases = [
        (lin, [3, 3, 2, 2, 1, 0]),                          # F0 F1 F2 B2 B1 B0: no step between F2 and B2 (same device), cap 3
        (dict(lin, NR=2), [1, 1, 1, 1, 1, 0]),
        (dict(lin, lead_step_q16=0), [0] * 6),
        (W.kshape_problem(4, 8, lead_step_q16=65536), [2, 2, 1, 1, 0, 0]),           # A_F B_F J_F J_B A_B B_B
        (W.diamond_problem(8, 16, lead_step_q16=65536), [4, 3, 3, 2, 2, 1, 1, 0]),   # S_F L_F R_F T_F T_B L_B R_B S_B
        (W.diamond_problem(3, 6, lead_step_q16=65536), [2, 2, 2, 2, 2, 1, 1, 0]),
        # a block on all devices at both ends of the chain: a step wherever the device sets differ
        (dict(W.config4(), lead_step_q16=65536), [3, 3, 3, 3, 3, 3, 3, 2, 1, 0]),
    ]
    for prob, want in cases:
        orc = Oracle(prob)
        for index in (0, 1, 12345, 1 << 40):
            status, leads, orders = orc.decode(index)
            assert leads == want, (prob["name"], index, leads)


def test_greedy_completion_matches_the_worked_example():
    """The tie order of the greedy rule (earliest start, then micro-batch, then type id), worked out by hand on one
    device, where every offered block can start when the device is free and only the tie order decides:
    types A, B, C (t = 1, 2, 3; no memory, no dependencies), N_R = 3, leads 2, 1, 0, window order AAA BBB CCC,
    N = 5 micro-batches, so one window between warm-up and cool-down.
    Warm-up (micro-batches below the leads: A0, A1, B0), all free to start at 0: A0 (micro-batch 0, type 0) before
    B0 (micro-batch 0, type 1); then B0 before A1 (micro-batch before type): A0 at 0, B0 at 1, A1 at 3.
    Window, back to back from 4: A2 A3 A4 at 4, 5, 6; B1 B2 B3 at 7, 9, 11; C0 C1 C2 at 13, 16, 19 (ends 22).
    Cool-down (B4, C3, C4): C3 (micro-batch 3) before B4 (micro-batch 4) at 22; then B4 before C4 (type) at 25;
    C4 at 27; the device never idles: makespan 30 = 5 (1 + 2 + 3)."""
    prob = {"name": "one-device", "D": 1, "K": 3, "NR": 3, "M": 0, "t": [1, 2, 3], "m": [0, 0, 0], "dev_mask": [1, 1, 1],
            "deps": [], "space": "sampled_repair", "seed": 1, "lead_step_q16": 0, "fixed_leads": None}
    leads, orders = [2, 1, 0], [[0, 0, 0, 1, 1, 1, 2, 2, 2]]
    orc = Oracle(prob)
    assert orc.eval_explicit(leads, orders)["status"] == OK
    c = orc.complete(leads, orders, 5)
    assert c["makespan"] == 30
    assert c["start"].tolist() == [[0, 3, 4, 5, 6], [1, 7, 9, 11, 25], [13, 16, 19, 22, 27]]
    ok, makespan, peaks = SC.check_flat_schedule(prob, 5, c["start"].tolist(), c["dev_order"])
    assert ok and makespan == 30


def test_error_paths():
    base = W.config1()
    with pytest.raises(OracleError):
        Oracle(dict(base, m=[1, 1, -1, 0]))                       # memory never returns to its level
    with pytest.raises(OracleError):
        Oracle(dict(base, deps=[(0, 1), (1, 0)]))                 # cyclic micro-batch graph
    with pytest.raises(OracleError):
        Oracle(dict(base, t=[0, 1, 2, 2]))
    with pytest.raises(OracleError):
        Oracle(W.pipeline_problem(W.folded_placement(8), [1] * 16, [1] * 16, 8, 8, 10, "canonical"))  # > 2^64


def _golden_lines(name, tag):
    path = os.path.join(os.path.dirname(__file__), "golden", name)
    return [ln[len(tag):].strip() for ln in open(path) if ln.startswith(tag)]


def test_sampler_matches_the_worked_example():
    """orc_draw16 against tests/golden/sampler_hand.txt: key mixing anchored on the published first output of
    SplitMix64 seeded with 0, every 32-bit step of the word hash written out."""
    from oracle.oracle import draw16
    rows = _golden_lines("sampler_hand.txt", "draw ")
    assert len(rows) == 6
    for row in rows:
        seed, ordinal, j, want = (int(x) for x in row.split())
        assert draw16(seed, ordinal, j) == want, row


def test_repair_matches_the_worked_examples():
    """The repair rule against tests/golden/repair_hand.txt, derived step by step there: the fallback goes to the
    lowest device that has a runnable block and takes the earliest such entry of its list; runnable lists stay."""
    orc = Oracle(dict(W.config1(), space="sampled_repair"))
    rows = _golden_lines("repair_hand.txt", "case ")
    assert len(rows) == 3
    for row in rows:
        leads, d0, d1, want0, want1 = ([int(x) for x in part.split()] for part in row.split("|"))
        assert orc.repair_explicit(leads, [d0, d1]) == [want0, want1], row
        # the repaired orders are executable and handle the same blocks
        assert orc.eval_explicit(leads, [want0, want1])["status"] in (OK, MEM)
        assert sorted(d0) == sorted(want0) and sorted(d1) == sorted(want1)


def test_repair_on_branching_graphs_and_shared_blocks_matches_the_worked_examples():
    """Examples 4-6 of tests/golden/repair_hand.txt: a block with two producers waits for both, the K-shape, a block
    on both devices placed by the fallback leaves both lists."""
    rows = _golden_lines("repair_hand.txt", "graph ")
    assert len(rows) == 3
    for row in rows:
        head, masks, deps, lists, want = (part.strip() for part in row.split("|"))
        D, K = (int(x) for x in head.split())
        prob = {"name": "repair-hand", "D": D, "K": K, "NR": 1, "M": 99, "t": [1] * K, "m": [0] * K,
                "dev_mask": [int(x) for x in masks.split()], "deps": [tuple(int(x) for x in e.split(">")) for e in deps.split()],
                "space": "sampled_repair", "seed": 1, "lead_step_q16": 0, "fixed_leads": None}
        orders = [[int(x) for x in part.split()] for part in lists.split(";")]
        wanted = [[int(x) for x in part.split()] for part in want.split(";")]
        orc = Oracle(prob)
        assert orc.repair_explicit([0] * K, orders) == wanted, row
        assert orc.eval_explicit([0] * K, wanted)["status"] == OK
        assert orc.eval_explicit([0] * K, orders)["status"] == DEADLOCK


def test_a_block_on_two_devices_with_two_leads_is_a_mismatch():
    """FACTORIAL space, one block type on both of two devices, windows of two micro-batches: each device orders
    the labelled blocks (0, 1); rank 0 = (0, 1) names lead 0, rank 1 = (1, 0) names lead 1.  Index = r_0 + 2 r_1:
    indices 1 and 2 give the block different leads on its two devices (TP_MISMATCH); 0 and 3 are the same schedule,
    both micro-batches one after the other: period 2 t."""
    prob = {"name": "tp-hand", "D": 2, "K": 1, "NR": 2, "M": 0, "t": [3], "m": [0], "dev_mask": [3], "deps": [],
            "space": "factorial", "seed": 0, "lead_step_q16": 0, "fixed_leads": None}
    orc = Oracle(prob)
    assert orc.count == 4
    got = [orc.eval_index(i) for i in range(4)]
    assert [g["status"] for g in got] == [OK, TP_MISMATCH, TP_MISMATCH, OK]
    assert got[0]["period"] == got[3]["period"] == 6


# ---------------------------------------------------------------- dependency graphs with fan-in and fan-out
def _tiny_graph_cases():
    """A block type with two producers (two branches that join) and with two consumers, on 2-3 devices, 4-6 blocks
    per window, small times: orders half from plain shuffles, half from the repaired sampled space."""
    rng = random.Random(20231116)
    shapes = [
        # A(0), B(1) -> J(2): fan-in only
        dict(D=3, K=3, dev_mask=[1, 2, 4], deps=[(0, 2), (1, 2)], m=[0, 0, 0]),
        # S(0) -> L(1), R(0): fan-out, then both into T(1): a diamond on two devices
        dict(D=2, K=4, dev_mask=[1, 2, 1, 2], deps=[(0, 1), (0, 2), (1, 3), (2, 3)], m=[1, 1, -1, -1]),
        # the K-shape, forward and backward: A_F(0), B_F(1) -> J_F(2) -> J_B(2) -> A_B(0), B_B(1)
        dict(D=3, K=6, dev_mask=[1, 2, 4, 4, 1, 2], deps=[(0, 2), (1, 2), (2, 3), (3, 4), (3, 5)], m=[1, 1, 1, -1, -1, -1]),
    ]
    cases = []
    for k in range(48):
        shape = shapes[k % 3]
        nr = 2 if shape["K"] <= 3 and k % 2 else 1
        K, D = shape["K"], shape["D"]
        prob = dict(shape, name="tiny-graph", NR=nr, M=99, t=[rng.randint(1, 3) for _ in range(K)], space="sampled_repair",
                    seed=k, lead_step_q16=40000, fixed_leads=None)
        if k % 4 == 0:
            leads = [0] * K
            if nr > 1:                                    # producers never behind their consumers (Property 2)
                for i in reversed(range(K)):
                    succ = [b for a, b in prob["deps"] if a == i]
                    if succ:
                        leads[i] = min(nr - 1, max(leads[b] for b in succ) + (rng.random() < 0.5))
            orders = []
            for d in range(D):
                seq = [g for g in range(K) if prob["dev_mask"][g] >> d & 1 for _ in range(nr)]
                rng.shuffle(seq)
                orders.append(seq)
        else:
            _, leads, orders = Oracle(prob).decode(rng.randrange(1 << 30))
        cases.append((prob, leads, orders))
    return cases


def test_period_of_graphs_with_fan_in_and_fan_out_equals_brute_force():
    """Sec. III-A allows any acyclic dependency graph inside a micro-batch (Eq. 1 [3] for every edge).  The same brute
    force over start vectors as above, on windows whose graph branches: a block waits for all its producers."""
    checked = deadlocked = 0
    for prob, leads, orders in _tiny_graph_cases():
        orc = Oracle(prob)
        r = orc.eval_explicit(leads, orders, want_starts=True)
        box = orc.upper_bound
        if r["status"] == DEADLOCK:
            assert not SC.exists_periodic_schedule(prob, leads, orders, 2 * orc.upper_bound, box)
            deadlocked += 1
            continue
        assert r["status"] == OK
        T = r["period"]
        assert orc.lower_bound <= T <= orc.upper_bound
        assert SC.check_periodic(prob, leads, orders, r["starts"].tolist(), T)
        assert SC.exists_periodic_schedule(prob, leads, orders, T, box)
        if T > 1:
            assert not SC.exists_periodic_schedule(prob, leads, orders, T - 1, box)
        checked += 1
    assert checked >= 25 and deadlocked >= 1


def test_one_micro_batch_of_the_k_shape_takes_its_critical_path():
    """One micro-batch per window (all leads 0): a device can only run its forward block before its backward block,
    and the next window's forward block follows this window's backward block on the same device, so the cycles of
    the constraint graph are, per branch device, forward + joint forward + joint backward + backward, and the joint
    device's own two blocks: T* = t_J + t_J' + max(t_A + t_A', t_B + t_B'); every other order deadlocks."""
    for tf, tb in (((2, 1, 3), (4, 2, 6)), ((1, 5, 2), (3, 1, 1)), ((4, 4, 1), (1, 2, 2)), ((1, 1, 7), (1, 1, 1))):
        prob = W.kshape_problem(1, 99, tf=tf, tb=tb, space="canonical")
        orc = Oracle(prob)
        assert orc.count == 8                              # two orders on each of the three devices
        best = orc.sweep(0, orc.count)
        assert best["n_feasible"] == 1 and best["n_reject"][DEADLOCK] == 7
        assert best["period"] == tf[2] + tb[2] + max(tf[0] + tb[0], tf[1] + tb[1])
        assert best["peak"] == [1, 1, 1]


def _tiny_shared_block_cases():
    """windows with a block that occupies both devices (tensor parallelism: it takes part in both device orders
    and needs both devices at once), 3-6 blocks per window"""
    rng = random.Random(20231117)
    shapes = [
        # X on both devices feeds A(0) and B(1)
        dict(D=2, K=3, dev_mask=[3, 1, 2], deps=[(0, 1), (0, 2)], m=[0, 0, 0]),
        # A(0), B(1) -> X on both -> Y(0)
        dict(D=2, K=4, dev_mask=[1, 2, 3, 1], deps=[(0, 2), (1, 2), (2, 3)], m=[0, 0, 0, 0]),
        # a chain X(both) -> A(0) -> B(1) -> X'(both), the shape of the 4-device benchmark configuration in small
        dict(D=2, K=4, dev_mask=[3, 1, 2, 3], deps=[(0, 1), (1, 2), (2, 3)], m=[1, 0, 0, -1]),
    ]
    cases = []
    for k in range(45):
        shape = shapes[k % 3]
        nr = 2 if shape["K"] == 3 and k % 2 else 1
        K, D = shape["K"], shape["D"]
        prob = dict(shape, name="tiny-shared", NR=nr, M=99, t=[rng.randint(1, 3) for _ in range(K)], space="sampled_repair",
                    seed=k, lead_step_q16=40000, fixed_leads=None)
        if k % 3 == 0:
            leads = [0] * K
            orders = []
            for d in range(D):
                seq = [g for g in range(K) if prob["dev_mask"][g] >> d & 1 for _ in range(nr)]
                rng.shuffle(seq)
                orders.append(seq)
        else:
            _, leads, orders = Oracle(prob).decode(rng.randrange(1 << 30))
        cases.append((prob, leads, orders))
    return cases


def test_period_with_a_block_on_two_devices_equals_brute_force():
    """A block that occupies several devices (d_B is a set, Sec. III-A) holds all of them for its time: exclusivity
    (Eq. 1 [1]) on every one of its devices.  Brute force over start vectors as above."""
    checked = deadlocked = 0
    for prob, leads, orders in _tiny_shared_block_cases():
        orc = Oracle(prob)
        r = orc.eval_explicit(leads, orders, want_starts=True)
        box = orc.upper_bound
        if r["status"] == DEADLOCK:
            assert not SC.exists_periodic_schedule(prob, leads, orders, 2 * orc.upper_bound, box)
            deadlocked += 1
            continue
        assert r["status"] == OK
        T = r["period"]
        assert orc.lower_bound <= T <= orc.upper_bound
        assert SC.check_periodic(prob, leads, orders, r["starts"].tolist(), T)
        assert SC.exists_periodic_schedule(prob, leads, orders, T, box)
        if T > 1:
            assert not SC.exists_periodic_schedule(prob, leads, orders, T - 1, box)
        checked += 1
    assert checked >= 25 and deadlocked >= 1


def test_peak_memory_is_the_running_sum_of_eq_1_on_the_expanded_schedule():
    """Eq. 1 [2] literally: repeat the window many times at its period, take every micro-batch whose blocks all lie
    inside the expansion, sort each device's blocks by start time and accumulate m.  Once the pipeline is full the
    largest value over a window is the peak the oracle reports (entry memory from the leads + prefix in device order)."""
    rng = random.Random(424242)
    checked = 0
    probs = [W.config1(), W.config3(), dict(W.config4(), M=99), W.kshape_problem(3, 99), W.diamond_problem(2, 99),
             W.pipeline_problem(W.folded_placement(3), [1, 2, 1, 1, 3, 2], [2, 2, 1, 3, 1, 2], 3, 3, 99, "sampled_repair",
                                seed=5, lead_step_q16=30000)]
    for prob in probs:
        prob = dict(prob, space="sampled_repair", M=99)
        orc = Oracle(prob)
        K, NR, D = prob["K"], prob["NR"], prob["D"]
        for _ in range(6):
            index = rng.randrange(1 << 40)
            status, leads, orders = orc.decode(index)
            r = orc.eval_explicit(leads, orders, want_starts=True)
            assert r["status"] == OK
            T, windows = r["period"], 8
            blocks = SC.expand_periodic(prob, leads, orders, r["starts"].tolist(), T, windows)
            lo, hi = max(leads), NR * windows + min(leads)             # micro-batches with every block inside
            per_dev = [[] for _ in range(D)]
            for (i, mu), s in blocks.items():
                if lo <= mu < hi:
                    for d in SC.devices_of(prob, i):
                        per_dev[d].append((s, prob["m"][i]))
            for d in range(D):
                cur, peak = 0, None
                for s, m in sorted(per_dev[d]):
                    cur += m
                    if 3 * T <= s < 5 * T:                               # two windows in the steady state
                        peak = cur if peak is None else max(peak, cur)
                want = r["peak"][d]
                assert (peak if peak is not None else 0) == want, (prob["name"], index, d, peak, want)
            checked += 1
    assert checked == 36
