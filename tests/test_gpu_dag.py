"""Dependency graphs that are not chains (Sec. III-A, Eq. 1 [3]: any acyclic graph inside a micro-batch): a block type
with two producers (two branches that join, the K-shape of Sec. VI-A) and with two consumers (a diamond), HIP path
(the general kernel's path for graphs) against the oracle element by element; seeded random graphs; and the same
path forced onto chain problems against the oracle and against the chain path."""
import numpy as np
import pytest

from paper_2311_15269_amd import workloads as W
from tests import schedule_checks as SC

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: the HIP path has no CPU fallback")
    from paper_2311_15269_amd import binding
    binding.load_library()
    return binding


def _compare(gpu, prob, first, n):
    from oracle import Oracle
    orc, g = Oracle(prob), gpu.Problem(prob)
    if prob["space"] in ("factorial", "canonical"):
        assert g.candidate_count() == orc.count
        n = min(n, orc.count - first)
    code, peak = g.score_candidates(first, n)
    want_code, want_peak = orc.score_range(first, n)
    code, peak = code.cpu().numpy(), peak.cpu().numpy()
    bad = np.nonzero((code != want_code) | (peak != want_peak))[0]
    assert bad.size == 0, (prob["name"], prob["space"], int(first + bad[0]), int(code[bad[0]]), int(want_code[bad[0]]))
    g.eval_candidates(first, n)
    got, want = g.best(), orc.sweep(first, n)
    assert got["n_evaluated"] == n and got["n_feasible"] == want["n_feasible"] and got["n_reject"][1:] == want["n_reject"][1:]
    if want["n_feasible"]:
        assert (got["period"], got["index"], got["peak"]) == (want["period"], want["index"], want["peak"])
        cand = g.best_candidate()
        status, leads, orders = orc.decode(got["index"])
        assert cand["leads"] == leads and cand["orders"] == orders
        ref = orc.eval_index(got["index"], want_starts=True)
        assert (cand["starts"] == ref["starts"]).all()
        assert SC.check_periodic(prob, leads, orders, cand["starts"].tolist(), got["period"])
    return want_code


SHAPES = [
    ("kshape-repair", W.kshape_problem(4, 6), 12345, 20000),
    ("kshape-strict", W.kshape_problem(3, 5, space="sampled_strict"), 0, 20000),
    ("kshape-canonical", W.kshape_problem(2, 3, space="canonical"), 0, 40000),
    ("kshape-factorial", W.kshape_problem(2, 3, space="factorial"), 0, 13824),
    ("kshape-wide", W.kshape_problem(8, 12, tf=(3, 3, 1), tb=(5, 7, 2)), 1 << 33, 6000),
    ("diamond-repair", W.diamond_problem(4, 6), 777, 20000),
    ("diamond-strict", W.diamond_problem(2, 4, space="sampled_strict"), 0, 30000),
    ("diamond-canonical", W.diamond_problem(2, 3, space="canonical"), 5000, 40000),
    ("diamond-tight", W.diamond_problem(6, 3), 99, 10000),
]


@pytest.mark.parametrize("name,prob,first,n", SHAPES, ids=[s[0] for s in SHAPES])
def test_fan_in_and_fan_out_graphs(gpu, name, prob, first, n):
    codes = _compare(gpu, prob, first, n)
    if name in ("kshape-repair", "diamond-repair", "kshape-canonical"):
        assert (codes > 0).sum() > 50                      # the comparison covers periods, not only rejects


def random_graph_problem(rng):
    """2-5 devices, up to 4 block types per device; forward types then their backward mirrors; every forward type
    depends on one or two earlier forward types, the backward graph is the reverse; m = +1 / -1."""
    while True:
        D = int(rng.integers(2, 6))
        S = int(rng.integers(2, 2 * D + 1))
        dev = [int(x) for x in rng.integers(0, D, size=S)]
        if max(2 * dev.count(d) for d in range(D)) > 4:
            continue
        fwd = []
        for i in range(1, S):
            for a in set(int(x) for x in rng.integers(0, i, size=int(rng.integers(1, 3)))):
                fwd.append((a, i))
        K = 2 * S
        deps = fwd + [(K - 1 - b, K - 1 - a) for a, b in fwd]
        sinks = [i for i in range(S) if all(a != i for a, _ in fwd)]
        deps += [(i, K - 1 - i) for i in sinks]             # the backward pass of a stage follows its forward pass
        if len(deps) > 60:
            continue
        per_dev = max(2 * dev.count(d) for d in range(D))
        nr = int(rng.integers(1, min(6, 32 // per_dev) + 1))
        t = [int(x) for x in rng.integers(1, 6, size=K)]
        masks = [1 << d for d in dev] + [1 << d for d in reversed(dev)]
        return {"name": "random-graph", "D": D, "K": K, "NR": nr, "M": int(rng.integers(1, 2 * nr + 2)), "t": t,
                "m": [1] * S + [-1] * S, "dev_mask": masks, "deps": deps,
                "space": ["sampled_repair", "sampled_repair", "sampled_strict"][int(rng.integers(0, 3))],
                "seed": int(rng.integers(1, 1 << 30)), "lead_step_q16": int(rng.integers(5000, 60000)), "fixed_leads": None}


@pytest.mark.parametrize("seed", [31, 32])
def test_random_graphs(gpu, seed):
    rng = np.random.default_rng(seed)
    for case in range(8):
        prob = random_graph_problem(rng)
        _compare(gpu, prob, int(rng.integers(0, 1 << 40)), int(rng.integers(2000, 8000)))


def test_the_graph_path_on_chains_equals_the_chain_paths(gpu, monkeypatch):
    """TESSEL_FORCE_DAG=1 sends chain problems down the path for graphs: same scores as the oracle, hence as the
    fast kernel and the chain path of the general kernel (with a multi-device block too)."""
    for prob, first, n in ((W.config1(), 0, 576), (W.config3(), 4321, 6000), (dict(W.config4(), M=9), 100, 5000),
                           (W.config2(), 1 << 20, 8000), (W.xshape_problem(4, 1, 2, 2, 4), 5, 4000)):
        monkeypatch.setenv("TESSEL_FORCE_DAG", "1")
        try:
            _compare(gpu, prob, first, n)
        finally:
            monkeypatch.delenv("TESSEL_FORCE_DAG")


def test_periods_by_bisection_alone(gpu, monkeypatch):
    """Without the eigenvector search every period comes from the bisection over T with the rest test of the
    boundary values: the definition of the least period, the way the oracle computes it."""
    monkeypatch.setenv("TESSEL_DAG_TRIES", "0")
    try:
        for prob, first, n in ((W.kshape_problem(4, 6), 12345, 4000), (W.diamond_problem(4, 6), 777, 4000),
                               (W.kshape_problem(2, 3, space="canonical"), 0, 1728)):
            _compare(gpu, prob, first, n)
        monkeypatch.setenv("TESSEL_FORCE_DAG", "1")
        _compare(gpu, W.config1(), 0, 576)
        _compare(gpu, W.config3(), 99, 3000)
    finally:
        monkeypatch.delenv("TESSEL_DAG_TRIES")
        monkeypatch.delenv("TESSEL_FORCE_DAG", raising=False)


def test_completions_of_graphs_and_where_the_search_ends(gpu):
    g = gpu.Problem(W.kshape_problem(4, 6))
    g.eval_candidates(0, 4096)
    assert g.best()["feasible"]
    sched = g.complete_schedule(12)                        # the greedy completion follows any graph
    ok, makespan, peaks = SC.check_flat_schedule(g.problem, 12, sched["start"].tolist(), sched["dev_order"])
    assert ok and makespan == sched["makespan"] and max(peaks) <= 6
    # ... and so does the completion search, whose candidate 0 is the greedy schedule
    assert int(g.score_completions(12, 2, 0, 64).cpu().numpy()[0]) == makespan
    # problems beyond the fast kernel's limits (here: 12 devices) have the greedy completion only
    wide = gpu.Problem(W.pipeline_problem(W.linear_placement(12), [1] * 12, [2] * 12, 12, 2, 4, "sampled_repair", seed=3,
                                          lead_step_q16=20000))
    wide.eval_candidates(0, 4096)
    assert wide.best()["feasible"]
    assert wide.complete_schedule(16)["makespan"] > 0
    with pytest.raises(gpu.TesselError) as err:
        wide.search_completions(16, 2, 0, 64)
    assert err.value.code == -9
