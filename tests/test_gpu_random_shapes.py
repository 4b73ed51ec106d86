"""Seeded random pipeline problems (devices, placements, times, window size, cap, candidate space, some with a
two-device block at both ends of the chain), HIP path against the oracle element by element: the repetend scores and
the best candidate, with one workgroup per compute unit and the cut between the build phases anywhere, so that the
queues of the fast kernel fill, wrap and drain; then the completion candidates around the best window."""
import numpy as np
import pytest

from paper_2311_15269_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: the HIP path has no CPU fallback")
    from paper_2311_15269_amd import binding
    binding.load_library()
    return binding


def random_problem(rng, spaces):
    while True:
        D = int(rng.integers(2, 9))
        kind = int(rng.integers(0, 3))
        if kind == 0:
            stage_dev = W.linear_placement(D)
        elif kind == 1:
            stage_dev = W.folded_placement(D)
        else:
            stage_dev = [int(x) for x in rng.integers(0, D, size=int(rng.integers(2, 2 * D + 1)))]
        S = len(stage_dev)
        per_dev = max(2 * stage_dev.count(d) for d in range(D))
        if 2 * S > 32 or per_dev > 4:
            continue
        nr = int(rng.integers(1, min(8, 256 // (2 * S), 32 // per_dev) + 1))
        tf = [int(x) for x in rng.integers(1, 5, size=S)]
        tb = [int(x) for x in rng.integers(1, 9, size=S)]
        cap = int(rng.integers(1, 2 * nr + 3))
        prob = W.pipeline_problem(stage_dev, tf, tb, D, nr, cap, spaces[int(rng.integers(0, len(spaces)))],
                                  seed=int(rng.integers(1, 1 << 30)), lead_step_q16=int(rng.integers(5000, 60000)),
                                  name="random")
        if rng.random() < 0.25:
            d2 = (stage_dev[0] + 1) % D                    # first forward and last backward block on two devices
            if (2 * stage_dev.count(d2) + 2) <= 4 and (2 * stage_dev.count(d2) + 2) * nr <= 32:
                prob["dev_mask"][0] |= 1 << d2
                prob["dev_mask"][-1] |= 1 << d2
        return prob


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_problems_scores_and_best(gpu, monkeypatch, seed):
    from oracle import Oracle
    rng = np.random.default_rng(seed)
    monkeypatch.setenv("TESSEL_BLOCKS_PER_CU", "1")
    for case in range(10):
        prob = random_problem(rng, ["sampled_repair", "sampled_repair", "sampled_repair", "sampled_strict"])
        if rng.random() < 0.5:
            monkeypatch.setenv("TESSEL_STAGE_WORDS", str(int(rng.integers(0, 6))))
        else:
            monkeypatch.delenv("TESSEL_STAGE_WORDS", raising=False)
        orc, g = Oracle(prob), gpu.Problem(prob)
        first, n = int(rng.integers(0, 1 << 40)), int(rng.integers(3000, 30000))
        code, peak = g.score_candidates(first, n)
        want_code, want_peak = orc.score_range(first, n)
        assert (code.cpu().numpy() == want_code).all() and (peak.cpu().numpy() == want_peak).all(), (seed, case, prob)
        g.eval_candidates(first, n)
        got, want = g.best(), orc.sweep(first, n)
        assert got["n_evaluated"] == n and got["n_feasible"] == want["n_feasible"], (seed, case, prob)
        assert got["n_reject"][1:] == want["n_reject"][1:], (seed, case, prob)
        if want["n_feasible"]:
            assert (got["period"], got["index"], got["peak"]) == (want["period"], want["index"], want["peak"]), (seed, case, prob)


@pytest.mark.parametrize("seed", [21, 22])
def test_random_problems_completion_candidates(gpu, seed):
    from oracle import Oracle
    rng = np.random.default_rng(seed)
    ran = 0
    for case in range(40):
        prob = random_problem(rng, ["sampled_repair"])
        prob["M"] = max(prob["M"], prob["NR"])
        orc, g = Oracle(prob), gpu.Problem(prob)
        g.eval_candidates(int(rng.integers(0, 1 << 30)), 8192)
        best = g.best()
        if not best["feasible"]:
            continue
        status, leads, orders = orc.decode(best["index"])
        N = int(rng.integers(max(prob["NR"] + max(leads), 2), 80))
        J, first, ncand = int(rng.integers(0, 8)), int(rng.integers(0, 50)), int(rng.integers(100, 600))
        try:
            got = g.score_completions(N, J, first, ncand).cpu().numpy()
        except gpu.TesselError as e:
            assert e.code in (-4, -8), (seed, case, e.code)          # too big for 16-bit times, or no whole window fits
            continue
        want, want_best, want_ord = orc.completion_scores(leads, orders, N, first, ncand, J)
        assert np.array_equal(got, want), (seed, case, prob, N, J, first)
        g.search_completions(N, J, first, ncand)
        sched = g.best_completion(N)
        assert (sched["makespan"], sched["ordinal"]) == (want_best, want_ord), (seed, case, prob, N, J, first)
        ran += 1
    assert ran >= 20
