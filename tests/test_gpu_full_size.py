"""The HIP path at the full sizes of the five benchmark configurations, in the launch shape
bench.py uses (2^26 candidates per launch), against stored brute-force results of the oracle
(written by tests/golden/make_exhaustive_golden.py, which calls the oracle only): best period,
lowest index attaining it, per-device peaks, feasible count and reject counts, for the whole
range and for every piece of 2^26 ordinals on its own.  On top of that, windows of per-candidate
scores spread over the ranges are recomputed by the oracle one by one."""
import json
import os

import numpy as np
import pytest

from paper_2311_15269_amd import workloads as W

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
CHUNK = 1 << 26


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: the HIP path has no CPU fallback")
    from paper_2311_15269_amd import binding
    binding.load_library()
    return binding


def sweep_in_chunks(g, total):
    for first in range(0, total, CHUNK):
        g.eval_candidates(first, min(CHUNK, total - first))
    return g.best()


def test_config2_whole_space_matches_stored_oracle_result(gpu):
    want = json.load(open(os.path.join(GOLDEN, "config2_exhaustive.json")))
    prob = W.config2()
    g = gpu.Problem(prob)
    assert g.candidate_count() == want["count"] == 120 * 70 ** 4
    got = sweep_in_chunks(g, want["count"])
    assert got["n_evaluated"] == want["n_evaluated"]
    assert got["n_feasible"] == want["n_feasible"]
    assert got["n_reject"][1:] == want["n_reject"][1:]
    assert (got["period"], got["index"], got["peak"]) == (want["period"], want["index"], want["peak"])
    assert got["period"] == got["lower_bound"] == 12          # the zero-bubble 1F1B repetend is found


def _same(got, want, what):
    assert got["n_evaluated"] == want["n_evaluated"], what
    assert got["n_feasible"] == want["n_feasible"], what
    assert got["n_reject"][1:] == want["n_reject"][1:], what
    if want["n_feasible"]:
        assert (got["period"], got["index"], got["peak"]) == (want["period"], want["index"], want["peak"]), what
    else:
        assert not got["feasible"], what


@pytest.mark.parametrize("cfg", [3, 4, 5])
def test_sampled_configs_full_size(gpu, cfg):
    """Every launch of 2^26 ordinals on its own, then the running best over the pieces in one search, equal the
    oracle's stored sweep field by field: 2^24, 2^26 and 2^28 ordinals."""
    from oracle import Oracle
    want = json.load(open(os.path.join(GOLDEN, "config%d_full.json" % cfg)))
    prob = W.CONFIGS[cfg]()
    assert want["seed"] == prob["seed"] and want["count"] == prob["n_candidates"] and want["workload"] == prob["name"]
    assert want["complete"] and sum(piece["count"] for piece in want["pieces"]) == prob["n_candidates"]
    orc = Oracle(prob)
    g = gpu.Problem(prob)
    assert want["lower_bound"] == orc.lower_bound
    for piece in want["pieces"]:
        g.reset()
        g.eval_candidates(piece["first"], piece["count"])
        got = g.best()
        _same(got, piece, (cfg, piece["first"]))
        assert got["lower_bound"] == want["lower_bound"]
    # one search over all the pieces, last piece first
    g.reset()
    for piece in reversed(want["pieces"]):
        g.eval_candidates(piece["first"], piece["count"])
    got = g.best()
    _same(got, want, cfg)
    assert got["n_evaluated"] == prob["n_candidates"]
    # windows of per-candidate scores spread over the whole range, the last one ending at the range end
    total = prob["n_candidates"]
    rng = np.random.default_rng(cfg)
    starts = sorted(int(x) for x in rng.integers(0, total - 600, size=6)) + [total - 513]
    for first in starts:
        code, peak = g.score_candidates(first, 513)
        want_code, want_peak = orc.score_range(first, 513)
        assert (code.cpu().numpy() == want_code).all() and (peak.cpu().numpy() == want_peak).all(), (cfg, first)


def test_fast_and_general_kernels_agree(gpu, monkeypatch):
    """The general kernel (cyclic scan, Karp's formula only) and the fast kernel are two
    implementations; force the general one and compare per candidate."""
    for cfg, n in ((3, 30000), (5, 6000), (2, 50000), (1, 576)):
        prob = W.CONFIGS[cfg]()
        first = 1234 if cfg in (3, 5) else 0
        fast = gpu.Problem(prob)
        code_f, peak_f = fast.score_candidates(first, n)
        monkeypatch.setenv("TESSEL_FORCE_GENERAL", "1")
        general = gpu.Problem(prob)
        monkeypatch.delenv("TESSEL_FORCE_GENERAL")
        code_g, peak_g = general.score_candidates(first, n)
        assert (code_f == code_g).all() and (peak_f == peak_g).all(), cfg
        fast.eval_candidates(first, n)
        general.eval_candidates(first, n)
        a, b = fast.best(), general.best()
        assert b["n_window_sweeps"] == 0 and (a["n_window_sweeps"] > 0 or a["n_feasible"] == 0)
        for key in ("period", "index", "peak", "n_feasible", "n_reject", "n_evaluated"):
            assert a[key] == b[key], (cfg, key)


def test_deferred_candidates_take_the_general_kernel(gpu, monkeypatch):
    """A candidate whose boundary vector is no eigenvector yet after its first sweeps queues inside the kernel for
    a longer search (from the start again), and what that leaves open goes through a list in the workspace to the
    general kernel.  With the first search cut to 1 or 0 sweeps all feasible candidates take the queue; with the
    longer one cut as well all of them reach the general kernel; results must not change."""
    from oracle import Oracle
    for tries, retry, cfg, n in ((2, 8, 5, 20000), (1, 8, 3, 30000), (0, 0, 1, 576), (1, 1, 2, 300000), (0, 8, 5, 5000),
                                 (0, 0, 5, 3000), (2, 0, 3, 30000)):
        prob = W.CONFIGS[cfg]()
        monkeypatch.setenv("TESSEL_EIGEN_TRIES", str(tries))
        monkeypatch.setenv("TESSEL_RETRY_TRIES", str(retry))
        g = gpu.Problem(prob)
        monkeypatch.delenv("TESSEL_EIGEN_TRIES")
        monkeypatch.delenv("TESSEL_RETRY_TRIES")
        first = 4321 if cfg in (3, 5) else 0
        code, peak = g.score_candidates(first, n)
        want_code, want_peak = Oracle(prob).score_range(first, n)
        assert (code.cpu().numpy() == want_code).all() and (peak.cpu().numpy() == want_peak).all(), (tries, retry, cfg)
        for pieces in ([(first, n)], [(first, n // 2), (first + n // 2, n - n // 2)]):
            g.reset()
            for a, k in pieces:
                g.eval_candidates(a, k)
            got = g.best()
            want = Oracle(prob).sweep(first, n)
            assert got["n_evaluated"] == n and got["n_feasible"] == want["n_feasible"]
            assert (got["period"], got["index"], got["peak"]) == (want["period"], want["index"], want["peak"])
            assert got["n_reject"][1:] == want["n_reject"][1:]


def test_list_overflow_is_recovered(gpu, monkeypatch):
    """More unfinished candidates in one launch than the list of the general kernel holds must not be dropped: the
    ranges are scored again in smaller pieces and the result equals the ordinary one."""
    prob = dict(W.config3(), M=100)                   # every candidate feasible
    want_g = gpu.Problem(prob)
    want_g.eval_candidates(0, 1 << 22)
    want_g.eval_candidates(1 << 25, 1000)
    want = want_g.best()
    monkeypatch.setenv("TESSEL_EIGEN_TRIES", "0")     # and every one left to the general kernel
    monkeypatch.setenv("TESSEL_RETRY_TRIES", "0")
    g = gpu.Problem(prob)
    monkeypatch.delenv("TESSEL_EIGEN_TRIES")
    monkeypatch.delenv("TESSEL_RETRY_TRIES")
    g.eval_candidates(0, 1 << 22)                     # the list holds 2^20
    g.eval_candidates(1 << 25, 1000)
    got = g.best()
    for key in ("period", "index", "peak", "n_evaluated", "n_feasible", "n_reject"):
        assert got[key] == want[key], key
    assert got["n_evaluated"] == (1 << 22) + 1000
    g.reset()
    g.eval_candidates(0, 1 << 15)
    assert g.best()["n_evaluated"] == 1 << 15
