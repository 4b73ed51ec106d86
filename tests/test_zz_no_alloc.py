"""tessel_eval_candidates_noalloc (the scoring entry point for callers that cannot allocate device memory: the
library's own buffer instead of a workspace) against tessel_eval_candidates, through the C ABI: two calls in a row on
the same GPU buffer, the second with a smaller input, then another handle and problem in the same buffer."""
import pytest

from paper_2311_15269_amd import workloads as W

pytestmark = pytest.mark.gpu
KEYS = ("period", "index", "peak", "peak_max", "n_evaluated", "n_feasible", "n_reject", "feasible")


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: the HIP path has no CPU fallback")
    from paper_2311_15269_amd import binding
    binding.load_library()
    return binding


def _reference(gpu, prob, first, count):
    g = gpu.Problem(prob)
    g.eval_candidates(first, count)
    return g.best()


def test_noalloc_equals_the_workspace_entry_point(gpu):
    import torch
    prob = W.config5()
    g = gpu.Problem(prob)
    import gc
    gc.collect()                                           # (workspaces of earlier tests go now, not during the call)
    before = torch.cuda.memory_allocated()
    # first call: a range that leaves the queues of the buffer full of stale candidates
    g.eval_candidates_noalloc(7, (1 << 20) + 3)
    got = g.best()
    assert torch.cuda.memory_allocated() <= before        # nothing came from torch's allocator either
    want = _reference(gpu, prob, 7, (1 << 20) + 3)
    for key in KEYS:
        assert got[key] == want[key], key
    # second call, a new search with a smaller input, in the buffer as the first left it
    g.reset()
    g.eval_candidates_noalloc(123456, 5000)
    got = g.best()
    want = _reference(gpu, prob, 123456, 5000)
    for key in KEYS:
        assert got[key] == want[key], key
    # the search goes on over further calls, and the schedule completion reads the same buffer
    g.eval_candidates_noalloc(0, 40000)
    g.eval_candidates_noalloc(123456 + 5000, 1)
    ref = gpu.Problem(prob)
    ref.eval_candidates(0, 40000)
    ref.eval_candidates(123456, 5001)
    got, want = g.best(), ref.best()
    for key in KEYS:
        assert got[key] == want[key], key
    assert g.complete_schedule(24)["makespan"] == ref.complete_schedule(24)["makespan"]


@pytest.mark.parametrize("cfg,count", [(1, 576), (2, 300000), (3, 200000), (4, 150000)])
def test_noalloc_other_problems_share_the_buffer(gpu, cfg, count):
    """every problem of the benchmark set, one handle after the other in the same buffer; the exhaustive spaces keep
    their tables in it as well"""
    prob = W.CONFIGS[cfg]() if cfg != 4 else dict(W.config4(), M=9)
    g = gpu.Problem(prob)
    g.eval_candidates_noalloc(0, count)
    got = g.best()
    want = _reference(gpu, prob, 0, count)
    for key in KEYS:
        assert got[key] == want[key], (cfg, key)
    g.reset()
    g.eval_candidates_noalloc(count // 3, count // 7)
    got = g.best()
    want = _reference(gpu, prob, count // 3, count // 7)
    for key in KEYS:
        assert got[key] == want[key], (cfg, key)


def test_noalloc_more_than_eight_devices(gpu):
    """16 and 32 devices: the general kernel keeps its lanes' program (and a state too large for the LDS) in the buffer too,
    on as many workgroups as fit"""
    from tests.test_gpu_wide import vshape
    for prob, first, count in ((vshape(16, 8, 12), 7, 3000), (vshape(12, 2, 2), 0, 20000), (vshape(32, 16, 40), 3, 700)):
        g = gpu.Problem(prob)
        g.eval_candidates_noalloc(first, count)
        got = g.best()
        want = _reference(gpu, prob, first, count)
        for key in KEYS:
            assert got[key] == want[key], (prob["name"], key)


def test_noalloc_refuses_what_it_cannot_hold(gpu):
    g = gpu.Problem(W.config5())
    with pytest.raises(gpu.TesselError) as err:
        g.eval_candidates_noalloc(0, (1 << 26) + 1)
    assert err.value.code == -4                            # TESSEL_E_TOOBIG
    g2 = gpu.Problem(W.config1())
    with pytest.raises(gpu.TesselError) as err:
        g2.eval_candidates_noalloc(500, 100)               # outside the 576 candidates of the space
    assert err.value.code == -8                            # TESSEL_E_RANGE
