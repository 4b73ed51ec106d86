"""Runtime instantiation (Sec. IV-D: one global sequence of blocks and send/receive pairs, pairs right after their
producer's time slot) of schedules that the GPU path produced: the window found by the scoring kernels, completed
by the greedy rule and by the searched completion, through the C ABI; compared with the oracle's sequence for the
same schedule and run through the blocking-execution checker."""
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


@pytest.mark.parametrize("name,prob,budget,N,J,ncand", [
    ("cfg1", W.config1(), 576, 7, 2, 300),
    ("cfg3", W.config3(), 1 << 16, 14, 3, 2000),
    ("cfg4-tp", dict(W.config4(), M=9), 1 << 14, 13, 2, 1000),
    ("cfg5", W.config5(), 1 << 16, 64, 2, 4000),
])
def test_sequences_of_gpu_schedules(gpu, name, prob, budget, N, J, ncand):
    from oracle import Oracle
    g = gpu.Problem(prob)
    g.eval_candidates(0, min(budget, g.candidate_count()))
    assert g.best()["feasible"]
    o = Oracle(prob)
    greedy = g.complete_schedule(N)
    g.search_completions(N, J, 0, ncand)
    searched = g.best_completion(N)
    assert searched["makespan"] <= greedy["makespan"]
    for sched in (greedy, searched):
        ok, makespan, peaks = SC.check_flat_schedule(prob, N, sched["start"].tolist(), sched["dev_order"])
        assert ok and makespan == sched["makespan"] and max(peaks) <= prob["M"]
        got = g.instantiate(N, sched["start"])
        want = o.instantiate(N, sched["start"], sched["dev_order"])
        assert got == want
        ok, why = SC.check_instantiation(prob, N, sched["start"].tolist(), got)
        assert ok, why
        # every block once, in non-decreasing start time
        blocks = [op for op in got if op[0] == 0]
        assert sorted(op[1] for op in blocks) == list(range(prob["K"] * N))
        assert all(a[3] <= b[3] for a, b in zip(blocks, blocks[1:]))


@pytest.mark.parametrize("name,prob,budget,N", [
    ("k-shape", W.kshape_problem(2, 4), 1 << 14, 9),
    ("diamond", W.diamond_problem(3, 5), 1 << 14, 10),
    ("12-devices", W.pipeline_problem(W.linear_placement(12), [1 + (i % 3) for i in range(12)], [2 + (i % 2) for i in range(12)],
                                      12, 2, 4, "sampled_repair", seed=9, lead_step_q16=20000), 1 << 13, 7),
    ("six-types-a-device", W.pipeline_problem([0, 1, 2, 0, 1, 2, 0, 1, 2], [1] * 9, [2] * 9, 3, 2, 6, "sampled_repair", seed=3,
                                              lead_step_q16=25000), 1 << 13, 8),
])
def test_sequences_of_greedy_schedules_on_graphs_and_wide_problems(gpu, name, prob, budget, N):
    """the greedy completion and its operation sequence where the completion search does not go: branching graphs
    (several send/receive pairs out of one block, several into one), more than 8 devices, six block types a device"""
    from oracle import Oracle
    g = gpu.Problem(prob)
    g.eval_candidates(0, budget)
    assert g.best()["feasible"]
    o = Oracle(prob)
    sched = g.complete_schedule(N)
    ok, makespan, peaks = SC.check_flat_schedule(prob, N, sched["start"].tolist(), sched["dev_order"])
    assert ok and makespan == sched["makespan"] and max(peaks) <= prob["M"]
    got = g.instantiate(N, sched["start"])
    assert got == o.instantiate(N, sched["start"], sched["dev_order"])
    ok, why = SC.check_instantiation(prob, N, sched["start"].tolist(), got)
    assert ok, why
    blocks = [op for op in got if op[0] == 0]
    assert sorted(op[1] for op in blocks) == list(range(prob["K"] * N))
