"""The C-ABI library loads and exports every symbol include/tessel.h declares; host-only
error paths.  No GPU, no compute calls."""
import ctypes as C
import os
import re

import pytest

from paper_2311_15269_amd import binding, workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "tessel.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tessel_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = binding.load_library()
    names = declared_functions()
    assert len(names) >= 10
    assert sorted(names) == sorted(binding.EXPORTS)
    for name in names:
        assert getattr(lib, name) is not None


def test_problem_create_validates_on_the_host():
    p = binding.Problem(W.config1())
    assert p.candidate_count() == 576
    assert binding.Problem(W.config2()).candidate_count() == 120 * 70 ** 4
    assert binding.Problem(W.config5()).candidate_count() == 2 ** 64 - 1
    assert p.workspace_bytes() > 0
    # a block type with two consumers: the micro-batch graph need not be a set of chains
    assert binding.Problem(dict(W.config1(), deps=[(0, 1), (0, 2), (2, 3)])).candidate_count() > 0
    # up to 32 devices
    wide = {"name": "wide", "D": 32, "K": 32, "NR": 2, "M": 0, "t": [1] * 32, "m": [0] * 32, "dev_mask": [1 << d for d in range(32)],
            "deps": [(i, i + 1) for i in range(31)], "space": "sampled_repair", "seed": 1, "lead_step_q16": 100, "fixed_leads": None}
    assert binding.Problem(wide).candidate_count() == 2 ** 64 - 1
    assert binding.Problem(wide).workspace_bytes() > 0
    many = dict(wide, K=64, t=[1] * 64, m=[0] * 64, dev_mask=[1 << (d % 32) for d in range(64)], deps=[(i, i + 1) for i in range(63)])
    assert binding.Problem(many).candidate_count() == 2 ** 64 - 1
    # up to eight block types on a device in the sampled spaces, four in the exhaustive ones
    crowded = W.pipeline_problem([0, 1, 0, 1, 0, 1], [1] * 6, [2] * 6, 2, 2, 9, "sampled_repair")
    assert binding.Problem(crowded).candidate_count() == 2 ** 64 - 1
    # windows of up to 16 micro-batches in the sampled spaces, 8 in the exhaustive ones
    assert binding.Problem(dict(W.config1(), NR=16, M=16, space="sampled_repair")).workspace_bytes() > 0
    assert binding.Problem(dict(wide, NR=16)).workspace_bytes() > 0
    for bad, code in (
        (dict(crowded, space="canonical"), -9),
        (dict(crowded, NR=6), -9),                             # 36 blocks on a device
        (dict(wide, D=33), -9),
        (dict(many, K=65, t=[1] * 65, m=[0] * 65, dev_mask=[1 << (d % 32) for d in range(65)]), -9),
        (dict(W.config1(), m=[1, 1, -1, 0]), -3),
        (dict(W.config1(), deps=[(0, 1), (1, 0)]), -2),
        (dict(W.config1(), t=[0, 1, 2, 2]), -1),
        (dict(W.config1(), NR=9), -9),                                  # windows of more than 8 micro-batches: sampled spaces only
        (dict(W.config1(), NR=17, space="sampled_repair"), -9),
        (dict(W.config3(), NR=9), -9),                                  # 4 types a device: at most 32 blocks per device and window
        (dict(W.config1(), fixed_leads=[0, 0, 0, 0]), -1),
        (W.pipeline_problem(W.folded_placement(8), [1] * 16, [1] * 16, 8, 8, 10, "canonical"), -4),
    ):
        with pytest.raises(binding.TesselError) as e:
            binding.Problem(bad)
        assert e.value.code == code, bad


def test_strerror_covers_all_codes():
    lib = binding.load_library()
    texts = {lib.tessel_strerror(c).decode() for c in range(0, -11, -1)}
    assert len(texts) == 11 and "unknown error" not in texts


def test_alu_probe_validates_its_arguments_on_the_host():
    lib = binding.load_library()
    import ctypes as C
    ops = C.c_uint64(0)
    assert lib.tessel_alu_probe(0, 10, 1, 1 << 20, None, C.byref(ops)) == -1
    assert lib.tessel_alu_probe(4, 0, 1, 1 << 20, None, C.byref(ops)) == -1
    assert lib.tessel_alu_probe(4, 10, None, 1 << 20, None, C.byref(ops)) == -1
    assert lib.tessel_alu_probe(4, 10, 256, 4 * 256 * 4 - 1, None, C.byref(ops)) == -5


def test_search_validates_its_arguments_on_the_host():
    import ctypes as C
    lib = binding.load_library()
    desc, keep = binding._describe(W.config1())
    n = C.c_size_t()
    io = binding.Search(max_nr=0)
    assert lib.tessel_search_workspace_bytes(C.byref(desc), C.byref(io), C.byref(n)) == -1
    assert lib.tessel_search_run(C.byref(desc), C.byref(io), None, 0, None, None) == -1
    io = binding.Search(max_nr=17)
    assert lib.tessel_search_run(C.byref(desc), C.byref(io), None, 0, None, None) == -1
    # window sizes beyond the in-flight bound are never created: the 4-stage canonical space has no table for N_R = 8
    desc, keep = binding._describe(W.config2())
    io = binding.Search(max_nr=8, use_inflight_bound=1)
    assert lib.tessel_search_workspace_bytes(C.byref(desc), C.byref(io), C.byref(n)) == 0 and n.value > 0
    io = binding.Search(max_nr=8, use_inflight_bound=0)
    assert lib.tessel_search_workspace_bytes(C.byref(desc), C.byref(io), C.byref(n)) == -4
