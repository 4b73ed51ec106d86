"""Thin ctypes binding of the C ABI in include/tessel.h -- argument marshalling only.

PyTorch is used for device memory (workspace, output buffers) and for the current HIP
stream; every step of the evaluation runs in the library's kernels.  There is no CPU
fallback: if the HIP library is missing or no GPU is present, calls raise.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

MAX_DEVICES = 32
MAX_POS = 32
NUM_STATUS = 6
STATUS_NAMES = ("OK", "DUP", "TP_MISMATCH", "PROP2", "DEADLOCK", "MEM")
SPACE = {"factorial": 0, "canonical": 1, "sampled_strict": 2, "sampled_repair": 3}

E_NO_FEASIBLE = -7
E_RANGE = -8

EXPORTS = (
    "tessel_problem_create", "tessel_problem_destroy", "tessel_candidate_count", "tessel_workspace_bytes",
    "tessel_eval_candidates", "tessel_eval_candidates_noalloc", "tessel_score_candidates", "tessel_best", "tessel_best_candidate", "tessel_reset",
    "tessel_complete_schedule", "tessel_search_completions", "tessel_score_completions", "tessel_best_completion",
    "tessel_instantiate", "tessel_search_workspace_bytes", "tessel_search_run", "tessel_alu_probe", "tessel_strerror", "tessel_last_hip_error",
)


class ProblemDesc(C.Structure):
    _fields_ = [("num_devices", C.c_int32), ("num_block_types", C.c_int32), ("nr", C.c_int32), ("mem_cap", C.c_int32),
                ("time", C.c_void_p), ("mem", C.c_void_p), ("dev_mask", C.c_void_p),
                ("num_deps", C.c_int32), ("dep_src", C.c_void_p), ("dep_dst", C.c_void_p),
                ("space", C.c_int32), ("fixed_leads", C.c_void_p), ("seed", C.c_uint64), ("lead_step_q16", C.c_uint32)]


class Result(C.Structure):
    _fields_ = [("period", C.c_int32), ("index", C.c_uint64), ("peak_mem", C.c_int32 * MAX_DEVICES),
                ("peak_max", C.c_int32), ("lower_bound", C.c_int32), ("n_evaluated", C.c_uint64),
                ("n_feasible", C.c_uint64), ("n_reject", C.c_uint64 * NUM_STATUS), ("n_window_sweeps", C.c_uint64), ("n_blocks_placed", C.c_uint64)]


class Schedule(C.Structure):
    _fields_ = [("num_microbatches", C.c_int32), ("capacity", C.c_int32), ("start", C.c_void_p),
                ("dev_order", C.c_void_p), ("dev_len", C.c_void_p), ("makespan", C.c_int32), ("period", C.c_int32),
                ("num_windows", C.c_int32)]


class TesselError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("tessel error %d: %s" % (code, text))
        self.code = code


_lib = None


def library_path():
    return _build.LIB


MAX_NR = 16


class Search(C.Structure):
    _fields_ = [("max_nr", C.c_int32), ("use_inflight_bound", C.c_int32), ("max_candidates", C.c_uint64),
                ("launch_candidates", C.c_uint64), ("inflights", C.c_int32), ("lower_bound", C.c_int32),
                ("nr_tried", C.c_int32), ("best_nr", C.c_int32), ("best_period", C.c_int32), ("early_exit", C.c_int32),
                ("best_index", C.c_uint64), ("period_nr", C.c_int32 * (MAX_NR + 1)),
                ("index_nr", C.c_uint64 * (MAX_NR + 1)), ("evaluated_nr", C.c_uint64 * (MAX_NR + 1))]


def load_library():
    """Loads the in-tree HIP library; builds it first only if it has never been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_build.LIB):
            _build.build_library()
        # torch (device memory and streams of this binding) brings its own HIP runtime: it has to be the one the
        # process loads first, or torch finds no GPU afterwards
        import torch  # noqa: F401
        lib = C.CDLL(_build.LIB)
        lib.tessel_problem_create.argtypes = [C.POINTER(ProblemDesc), C.POINTER(C.c_void_p)]
        lib.tessel_problem_destroy.argtypes = [C.c_void_p]
        lib.tessel_problem_destroy.restype = None
        lib.tessel_candidate_count.argtypes = [C.c_void_p, C.POINTER(C.c_uint64)]
        lib.tessel_workspace_bytes.argtypes = [C.c_void_p, C.POINTER(C.c_size_t)]
        lib.tessel_eval_candidates.argtypes = [C.c_void_p, C.c_uint64, C.c_uint64, C.c_void_p, C.c_size_t, C.c_void_p]
        lib.tessel_eval_candidates_noalloc.argtypes = [C.c_void_p, C.c_uint64, C.c_uint64, C.c_void_p]
        lib.tessel_score_candidates.argtypes = [C.c_void_p, C.c_uint64, C.c_uint64, C.c_void_p, C.c_void_p,
                                                C.c_void_p, C.c_size_t, C.c_void_p]
        lib.tessel_best.argtypes = [C.c_void_p, C.POINTER(Result)]
        lib.tessel_best_candidate.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.tessel_reset.argtypes = [C.c_void_p]
        lib.tessel_complete_schedule.argtypes = [C.c_void_p, C.POINTER(Schedule)]
        lib.tessel_search_completions.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_uint64, C.c_uint64]
        lib.tessel_score_completions.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_uint64, C.c_uint64, C.c_void_p]
        lib.tessel_best_completion.argtypes = [C.c_void_p, C.POINTER(Schedule), C.POINTER(C.c_uint64)]
        lib.tessel_instantiate.argtypes = [C.c_void_p, C.POINTER(Schedule), C.c_void_p, C.c_int32, C.POINTER(C.c_int32)]
        lib.tessel_search_workspace_bytes.argtypes = [C.POINTER(ProblemDesc), C.POINTER(Search), C.POINTER(C.c_size_t)]
        lib.tessel_search_run.argtypes = [C.POINTER(ProblemDesc), C.POINTER(Search), C.c_void_p, C.c_size_t, C.c_void_p,
                                          C.POINTER(C.c_void_p)]
        lib.tessel_alu_probe.argtypes = [C.c_int, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(C.c_uint64)]
        lib.tessel_strerror.argtypes = [C.c_int]
        lib.tessel_strerror.restype = C.c_char_p
        lib.tessel_last_hip_error.argtypes = [C.c_void_p]
        _lib = lib
    return _lib


def alu_probe(blocks, rounds, out=None):
    """tessel_alu_probe on torch's current stream; returns (lane operations of the launch, out tensor)."""
    import torch
    if out is None:
        out = torch.empty(blocks * 256, dtype=torch.int32, device="cuda")
    ops = C.c_uint64(0)
    _check(load_library().tessel_alu_probe(blocks, rounds, out.data_ptr(), out.numel() * 4,
                                           torch.cuda.current_stream().cuda_stream, C.byref(ops)))
    return int(ops.value), out


def _check(rc, allow=()):
    if rc != 0 and rc not in allow:
        raise TesselError(rc, load_library().tessel_strerror(rc).decode())
    return rc


def _i32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _describe(problem):
    """tessel_problem_desc of a workload dict + the arrays it points into (keep them alive)"""
    t, m = _i32(problem["t"]), _i32(problem["m"])
    mask = np.ascontiguousarray(np.asarray(problem["dev_mask"], dtype=np.uint32))
    deps = problem["deps"]
    src, dst = _i32([a for a, _ in deps]), _i32([b for _, b in deps])
    fixed = problem.get("fixed_leads")
    fixed = _i32(fixed) if fixed is not None else None
    desc = ProblemDesc(problem["D"], problem["K"], problem["NR"], problem["M"], t.ctypes.data, m.ctypes.data,
                       mask.ctypes.data, len(deps), src.ctypes.data if len(deps) else None,
                       dst.ctypes.data if len(deps) else None, SPACE[problem["space"]],
                       fixed.ctypes.data if fixed is not None else None,
                       problem.get("seed", 0), problem.get("lead_step_q16", 0))
    return desc, (t, m, mask, src, dst, fixed)


def search(problem, max_nr, max_candidates, launch_candidates=0, use_inflight_bound=True):
    """tessel_search_run: Alg. 1 over window sizes 1..max_nr.  Returns (dict of the out fields, Problem of
    the incumbent's window size with the incumbent as its running best, or None if nothing is feasible)."""
    import torch
    lib = load_library()
    desc, keep = _describe(problem)
    io = Search(max_nr=max_nr, use_inflight_bound=1 if use_inflight_bound else 0, max_candidates=max_candidates,
                launch_candidates=launch_candidates)
    n = C.c_size_t()
    _check(lib.tessel_search_workspace_bytes(C.byref(desc), C.byref(io), C.byref(n)))
    ws = torch.empty(n.value + 256, dtype=torch.uint8, device="cuda")
    ptr = (ws.data_ptr() + 255) & ~255
    h = C.c_void_p()
    rc = _check(lib.tessel_search_run(C.byref(desc), C.byref(io), ptr, ws.numel() - (ptr - ws.data_ptr()),
                                      torch.cuda.current_stream().cuda_stream, C.byref(h)), allow=(E_NO_FEASIBLE,))
    k = io.nr_tried
    out = {"inflights": io.inflights, "lower_bound": io.lower_bound, "nr_tried": k, "best_nr": io.best_nr,
           "best_period": io.best_period, "best_index": int(io.best_index), "early_exit": bool(io.early_exit),
           "period_nr": list(io.period_nr[1:k + 1]), "index_nr": [int(x) for x in io.index_nr[1:k + 1]],
           "evaluated_nr": [int(x) for x in io.evaluated_nr[1:k + 1]]}
    best = Problem._adopt(dict(problem, NR=io.best_nr), h, ws) if rc == 0 else None
    return out, best


class Problem:
    """tessel_problem_create / _destroy and the calls on the handle, same names as the C ABI."""

    def __init__(self, problem):
        lib = load_library()
        self.problem = problem
        self.D, self.K, self.NR = problem["D"], problem["K"], problem["NR"]
        desc, self._keep = _describe(problem)
        h = C.c_void_p()
        _check(lib.tessel_problem_create(C.byref(desc), C.byref(h)))
        self._h = h
        self._ws = None

    @classmethod
    def _adopt(cls, problem, handle, ws):
        """wraps a handle the library returned (tessel_search_run) and the workspace it is bound to"""
        self = cls.__new__(cls)
        self.problem = problem
        self.D, self.K, self.NR = problem["D"], problem["K"], problem["NR"]
        self._keep = None
        self._h = handle
        self._ws = ws
        return self

    def close(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.tessel_problem_destroy(self._h)
        self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:       # interpreter shutdown
            pass

    # ---- plumbing: device memory and stream come from torch
    def _workspace(self):
        import torch
        if self._ws is None:
            n = C.c_size_t()
            _check(load_library().tessel_workspace_bytes(self._h, C.byref(n)))
            self._ws = torch.empty(n.value + 256, dtype=torch.uint8, device="cuda")
        ptr = (self._ws.data_ptr() + 255) & ~255
        return ptr, self._ws.numel() - (ptr - self._ws.data_ptr())

    @staticmethod
    def _stream():
        import torch
        return torch.cuda.current_stream().cuda_stream

    # ---- the C ABI
    def candidate_count(self):
        n = C.c_uint64()
        _check(load_library().tessel_candidate_count(self._h, C.byref(n)))
        return n.value

    def workspace_bytes(self):
        n = C.c_size_t()
        _check(load_library().tessel_workspace_bytes(self._h, C.byref(n)))
        return n.value

    def eval_candidates(self, first, count, stream=None):
        ptr, size = self._workspace()
        _check(load_library().tessel_eval_candidates(self._h, first, count, ptr, size,
                                                      self._stream() if stream is None else stream))

    def eval_candidates_noalloc(self, first, count, stream=None):
        """tessel_eval_candidates_noalloc: the library's own device buffer instead of a workspace tensor"""
        _check(load_library().tessel_eval_candidates_noalloc(self._h, first, count,
                                                              self._stream() if stream is None else stream))

    def score_candidates(self, first, count):
        """returns (code, peak) int32 CUDA tensors"""
        import torch
        ptr, size = self._workspace()
        code = torch.empty(count, dtype=torch.int32, device="cuda")
        peak = torch.empty(count, dtype=torch.int32, device="cuda")
        _check(load_library().tessel_score_candidates(self._h, first, count, code.data_ptr(), peak.data_ptr(), ptr,
                                                       size, self._stream()))
        return code, peak

    def best(self):
        r = Result()
        rc = _check(load_library().tessel_best(self._h, C.byref(r)), allow=(E_NO_FEASIBLE,))
        return {"period": r.period, "index": int(r.index), "peak": list(r.peak_mem[:self.D]), "peak_max": r.peak_max,
                "lower_bound": r.lower_bound, "n_evaluated": int(r.n_evaluated), "n_feasible": int(r.n_feasible),
                "n_reject": [int(x) for x in r.n_reject], "n_window_sweeps": int(r.n_window_sweeps), "n_blocks_placed": int(r.n_blocks_placed),
                "feasible": rc == 0}

    def best_candidate(self):
        leads = np.zeros(self.K, dtype=np.int32)
        olen = np.zeros(self.D, dtype=np.int32)
        orders = np.zeros((self.D, MAX_POS), dtype=np.int32)
        starts = np.zeros(self.K * self.NR, dtype=np.int32)
        _check(load_library().tessel_best_candidate(self._h, leads.ctypes.data, olen.ctypes.data, orders.ctypes.data,
                                                     starts.ctypes.data))
        return {"leads": leads.tolist(), "orders": [orders[d, :olen[d]].tolist() for d in range(self.D)],
                "starts": starts.reshape(self.K, self.NR)}

    def reset(self):
        _check(load_library().tessel_reset(self._h))

    def search_completions(self, num_microbatches, jitter, first, count):
        _check(load_library().tessel_search_completions(self._h, num_microbatches, jitter, first, count))

    def score_completions(self, num_microbatches, jitter, first, count):
        """returns the makespans as an int32 CUDA tensor"""
        import torch
        out = torch.empty(max(1, count), dtype=torch.int32, device="cuda")
        _check(load_library().tessel_score_completions(self._h, num_microbatches, jitter, first, count, out.data_ptr()))
        torch.cuda.synchronize()
        return out[:count]

    def best_completion(self, num_microbatches):
        N = num_microbatches
        cap = self.K * N
        start = np.full(cap, -1, dtype=np.int32)
        dev_order = np.full((self.D, cap), -1, dtype=np.int32)
        dev_len = np.zeros(self.D, dtype=np.int32)
        s = Schedule(N, cap, start.ctypes.data, dev_order.ctypes.data, dev_len.ctypes.data, 0, 0, 0)
        ordinal = C.c_uint64(0)
        _check(load_library().tessel_best_completion(self._h, C.byref(s), C.byref(ordinal)))
        return {"makespan": s.makespan, "period": s.period, "num_windows": s.num_windows, "ordinal": int(ordinal.value),
                "start": start.reshape(self.K, N), "dev_order": [dev_order[d, :dev_len[d]].tolist() for d in range(self.D)]}

    def instantiate(self, num_microbatches, start):
        """tessel_instantiate: list of (kind, block, src, dst, aux) for the schedule with these start times [K][N]"""
        N = num_microbatches
        start = _i32(np.asarray(start).reshape(-1))
        s = Schedule(N, self.K * N, start.ctypes.data, None, None, 0, 0, 0)
        n = C.c_int32(0)
        rc = load_library().tessel_instantiate(self._h, C.byref(s), None, 0, C.byref(n))
        if rc not in (0, E_RANGE):
            _check(rc)
        ops = np.zeros((max(1, n.value), 5), dtype=np.int32)
        _check(load_library().tessel_instantiate(self._h, C.byref(s), ops.ctypes.data, n.value, C.byref(n)))
        return [tuple(int(v) for v in row) for row in ops[:n.value]]

    def complete_schedule(self, num_microbatches):
        N = num_microbatches
        cap = self.K * N
        start = np.full(cap, -1, dtype=np.int32)
        dev_order = np.full((self.D, cap), -1, dtype=np.int32)
        dev_len = np.zeros(self.D, dtype=np.int32)
        s = Schedule(N, cap, start.ctypes.data, dev_order.ctypes.data, dev_len.ctypes.data, 0, 0, 0)
        _check(load_library().tessel_complete_schedule(self._h, C.byref(s)))
        return {"makespan": s.makespan, "period": s.period, "num_windows": s.num_windows,
                "start": start.reshape(self.K, N), "dev_order": [dev_order[d, :dev_len[d]].tolist() for d in range(self.D)]}
