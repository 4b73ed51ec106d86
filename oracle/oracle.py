"""ctypes front end of oracle/tessel_oracle.c (test infrastructure, not the product).

Argument marshalling only: every number comes out of the C file, which is written from the
paper's definitions (Eq. 1, Eq. 3-6, Properties 1-2, Alg. 1) and shares nothing with the
HIP library.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tessel_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

MAX_D = 32
NSTATUS = 6
STATUS_NAMES = ("OK", "DUP", "TP_MISMATCH", "PROP2", "DEADLOCK", "MEM")
SPACE = {"factorial": 0, "canonical": 1, "sampled_strict": 2, "sampled_repair": 3}


def build_oracle(force=False):
    """Compile the oracle with gcc (plain C, -O2) if the library is missing or stale."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-Wall", "-shared", "-fPIC", "-pthread", "-o", _LIB, _SRC])
    return _LIB


class OracleScore(C.Structure):
    _fields_ = [("status", C.c_int), ("period", C.c_int), ("peak", C.c_int * MAX_D), ("peak_max", C.c_int)]


class OracleResult(C.Structure):
    _fields_ = [("period", C.c_int), ("index", C.c_uint64), ("peak", C.c_int * MAX_D), ("peak_max", C.c_int),
                ("n_evaluated", C.c_uint64), ("n_feasible", C.c_uint64), ("n_reject", C.c_uint64 * NSTATUS),
                ("ops", C.c_uint64)]


_lib = None


MAX_NR = 16


class OracleSearch(C.Structure):
    _fields_ = [("inflights", C.c_int), ("lower_bound", C.c_int), ("nr_tried", C.c_int), ("best_nr", C.c_int),
                ("best_period", C.c_int), ("best_index", C.c_uint64), ("early_exit", C.c_int),
                ("period_nr", C.c_int * (MAX_NR + 1)), ("index_nr", C.c_uint64 * (MAX_NR + 1)),
                ("evaluated_nr", C.c_uint64 * (MAX_NR + 1))]


def _load():
    global _lib
    if _lib is None:
        lib = C.CDLL(build_oracle())
        lib.orc_create.restype = C.c_void_p
        lib.orc_create.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                   C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_uint64, C.c_uint32,
                                   C.POINTER(C.c_int)]
        lib.orc_destroy.argtypes = [C.c_void_p]
        lib.orc_candidate_count.restype = C.c_uint64
        lib.orc_candidate_count.argtypes = [C.c_void_p]
        for f in (lib.orc_lower_bound, lib.orc_upper_bound, lib.orc_num_lead_vectors):
            f.restype = C.c_int
            f.argtypes = [C.c_void_p]
        lib.orc_eval_index.argtypes = [C.c_void_p, C.c_uint64, C.POINTER(OracleScore), C.c_void_p]
        lib.orc_decode_index.argtypes = [C.c_void_p, C.c_uint64, C.POINTER(C.c_int), C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_int]
        lib.orc_eval_explicit.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                          C.POINTER(OracleScore), C.c_void_p]
        lib.orc_feasible_explicit.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int]
        lib.orc_repair_explicit.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p]
        lib.orc_sweep.argtypes = [C.c_void_p, C.c_uint64, C.c_uint64, C.POINTER(OracleResult)]
        lib.orc_sweep_mt.argtypes = [C.c_void_p, C.c_uint64, C.c_uint64, C.c_int, C.POINTER(OracleResult)]
        lib.orc_score_range.argtypes = [C.c_void_p, C.c_uint64, C.c_uint64, C.c_void_p, C.c_void_p]
        lib.orc_complete.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int,
                                     C.c_void_p, C.c_void_p, C.c_void_p]
        lib.orc_draw16.restype = C.c_uint32
        lib.orc_draw16.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32]
        lib.orc_complete_jitter.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_uint64,
                                            C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.orc_completion_scores.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int,
                                              C.c_uint64, C.c_uint64, C.c_int, C.c_void_p, C.POINTER(C.c_uint64)]
        lib.orc_instantiate.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int]
        lib.orc_max_inflight.argtypes = [C.c_void_p, C.c_int]
        lib.orc_search.argtypes = [C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p,
                                   C.c_void_p, C.c_int, C.c_uint64, C.c_uint32, C.c_int, C.c_int, C.c_uint64,
                                   C.POINTER(OracleSearch)]
        lib.orc_sizeof_search_result.restype = C.c_uint64
        assert lib.orc_sizeof_search_result() == C.sizeof(OracleSearch)
        assert lib.orc_sizeof_score() == C.sizeof(OracleScore)
        assert lib.orc_sizeof_result() == C.sizeof(OracleResult)
        _lib = lib
    return _lib


def draw16(seed, ordinal, j):
    return int(_load().orc_draw16(seed, ordinal, j))


class OracleError(Exception):
    def __init__(self, code):
        super().__init__("oracle error %d" % code)
        self.code = code


def _i32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def search(problem, max_nr, max_candidates, use_inflight_bound=True):
    """Alg. 1 over window sizes 1..max_nr (the problem's own NR is ignored), candidate by candidate."""
    t, m = _i32(problem["t"]), _i32(problem["m"])
    mask = np.ascontiguousarray(np.asarray(problem["dev_mask"], dtype=np.uint32))
    deps = problem["deps"]
    src, dst = _i32([a for a, _ in deps]), _i32([b for _, b in deps])
    r = OracleSearch()
    rc = _load().orc_search(problem["D"], problem["K"], problem["M"], t.ctypes.data, m.ctypes.data, mask.ctypes.data,
                            len(deps), src.ctypes.data, dst.ctypes.data, SPACE[problem["space"]],
                            problem.get("seed", 0), problem.get("lead_step_q16", 0), max_nr,
                            1 if use_inflight_bound else 0, max_candidates, C.byref(r))
    if rc:
        raise OracleError(rc)
    n = r.nr_tried
    return {"inflights": r.inflights, "lower_bound": r.lower_bound, "nr_tried": n, "best_nr": r.best_nr,
            "best_period": r.best_period, "best_index": int(r.best_index), "early_exit": bool(r.early_exit),
            "period_nr": list(r.period_nr[1:n + 1]), "index_nr": [int(x) for x in r.index_nr[1:n + 1]],
            "evaluated_nr": [int(x) for x in r.evaluated_nr[1:n + 1]]}


class Oracle:
    """One scheduling problem held by the C oracle.  `problem` is a dict with the keys of
    the workload generators: D, K, NR, M, t, m, dev_mask, deps, space, fixed_leads, seed,
    lead_step_q16."""

    def __init__(self, problem):
        lib = _load()
        self.problem = problem
        self.D, self.K, self.NR, self.M = problem["D"], problem["K"], problem["NR"], problem["M"]
        t, m = _i32(problem["t"]), _i32(problem["m"])
        mask = np.ascontiguousarray(np.asarray(problem["dev_mask"], dtype=np.uint32))
        deps = problem["deps"]
        src, dst = _i32([a for a, _ in deps]), _i32([b for _, b in deps])
        fixed = problem.get("fixed_leads")
        fixed_arr = _i32(fixed) if fixed is not None else None
        err = C.c_int(0)
        self._h = lib.orc_create(self.D, self.K, self.NR, self.M, t.ctypes.data, m.ctypes.data, mask.ctypes.data,
                                 len(deps), src.ctypes.data, dst.ctypes.data, SPACE[problem["space"]],
                                 fixed_arr.ctypes.data if fixed_arr is not None else None,
                                 problem.get("seed", 0), problem.get("lead_step_q16", 0), C.byref(err))
        if not self._h:
            raise OracleError(err.value)
        self.n_on_dev = [sum(1 for k in range(self.K) if mask[k] >> d & 1) * self.NR for d in range(self.D)]
        self.stride = max(self.n_on_dev)

    def __del__(self):
        if getattr(self, "_h", None):
            _load().orc_destroy(self._h)
            self._h = None

    def complete_jitter(self, leads, orders, N, ordinal, J):
        """schedule of completion candidate `ordinal` (jitter amplitude J); ordinal 0 = the plain greedy one"""
        length, seq = self._pack(orders)
        leads = _i32(leads)
        start = np.full(self.K * N, -1, dtype=np.int32)
        dev_order = np.full((self.D, self.K * N), -1, dtype=np.int32)
        dev_len = np.zeros(self.D, dtype=np.int32)
        rc = _load().orc_complete_jitter(self._h, leads.ctypes.data, length.ctypes.data, seq.ctypes.data, self.stride, N,
                                         ordinal, J, start.ctypes.data, dev_order.ctypes.data, dev_len.ctypes.data)
        if rc < 0:
            raise OracleError(rc)
        return {"makespan": rc, "start": start.reshape(self.K, N),
                "dev_order": [dev_order[d, :dev_len[d]].tolist() for d in range(self.D)]}

    def completion_scores(self, leads, orders, N, first, count, J):
        """(makespans int32[count] with INT32_MAX = no schedule, best makespan, lowest ordinal attaining it)"""
        length, seq = self._pack(orders)
        leads = _i32(leads)
        out = np.zeros(count, dtype=np.int32)
        best = C.c_uint64(0)
        rc = _load().orc_completion_scores(self._h, leads.ctypes.data, length.ctypes.data, seq.ctypes.data, self.stride,
                                           N, first, count, J, out.ctypes.data, C.byref(best))
        if rc < 0 and rc != -10:
            raise OracleError(rc)
        return out, (rc if rc >= 0 else None), int(best.value)

    def instantiate(self, N, start, dev_order):
        """global operation sequence of a complete schedule (Sec. IV-D): list of (kind, block, src, dst, aux)"""
        start = _i32(np.asarray(start).reshape(-1))
        stride = self.K * N
        order = np.full((self.D, stride), -1, dtype=np.int32)
        length = np.zeros(self.D, dtype=np.int32)
        for d, row in enumerate(dev_order):
            order[d, :len(row)] = row
            length[d] = len(row)
        cap = self.K * N * (1 + self.D * max(1, len(self.problem["deps"])))
        ops = np.zeros((cap, 5), dtype=np.int32)
        n = _load().orc_instantiate(self._h, N, start.ctypes.data, order.ctypes.data, length.ctypes.data, stride,
                                    ops.ctypes.data, cap)
        if n < 0:
            raise OracleError(n)
        return [tuple(int(v) for v in row) for row in ops[:n]]

    def max_inflight(self, unbounded=MAX_NR):
        return int(_load().orc_max_inflight(self._h, unbounded))

    @property
    def count(self):
        return int(_load().orc_candidate_count(self._h))

    @property
    def lower_bound(self):
        return _load().orc_lower_bound(self._h)

    @property
    def upper_bound(self):
        return _load().orc_upper_bound(self._h)

    @property
    def num_lead_vectors(self):
        return _load().orc_num_lead_vectors(self._h)

    def _pack(self, orders):
        length = _i32([len(o) for o in orders])
        seq = np.full((self.D, self.stride), -1, dtype=np.int32)
        for d, o in enumerate(orders):
            seq[d, :len(o)] = o
        return length, seq

    def eval_index(self, index, want_starts=False):
        sc = OracleScore()
        starts = np.zeros(self.K * self.NR, dtype=np.int32)
        rc = _load().orc_eval_index(self._h, index, C.byref(sc), starts.ctypes.data if want_starts else None)
        if rc:
            raise OracleError(rc)
        out = {"status": sc.status, "period": sc.period, "peak": list(sc.peak[:self.D]), "peak_max": sc.peak_max}
        if want_starts:
            out["starts"] = starts.reshape(self.K, self.NR)
        return out

    def decode(self, index):
        status = C.c_int(0)
        leads = np.zeros(self.K, dtype=np.int32)
        length = np.zeros(self.D, dtype=np.int32)
        seq = np.zeros((self.D, self.stride), dtype=np.int32)
        rc = _load().orc_decode_index(self._h, index, C.byref(status), leads.ctypes.data, length.ctypes.data,
                                      seq.ctypes.data, self.stride)
        if rc:
            raise OracleError(rc)
        return status.value, leads.tolist(), [seq[d, :length[d]].tolist() for d in range(self.D)]

    def eval_explicit(self, leads, orders, want_starts=False):
        length, seq = self._pack(orders)
        leads = _i32(leads)
        sc = OracleScore()
        starts = np.zeros(self.K * self.NR, dtype=np.int32)
        rc = _load().orc_eval_explicit(self._h, leads.ctypes.data, length.ctypes.data, seq.ctypes.data, self.stride,
                                       C.byref(sc), starts.ctypes.data if want_starts else None)
        if rc:
            raise OracleError(rc)
        out = {"status": sc.status, "period": sc.period, "peak": list(sc.peak[:self.D]), "peak_max": sc.peak_max}
        if want_starts:
            out["starts"] = starts.reshape(self.K, self.NR)
        return out

    def repair_explicit(self, leads, orders):
        """the repair rule of the REPAIR space applied to explicit priority lists: repaired per-device orders"""
        length, seq = self._pack(orders)
        leads = _i32(leads)
        out = np.zeros_like(seq)
        rc = _load().orc_repair_explicit(self._h, leads.ctypes.data, length.ctypes.data, seq.ctypes.data, self.stride,
                                         out.ctypes.data)
        if rc:
            raise OracleError(rc)
        return [out[d, :length[d]].tolist() for d in range(self.D)]

    def feasible_explicit(self, leads, orders, T):
        length, seq = self._pack(orders)
        leads = _i32(leads)
        return _load().orc_feasible_explicit(self._h, leads.ctypes.data, length.ctypes.data, seq.ctypes.data,
                                             self.stride, T)

    def sweep(self, first, count, threads=1):
        r = OracleResult()
        if threads > 1:
            rc = _load().orc_sweep_mt(self._h, first, count, threads, C.byref(r))
        else:
            rc = _load().orc_sweep(self._h, first, count, C.byref(r))
        if rc:
            raise OracleError(rc)
        return {"period": r.period, "index": int(r.index), "peak": list(r.peak[:self.D]), "peak_max": r.peak_max,
                "n_evaluated": int(r.n_evaluated), "n_feasible": int(r.n_feasible),
                "n_reject": [int(x) for x in r.n_reject], "ops": int(r.ops)}

    def score_range(self, first, count):
        code = np.zeros(count, dtype=np.int32)
        peak = np.zeros(count, dtype=np.int32)
        rc = _load().orc_score_range(self._h, first, count, code.ctypes.data, peak.ctypes.data)
        if rc:
            raise OracleError(rc)
        return code, peak

    def complete(self, leads, orders, N):
        length, seq = self._pack(orders)
        leads = _i32(leads)
        start = np.full(self.K * N, -1, dtype=np.int32)
        dev_order = np.full((self.D, self.K * N), -1, dtype=np.int32)
        dev_len = np.zeros(self.D, dtype=np.int32)
        rc = _load().orc_complete(self._h, leads.ctypes.data, length.ctypes.data, seq.ctypes.data, self.stride, N,
                                  start.ctypes.data, dev_order.ctypes.data, dev_len.ctypes.data)
        if rc < 0:
            raise OracleError(rc)
        return {"makespan": rc, "start": start.reshape(self.K, N),
                "dev_order": [dev_order[d, :dev_len[d]].tolist() for d in range(self.D)]}
