"""ctypes front end of the CPU oracle (oracle/chm_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the benchmark's
CPU-baseline leg.  It does not import the HIP package and the HIP package does not
import it.  Arrays go in as numpy arrays; nothing here does any of the method's
arithmetic.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# ORC_SANITIZE=1: the oracle built with AddressSanitizer and UndefinedBehaviorSanitizer (host code only), as a
# library of its own.  The interpreter is not instrumented, so the sanitizer runtime has to be loaded first:
#   ORC_SANITIZE=1 LD_PRELOAD=$(gcc -print-file-name=libasan.so) ASAN_OPTIONS=detect_leaks=0 \
#       python -m pytest tests/test_oracle_pins.py tests/test_full_space_script.py -q
SANITIZE = os.environ.get("ORC_SANITIZE", "") == "1"
_LIB_PATH = os.path.join(_HERE, "liborc_san.so" if SANITIZE else "liborc.so")
_SRC = os.path.join(_HERE, "chm_oracle.cpp")

OK, ERR_ARG, ERR_RANGE, ERR_OVERFLOW, ERR_UNRECOVERABLE, ERR_NO_FEASIBLE = 0, -1, -2, -3, -4, -5
INF = np.iinfo(np.int64).max


def build(force=False):
    """Compile the oracle with the host compiler (-O2, single-threaded code)."""
    if not force and os.path.exists(_LIB_PATH) and os.path.getmtime(_LIB_PATH) >= max(
            os.path.getmtime(_SRC), os.path.getmtime(os.path.join(_HERE, "chm_oracle.h"))):
        return _LIB_PATH
    opt = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"] if SANITIZE else ["-O2"]
    cmd = ["g++"] + opt + ["-std=c++17", "-fPIC", "-shared", "-Wall", "-o", _LIB_PATH, _SRC]
    subprocess.run(cmd, check=True)
    return _LIB_PATH


class Desc(C.Structure):
    _fields_ = [("L", C.c_int32), ("PP", C.c_int32), ("DP", C.c_int32), ("M", C.c_int32),
                ("fwd_us", C.POINTER(C.c_int32)), ("bwd_us", C.POINTER(C.c_int32)),
                ("mem_mib", C.POINTER(C.c_int32)), ("speed_q16", C.POINTER(C.c_uint32)),
                ("n_failed", C.c_int32), ("failed_nodes", C.POINTER(C.c_int32)),
                ("comm_us", C.c_int32), ("mem_cap_mib", C.c_int32), ("reroute_cap", C.c_int32),
                ("horizon_steps", C.c_int32), ("reconf_us", C.c_int32 * 3),
                ("xfer_us_per_mib", C.c_int32), ("act_mib", C.POINTER(C.c_int32)),
                ("transfer_assign", C.c_int32), ("allreduce_us", C.c_int32)]


class ReplanDesc(C.Structure):
    _fields_ = [("L", C.c_int32),
                ("fwd_us", C.POINTER(C.c_int32)), ("bwd_us", C.POINTER(C.c_int32)),
                ("mem_mib", C.POINTER(C.c_int32)), ("act_mib", C.POINTER(C.c_int32)),
                ("old_dp", C.c_int32), ("old_pp", C.c_int32),
                ("n_failed", C.c_int32), ("failed_nodes", C.POINTER(C.c_int32)),
                ("dp_min", C.c_int32), ("dp_max", C.c_int32), ("pp_min", C.c_int32), ("pp_max", C.c_int32),
                ("micro_batches", C.c_int32), ("comm_us", C.c_int32), ("mem_cap_mib", C.c_int32),
                ("horizon_us", C.c_int64), ("restart_us", C.c_int32), ("xfer_us_per_mib", C.c_int32),
                ("allreduce_us", C.c_int32)]


class ReplanPlan(C.Structure):
    _fields_ = [("found", C.c_int32), ("n_candidates", C.c_int32), ("dp", C.c_int32),
                ("length", C.c_int32 * 16), ("micro_batches", C.c_int32 * 16),
                ("cuts", (C.c_uint8 * 32) * 16), ("pipeline_us", C.c_int64 * 16),
                ("t_step_us", C.c_int64), ("fetch_mib", C.c_int64), ("t_trans_us", C.c_int64),
                ("comm_rounds", C.c_int32)]


class Family(C.Structure):
    _fields_ = [("offset", C.c_uint64), ("n_part", C.c_uint64), ("n_reroute", C.c_uint64),
                ("stages", C.c_int32), ("strategy", C.c_int32)]


class Space(C.Structure):
    _fields_ = [("n_families", C.c_int32), ("fam", Family * 3), ("n_plans", C.c_uint64)]


class Plan(C.Structure):
    _fields_ = [("index", C.c_uint64), ("cost", C.c_int64), ("strategy", C.c_int32),
                ("stages", C.c_int32), ("cuts", C.c_uint8 * 32), ("n_affected", C.c_int32),
                ("affected_stage", C.c_int32 * 4), ("reroute", (C.c_uint16 * 16) * 4),
                ("t_step_us", C.c_int64), ("t_trans_us", C.c_int64)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB_PATH)
        u8p, u16p, i32p, i64p, u64p = (C.POINTER(t) for t in (C.c_uint8, C.c_uint16, C.c_int32, C.c_int64, C.c_uint64))
        sig = {
            "orc_binom": (C.c_uint64, [C.c_int32, C.c_int32]),
            "orc_partition_rank": (C.c_uint64, [C.c_int32, u8p]),
            "orc_partition_rank_batch": (None, [C.c_int32, u8p, C.c_uint64, u64p]),
            "orc_partition_unrank": (C.c_int, [C.c_int32, C.c_int32, C.c_uint64, u8p]),
            "orc_reroute_count": (C.c_uint64, [C.c_int32, C.c_int32, C.c_int32]),
            "orc_reroute_unrank": (C.c_int, [C.c_int32, C.c_int32, C.c_int32, C.c_uint64, u16p]),
            "orc_reroute_rank": (C.c_uint64, [C.c_int32, C.c_int32, C.c_int32, u16p]),
            "orc_scale_q16": (C.c_int64, [C.c_int64, C.c_uint32]),
            "orc_makespan_1f1b": (C.c_int64, [C.c_int32, i64p, i64p, C.c_int32]),
            "orc_missing_interval": (C.c_int64, [i64p, C.c_int32, C.c_int32, C.c_int32, C.c_int32]),
            "orc_distribute_batch": (None, [C.c_int32, C.c_int32, i32p, i32p]),
            "orc_layout_p0": (None, [C.c_int32, C.c_int32, i32p]),
            "orc_min_assignment": (C.c_int64, [C.c_int32, i64p, i32p]),
            "orc_integer_partition": (C.c_int, [C.c_int32, C.c_int32, C.c_int32, C.c_int32, i32p]),
            "orc_best_split": (C.c_int64, [C.c_int32, i32p, i32p, i32p, i32p, C.c_int32, C.c_int32, C.c_int32, u8p]),
            "orc_replan": (C.c_int, [C.POINTER(ReplanDesc), C.POINTER(ReplanPlan)]),
            "orc_comm_rounds": (C.c_int32, [C.c_int32, C.c_int32, u8p]),
            "orc_open": (C.c_int, [C.POINTER(Desc), C.POINTER(C.c_void_p)]),
            "orc_close": (None, [C.c_void_p]),
            "orc_plan_space": (C.c_int, [C.c_void_p, C.POINTER(Space)]),
            "orc_decode": (C.c_int, [C.c_void_p, C.c_uint64, C.POINTER(Plan)]),
            "orc_plan_cost": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, u8p, u16p, i64p]),
            "orc_score": (C.c_int, [C.c_void_p, C.c_uint64, C.c_uint64, i64p]),
            "orc_score_ranks": (C.c_int, [C.c_void_p, C.c_int32, u64p, C.c_uint64, i64p]),
            "orc_search": (C.c_int, [C.c_void_p, C.c_uint32, C.POINTER(Plan)]),
            "orc_search_range": (C.c_int, [C.c_void_p, C.c_int32, C.c_uint64, C.c_uint64, C.POINTER(Plan), u64p]),
            "orc_search_range_counted": (C.c_int, [C.c_void_p, C.c_int32, C.c_uint64, C.c_uint64, C.POINTER(Plan), u64p]),
            "orc_search_joint": (C.c_int, [C.c_void_p, C.c_uint64, C.c_uint64, C.POINTER(Plan)]),
        }
        for name, (res, args) in sig.items():
            f = getattr(L, name)
            f.restype, f.argtypes = res, args
        _lib = L
    return _lib


def _ptr(a, t):
    return a.ctypes.data_as(C.POINTER(t))


class OracleError(RuntimeError):
    def __init__(self, code):
        super().__init__("oracle error %d" % code)
        self.code = code


def binom(n, k):
    return int(lib().orc_binom(n, k))


def partition_rank(cuts):
    a = np.ascontiguousarray(cuts, dtype=np.uint8)
    return int(lib().orc_partition_rank(len(a), _ptr(a, C.c_uint8)))


def partition_rank_batch(cuts):
    """ranks of an (n, k) uint8 array of cut positions"""
    a = np.ascontiguousarray(cuts, dtype=np.uint8)
    out = np.empty(a.shape[0], dtype=np.uint64)
    lib().orc_partition_rank_batch(a.shape[1], _ptr(a, C.c_uint8), a.shape[0], _ptr(out, C.c_uint64))
    return out


def partition_unrank(L, k, rank):
    a = np.zeros(max(k, 1), dtype=np.uint8)
    rc = lib().orc_partition_unrank(L, k, rank, _ptr(a, C.c_uint8))
    if rc:
        raise OracleError(rc)
    return [int(x) for x in a[:k]]


def reroute_count(parts, total, cap):
    return int(lib().orc_reroute_count(parts, total, cap))


def reroute_unrank(parts, total, cap, rank):
    a = np.zeros(max(parts, 1), dtype=np.uint16)
    rc = lib().orc_reroute_unrank(parts, total, cap, rank, _ptr(a, C.c_uint16))
    if rc:
        raise OracleError(rc)
    return [int(x) for x in a[:parts]]


def reroute_rank(parts, total, cap, r):
    a = np.ascontiguousarray(r, dtype=np.uint16)
    return int(lib().orc_reroute_rank(parts, total, cap, _ptr(a, C.c_uint16)))


def scale_q16(x, q):
    return int(lib().orc_scale_q16(int(x), int(q)))


def makespan_1f1b(F, B, M):
    f = np.ascontiguousarray(F, dtype=np.int64)
    b = np.ascontiguousarray(B, dtype=np.int64)
    assert len(f) == len(b)
    return int(lib().orc_makespan_1f1b(len(f), _ptr(f, C.c_int64), _ptr(b, C.c_int64), int(M)))


def missing_interval(mem, a, b, a0, b0):
    pw = np.concatenate([[0], np.cumsum(np.asarray(mem, dtype=np.int64))]).astype(np.int64)
    return int(lib().orc_missing_interval(_ptr(pw, C.c_int64), a, b, a0, b0))


def distribute_batch(total, nodes):
    n = np.ascontiguousarray(nodes, dtype=np.int32)
    out = np.zeros(len(n), dtype=np.int32)
    lib().orc_distribute_batch(len(n), int(total), _ptr(n, C.c_int32), _ptr(out, C.c_int32))
    return [int(x) for x in out]


def layout_p0(L, S):
    out = np.zeros(S + 1, dtype=np.int32)
    lib().orc_layout_p0(L, S, _ptr(out, C.c_int32))
    return [int(x) for x in out]


def min_assignment(cost):
    """(minimum total, position of every node) for a square cost matrix cost[node][position]"""
    c = np.ascontiguousarray(cost, dtype=np.int64)
    assert c.ndim == 2 and c.shape[0] == c.shape[1]
    pos = np.zeros(c.shape[0], dtype=np.int32)
    total = lib().orc_min_assignment(c.shape[0], _ptr(c, C.c_int64), _ptr(pos, C.c_int32))
    return int(total), [int(x) for x in pos]


def comm_rounds(holds):
    """greedy colouring rounds for a (devices x layers) 0/1 array of which device holds which layer"""
    h = np.ascontiguousarray(holds, dtype=np.uint8)
    assert h.ndim == 2
    return int(lib().orc_comm_rounds(h.shape[1], h.shape[0], _ptr(h, C.c_uint8)))


def integer_partition(n, dp, pp_min, pp_max):
    """pipeline lengths, or None when the split is impossible within the range"""
    out = np.zeros(max(int(dp), 1), dtype=np.int32)
    ok = lib().orc_integer_partition(n, dp, pp_min, pp_max, _ptr(out, C.c_int32))
    return [int(x) for x in out[:dp]] if ok else None


def best_split(fwd, bwd, mem, act, n, M, cap):
    """(least 1F1B time or INF, cuts) over all contiguous splits into n stages that fit"""
    f, b, m = (np.ascontiguousarray(x, dtype=np.int32) for x in (fwd, bwd, mem))
    a = np.ascontiguousarray(act, dtype=np.int32) if act is not None else None
    cuts = np.zeros(32, dtype=np.uint8)
    t = lib().orc_best_split(len(f), _ptr(f, C.c_int32), _ptr(b, C.c_int32), _ptr(m, C.c_int32),
                             _ptr(a, C.c_int32) if a is not None else None, n, M, cap, _ptr(cuts, C.c_uint8))
    return int(t), [int(x) for x in cuts[:n - 1]]


def replan_dict(p):
    """plain dict of a re-planning result structure (field names shared by oracle and library)"""
    if not p.found:
        return {"found": False, "n_candidates": int(p.n_candidates)}
    dp = int(p.dp)
    return {"found": True, "n_candidates": int(p.n_candidates), "dp": dp,
            "length": [int(p.length[i]) for i in range(dp)],
            "micro_batches": [int(p.micro_batches[i]) for i in range(dp)],
            "cuts": [[int(p.cuts[i][j]) for j in range(p.length[i] - 1)] for i in range(dp)],
            "pipeline_us": [int(p.pipeline_us[i]) for i in range(dp)],
            "t_step_us": int(p.t_step_us), "fetch_mib": int(p.fetch_mib), "t_trans_us": int(p.t_trans_us),
            "comm_rounds": int(p.comm_rounds)}


def replan(rp):
    """orc_replan on a dict as produced by the seeded generators (synth.replan_case)"""
    keep = []
    d = ReplanDesc()
    d.L = rp["L"]
    for name in ("fwd_us", "bwd_us", "mem_mib", "act_mib"):
        if rp.get(name) is None:
            continue
        a = np.ascontiguousarray(rp[name], dtype=np.int32)
        keep.append(a)
        setattr(d, name, _ptr(a, C.c_int32))
    f = np.ascontiguousarray(rp.get("failed_nodes", []), dtype=np.int32)
    keep.append(f)
    d.n_failed = len(f)
    if len(f):
        d.failed_nodes = _ptr(f, C.c_int32)
    for name in ("old_dp", "old_pp", "dp_min", "dp_max", "pp_min", "pp_max", "micro_batches", "comm_us",
                 "mem_cap_mib", "horizon_us", "restart_us", "xfer_us_per_mib"):
        setattr(d, name, int(rp[name]))
    d.allreduce_us = int(rp.get("allreduce_us", 0))
    out = ReplanPlan()
    rc = lib().orc_replan(C.byref(d), C.byref(out))
    if rc:
        raise OracleError(rc)
    return replan_dict(out)


def _plan_dict(p):
    k = p.stages - 1
    d = {"index": int(p.index), "cost": int(p.cost), "strategy": int(p.strategy), "stages": int(p.stages),
         "cuts": [int(p.cuts[i]) for i in range(k)], "n_affected": int(p.n_affected),
         "affected_stage": [int(p.affected_stage[a]) for a in range(p.n_affected)],
         "reroute": [[int(p.reroute[a][d]) for d in range(16)] for a in range(p.n_affected)],
         "t_step_us": int(p.t_step_us), "t_trans_us": int(p.t_trans_us)}
    return d


class Scenario:
    """One failure scenario held by the oracle.  `sc` is a dict as produced by the seeded
    input generators: L, PP, DP, M, fwd_us, bwd_us, mem_mib, speed_q16 (or None),
    failed_nodes, comm_us, mem_cap_mib, reroute_cap, horizon_steps, reconf_us, xfer_us_per_mib,
    act_mib (or None), transfer_assign (0/1)."""

    def __init__(self, sc):
        self._keep = []
        d = Desc()
        d.L, d.PP, d.DP, d.M = sc["L"], sc["PP"], sc["DP"], sc["M"]
        for name in ("fwd_us", "bwd_us", "mem_mib"):
            a = np.ascontiguousarray(sc[name], dtype=np.int32)
            self._keep.append(a)
            setattr(d, name, _ptr(a, C.c_int32))
        if sc.get("speed_q16") is not None:
            a = np.ascontiguousarray(sc["speed_q16"], dtype=np.uint32)
            self._keep.append(a)
            d.speed_q16 = _ptr(a, C.c_uint32)
        f = np.ascontiguousarray(sc.get("failed_nodes", []), dtype=np.int32)
        self._keep.append(f)
        d.n_failed = len(f)
        if len(f):
            d.failed_nodes = _ptr(f, C.c_int32)
        d.comm_us, d.mem_cap_mib = sc["comm_us"], sc["mem_cap_mib"]
        d.reroute_cap, d.horizon_steps = sc.get("reroute_cap", 0), sc["horizon_steps"]
        for i in range(3):
            d.reconf_us[i] = sc["reconf_us"][i]
        d.xfer_us_per_mib = sc["xfer_us_per_mib"]
        if sc.get("act_mib") is not None:
            a = np.ascontiguousarray(sc["act_mib"], dtype=np.int32)
            self._keep.append(a)
            d.act_mib = _ptr(a, C.c_int32)
        d.transfer_assign = int(sc.get("transfer_assign", 0))
        d.allreduce_us = int(sc.get("allreduce_us", 0))
        h = C.c_void_p()
        rc = lib().orc_open(C.byref(d), C.byref(h))
        if rc:
            raise OracleError(rc)
        self._h = h
        sp = Space()
        lib().orc_plan_space(self._h, C.byref(sp))
        self.n_plans = int(sp.n_plans)
        self.families = [dict(offset=int(sp.fam[i].offset), n_part=int(sp.fam[i].n_part),
                              n_reroute=int(sp.fam[i].n_reroute), stages=int(sp.fam[i].stages),
                              strategy=int(sp.fam[i].strategy)) for i in range(sp.n_families)]

    def close(self):
        if self._h:
            lib().orc_close(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def family(self, strategy):
        for f in self.families:
            if f["strategy"] == strategy:
                return f
        return None

    def decode(self, index):
        p = Plan()
        rc = lib().orc_decode(self._h, index, C.byref(p))
        if rc:
            raise OracleError(rc)
        return _plan_dict(p)

    def plan_cost(self, strategy, cuts, reroute=None):
        c = np.ascontiguousarray(cuts, dtype=np.uint8)
        r = np.zeros(64, dtype=np.uint16)
        if reroute is not None:
            for a, row in enumerate(reroute):
                r[a * 16:a * 16 + len(row)] = row
        out = C.c_int64()
        rc = lib().orc_plan_cost(self._h, strategy, len(c), _ptr(c, C.c_uint8) if len(c) else None,
                                 _ptr(r, C.c_uint16), C.byref(out))
        if rc:
            raise OracleError(rc)
        return int(out.value)

    def score(self, first, count):
        out = np.empty(count, dtype=np.int64)
        rc = lib().orc_score(self._h, first, count, _ptr(out, C.c_int64))
        if rc:
            raise OracleError(rc)
        return out

    def score_ranks(self, strategy, ranks):
        r = np.ascontiguousarray(ranks, dtype=np.uint64)
        out = np.empty(len(r), dtype=np.int64)
        rc = lib().orc_score_ranks(self._h, strategy, _ptr(r, C.c_uint64), len(r), _ptr(out, C.c_int64))
        if rc:
            raise OracleError(rc)
        return out

    def search(self, mask=7):
        p = Plan()
        rc = lib().orc_search(self._h, mask, C.byref(p))
        return rc, _plan_dict(p)

    def search_range(self, strategy, first, count):
        p = Plan()
        ev = C.c_uint64()
        rc = lib().orc_search_range(self._h, strategy, first, count, C.byref(p), C.byref(ev))
        return rc, _plan_dict(p), int(ev.value)

    def search_range_counted(self, strategy, first, count):
        """(return code, best plan of the range, partitions of the range that pass the memory filter)"""
        p = Plan()
        fit = C.c_uint64()
        rc = lib().orc_search_range_counted(self._h, strategy, first, count, C.byref(p), C.byref(fit))
        return rc, _plan_dict(p), int(fit.value)

    def search_joint(self, first=0, count=None):
        p = Plan()
        if count is None:
            count = self.n_plans - first
        rc = lib().orc_search_joint(self._h, first, count, C.byref(p))
        return rc, _plan_dict(p)
