"""Thin ctypes binding of libchm.so (the C-ABI of include/chm.h): argument marshalling only.

Every step of the path runs in the library's HIP kernels.  Device buffers are torch tensors
(torch is used for device memory and streams, nothing else).  If the library is missing or no
GPU is usable the calls fail loudly; there is no fallback.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# CHM_SANITIZE=1 selects the build whose host code is instrumented with sanitizers (see build.py)
LIB_PATH = os.path.join(_HERE, "libchm_san.so" if os.environ.get("CHM_SANITIZE", "") == "1" else "libchm.so")

OK, ERR_ARG, ERR_RANGE, ERR_OVERFLOW, ERR_UNRECOVERABLE, ERR_NO_FEASIBLE, ERR_HIP, ERR_LIMIT = 0, -1, -2, -3, -4, -5, -6, -7
INFEASIBLE = (1 << 63) - 1

SYMBOLS = ["chm_load_scenario", "chm_plan_space", "chm_score_plans", "chm_score_ranks", "chm_search_best", "chm_search_best_static", "chm_search_best_batch", "chm_kernel_selection",
           "chm_search_range", "chm_search_ranks", "chm_search_cuts", "chm_rank_partitions", "chm_decode_plan", "chm_set_timing", "chm_set_filter_compaction", "chm_set_bounded_search", "chm_get_timing", "chm_family_classes",
           "chm_reroute_shape", "chm_transfer_plan", "chm_replan", "chm_replan_table", "chm_compare_objective", "chm_valu_probe", "chm_free_scenario",
           "chm_strerror"]


class Desc(C.Structure):
    _fields_ = [("L", C.c_int32), ("PP", C.c_int32), ("DP", C.c_int32), ("M", C.c_int32),
                ("fwd_us", C.POINTER(C.c_int32)), ("bwd_us", C.POINTER(C.c_int32)),
                ("mem_mib", C.POINTER(C.c_int32)), ("speed_q16", C.POINTER(C.c_uint32)),
                ("n_failed", C.c_int32), ("failed_nodes", C.POINTER(C.c_int32)),
                ("comm_us", C.c_int32), ("mem_cap_mib", C.c_int32), ("reroute_cap", C.c_int32),
                ("horizon_steps", C.c_int32), ("reconf_us", C.c_int32 * 3),
                ("xfer_us_per_mib", C.c_int32), ("act_mib", C.POINTER(C.c_int32)),
                ("transfer_assign", C.c_int32), ("allreduce_us", C.c_int32)]


class Family(C.Structure):
    _fields_ = [("offset", C.c_uint64), ("n_part", C.c_uint64), ("n_reroute", C.c_uint64),
                ("stages", C.c_int32), ("strategy", C.c_int32)]


class Space(C.Structure):
    _fields_ = [("n_families", C.c_int32), ("fam", Family * 3), ("n_plans", C.c_uint64)]


class Best(C.Structure):
    _fields_ = [("index", C.c_uint64), ("cost", C.c_int64), ("strategy", C.c_int32),
                ("stages", C.c_int32), ("cuts", C.c_uint8 * 32), ("n_affected", C.c_int32),
                ("affected_stage", C.c_int32 * 4), ("reroute", (C.c_uint16 * 16) * 4),
                ("t_step_us", C.c_int64), ("t_trans_us", C.c_int64)]


class ReplanDesc(C.Structure):
    _fields_ = [("L", C.c_int32),
                ("fwd_us", C.POINTER(C.c_int32)), ("bwd_us", C.POINTER(C.c_int32)),
                ("mem_mib", C.POINTER(C.c_int32)), ("act_mib", C.POINTER(C.c_int32)),
                ("old_dp", C.c_int32), ("old_pp", C.c_int32),
                ("n_failed", C.c_int32), ("failed_nodes", C.POINTER(C.c_int32)),
                ("dp_min", C.c_int32), ("dp_max", C.c_int32), ("pp_min", C.c_int32), ("pp_max", C.c_int32),
                ("micro_batches", C.c_int32), ("comm_us", C.c_int32), ("mem_cap_mib", C.c_int32),
                ("horizon_us", C.c_int64), ("restart_us", C.c_int32), ("xfer_us_per_mib", C.c_int32),
                ("allreduce_us", C.c_int32), ("bounded_search", C.c_int32)]


class ReplanPlan(C.Structure):
    _fields_ = [("found", C.c_int32), ("n_candidates", C.c_int32), ("dp", C.c_int32),
                ("length", C.c_int32 * 16), ("micro_batches", C.c_int32 * 16),
                ("cuts", (C.c_uint8 * 32) * 16), ("pipeline_us", C.c_int64 * 16),
                ("t_step_us", C.c_int64), ("fetch_mib", C.c_int64), ("t_trans_us", C.c_int64),
                ("comm_rounds", C.c_int32),
                ("splits_scored", C.c_uint64), ("splits_feasible", C.c_uint64), ("splits_evaluated", C.c_uint64),
                ("algorithmic_ops", C.c_double),
                ("search_ms", C.c_float), ("assign_ms", C.c_float)]


class Selection(C.Structure):
    _fields_ = [("idx_bits", C.c_int32), ("int32_recurrence", C.c_int32), ("present", C.c_int32 * 3),
                ("specialised", C.c_int32 * 3), ("sharp_bound", C.c_int32 * 3), ("reroute_mul24", C.c_int32),
                ("reroute_swept_apart", C.c_int32)]


class Timing(C.Structure):
    _fields_ = [("family_ms", C.c_float * 3), ("total_ms", C.c_float),
                ("partitions", C.c_uint64 * 3), ("evaluations", C.c_uint64 * 3), ("feasible", C.c_uint64 * 3),
                ("evaluated", C.c_uint64 * 3)]


class ChmError(RuntimeError):
    def __init__(self, code, msg=""):
        super().__init__("libchm error %d: %s" % (code, msg))
        self.code = code


_lib = None


def lib():
    """Loads libchm.so; raises if it has not been built (python -m paper_2508_21613_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libchm.so is not built: run `python -m paper_2508_21613_amd.build`")
        # torch brings its own copy of the HIP runtime and must reach the device before the library's does:
        # initialised the other way round, torch reports that no GPU is available
        try:
            import torch
            if torch.cuda.is_available():
                torch.cuda.init()
        except ImportError:
            pass
        L = C.CDLL(LIB_PATH)
        vp = C.c_void_p
        L.chm_load_scenario.argtypes = [C.POINTER(Desc), C.POINTER(vp)]
        L.chm_kernel_selection.argtypes = [C.POINTER(Desc), C.POINTER(Selection)]
        L.chm_plan_space.argtypes = [vp, C.POINTER(Space)]
        L.chm_score_plans.argtypes = [vp, C.c_uint64, C.c_uint64, vp, vp]
        L.chm_score_ranks.argtypes = [vp, C.c_int32, vp, C.c_uint64, vp, vp]
        L.chm_search_best.argtypes = [vp, C.c_uint32, C.POINTER(Best), vp]
        L.chm_search_best_batch.argtypes = [C.POINTER(vp), C.c_int32, C.c_uint32, C.POINTER(Best), C.POINTER(C.c_int32), vp]
        L.chm_search_best_static.argtypes = [vp, C.c_uint32, C.POINTER(Best), vp]
        L.chm_search_range.argtypes = [vp, C.c_int32, C.c_uint64, C.c_uint64, C.POINTER(Best), vp]
        L.chm_search_ranks.argtypes = [vp, C.c_int32, vp, C.c_uint64, vp, C.POINTER(Best), C.POINTER(C.c_uint64), vp]
        L.chm_search_cuts.argtypes = [vp, C.c_int32, vp, C.c_uint64, vp, C.POINTER(Best), C.POINTER(C.c_uint64), vp]
        L.chm_rank_partitions.argtypes = [vp, C.c_int32, vp, C.c_uint64, vp, vp]
        L.chm_decode_plan.argtypes = [vp, C.c_uint64, C.POINTER(Best)]
        L.chm_set_timing.argtypes = [vp, C.c_int32]
        L.chm_set_filter_compaction.argtypes = [vp, C.c_int32, C.POINTER(C.c_float)]
        L.chm_set_bounded_search.argtypes = [vp, C.c_int32]
        L.chm_get_timing.argtypes = [vp, C.POINTER(Timing)]
        L.chm_family_classes.argtypes = [vp, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        L.chm_reroute_shape.argtypes = [vp, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_uint64)]
        L.chm_transfer_plan.argtypes = [vp, C.c_uint64, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_uint8 * 32),
                                        C.POINTER(C.c_uint8 * 32), C.POINTER(C.c_int64), vp]
        L.chm_replan.argtypes = [C.POINTER(ReplanDesc), C.POINTER(ReplanPlan), vp]
        L.chm_replan_table.argtypes = [C.POINTER(ReplanDesc), C.c_int32, C.POINTER(ReplanPlan), vp]
        L.chm_compare_objective.argtypes = [C.c_int64] * 5
        L.chm_valu_probe.argtypes = [C.c_int32, C.c_uint32, C.POINTER(C.c_double), vp]
        L.chm_free_scenario.argtypes = [vp]
        L.chm_free_scenario.restype = None
        L.chm_strerror.argtypes = [C.c_int]
        L.chm_strerror.restype = C.c_char_p
        for n in SYMBOLS:
            if n not in ("chm_free_scenario", "chm_strerror"):
                getattr(L, n).restype = C.c_int
        _lib = L
    return _lib


def strerror(code):
    return lib().chm_strerror(code).decode()


def _check(rc, allowed=()):
    if rc != OK and rc not in allowed:
        raise ChmError(rc, strerror(rc))
    return rc


def _best_dict(b):
    k = max(b.stages - 1, 0)
    return {"index": int(b.index), "cost": int(b.cost), "strategy": int(b.strategy), "stages": int(b.stages),
            "cuts": [int(b.cuts[i]) for i in range(k)], "n_affected": int(b.n_affected),
            "affected_stage": [int(b.affected_stage[a]) for a in range(b.n_affected)],
            "reroute": [[int(b.reroute[a][d]) for d in range(16)] for a in range(b.n_affected)],
            "t_step_us": int(b.t_step_us), "t_trans_us": int(b.t_trans_us)}


def _stream_ptr(stream):
    if stream is None:
        import torch
        return C.c_void_p(torch.cuda.current_stream().cuda_stream)
    return C.c_void_p(stream if isinstance(stream, int) else stream.cuda_stream)


def valu_probe(kind, iters=4000, stream=None):
    """chm_valu_probe: executed int32 lane operations per second of a register-only kernel"""
    out = C.c_double()
    _check(lib().chm_valu_probe(kind, iters, C.byref(out), _stream_ptr(stream)))
    return float(out.value)


def compare_objective(a, b, horizon_us):
    """chm_compare_objective on two plan dicts carrying t_step_us and t_trans_us: 1 if a is better, -1 if b, 0 on a tie"""
    rc = lib().chm_compare_objective(a["t_step_us"], a["t_trans_us"], b["t_step_us"], b["t_trans_us"], horizon_us)
    if rc == -100:
        raise ChmError(ERR_ARG, strerror(ERR_ARG))
    return rc


def _replan_desc(rp):
    """chm_replan_desc of a re-planning dict, and the arrays it points into"""
    keep = []
    d = ReplanDesc()
    d.L = rp["L"]
    for name in ("fwd_us", "bwd_us", "mem_mib", "act_mib"):
        if rp.get(name) is None:
            continue
        a = np.ascontiguousarray(rp[name], dtype=np.int32)
        keep.append(a)
        setattr(d, name, a.ctypes.data_as(C.POINTER(C.c_int32)))
    f = np.ascontiguousarray(rp.get("failed_nodes", []), dtype=np.int32)
    keep.append(f)
    d.n_failed = len(f)
    if len(f):
        d.failed_nodes = f.ctypes.data_as(C.POINTER(C.c_int32))
    for name in ("old_dp", "old_pp", "dp_min", "dp_max", "pp_min", "pp_max", "micro_batches", "comm_us",
                 "mem_cap_mib", "horizon_us", "restart_us", "xfer_us_per_mib"):
        setattr(d, name, int(rp[name]))
    d.allreduce_us = int(rp.get("allreduce_us", 0))
    d.bounded_search = int(rp.get("bounded_search", 0))
    return d, keep


def _replan_stats(p):
    return {"splits_scored": int(p.splits_scored), "splits_feasible": int(p.splits_feasible),
            "splits_evaluated": int(p.splits_evaluated),
            "algorithmic_ops": float(p.algorithmic_ops), "search_ms": float(p.search_ms), "assign_ms": float(p.assign_ms)}


def replan(rp, stream=None, with_stats=False):
    """chm_replan: search over DP/PP degrees for the nodes that survive (Algorithm 1).  `rp` is a dict with the
    fields of chm_replan_desc; returns a dict with the plan fields of chm_replan_plan (and, with_stats, a second
    dict with the work accounting of the call)."""
    d, keep = _replan_desc(rp)
    p = ReplanPlan()
    _check(lib().chm_replan(C.byref(d), C.byref(p), _stream_ptr(stream)))
    plan = _replan_dict(p)
    return (plan, _replan_stats(p)) if with_stats else plan


def replan_table(rp, k=None, stream=None, with_stats=False):
    """chm_replan_table: the re-plans after the first 1 .. k nodes of rp["failed_nodes"] have failed"""
    d, keep = _replan_desc(rp)
    k = d.n_failed if k is None else int(k)
    plans = (ReplanPlan * max(k, 1))()
    _check(lib().chm_replan_table(C.byref(d), k, plans, _stream_ptr(stream)))
    out = [_replan_dict(plans[i]) for i in range(k)]
    return (out, [_replan_stats(plans[i]) for i in range(k)]) if with_stats else out


def _replan_dict(p):
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


def _desc(sc):
    """chm_scenario_desc of a scenario dict, and the arrays it points into (keep them alive for the call)"""
    keep = []
    d = Desc()
    d.L, d.PP, d.DP, d.M = sc["L"], sc["PP"], sc["DP"], sc["M"]
    for name in ("fwd_us", "bwd_us", "mem_mib"):
        a = np.ascontiguousarray(sc[name], dtype=np.int32)
        keep.append(a)
        setattr(d, name, a.ctypes.data_as(C.POINTER(C.c_int32)))
    if sc.get("speed_q16") is not None:
        a = np.ascontiguousarray(sc["speed_q16"], dtype=np.uint32)
        keep.append(a)
        d.speed_q16 = a.ctypes.data_as(C.POINTER(C.c_uint32))
    f = np.ascontiguousarray(sc.get("failed_nodes", []), dtype=np.int32)
    keep.append(f)
    d.n_failed = len(f)
    if len(f):
        d.failed_nodes = f.ctypes.data_as(C.POINTER(C.c_int32))
    d.comm_us, d.mem_cap_mib = sc["comm_us"], sc["mem_cap_mib"]
    d.reroute_cap, d.horizon_steps = sc.get("reroute_cap", 0), sc["horizon_steps"]
    for i in range(3):
        d.reconf_us[i] = sc["reconf_us"][i]
    d.xfer_us_per_mib = sc["xfer_us_per_mib"]
    if sc.get("act_mib") is not None:
        a = np.ascontiguousarray(sc["act_mib"], dtype=np.int32)
        keep.append(a)
        d.act_mib = a.ctypes.data_as(C.POINTER(C.c_int32))
    d.transfer_assign = int(sc.get("transfer_assign", 0))
    d.allreduce_us = int(sc.get("allreduce_us", 0))
    return d, keep


def kernel_selection(sc):
    """chm_kernel_selection: which kernels a scenario would run on (host only)"""
    d, keep = _desc(sc)
    out = Selection()
    _check(lib().chm_kernel_selection(C.byref(d), C.byref(out)))
    return {"idx_bits": int(out.idx_bits), "int32_recurrence": bool(out.int32_recurrence),
            "present": [bool(x) for x in out.present], "specialised": [bool(x) for x in out.specialised],
            "sharp_bound": [bool(x) for x in out.sharp_bound], "reroute_mul24": bool(out.reroute_mul24),
            "reroute_swept_apart": bool(out.reroute_swept_apart)}


def search_best_batch(scenarios, mask=7, stream=None):
    """chm_search_best_batch over a list of Scenario objects: [(code, best plan)] in the same order"""
    n = len(scenarios)
    handles = (C.c_void_p * max(n, 1))(*[g._h for g in scenarios])
    outs = (Best * max(n, 1))()
    codes = (C.c_int32 * max(n, 1))()
    _check(lib().chm_search_best_batch(handles, n, mask, outs, codes, _stream_ptr(stream)))
    return [(int(codes[i]), _best_dict(outs[i])) for i in range(n)]


class Scenario:
    """chm_load_scenario ... chm_free_scenario.  `sc` is a dict with the fields of chm_scenario_desc."""

    def __init__(self, sc):
        d, keep = _desc(sc)
        self._h = C.c_void_p()
        _check(lib().chm_load_scenario(C.byref(d), C.byref(self._h)))
        sp = Space()
        _check(lib().chm_plan_space(self._h, C.byref(sp)))
        self.n_plans = int(sp.n_plans)
        self.families = [dict(offset=int(sp.fam[i].offset), n_part=int(sp.fam[i].n_part),
                              n_reroute=int(sp.fam[i].n_reroute), stages=int(sp.fam[i].stages),
                              strategy=int(sp.fam[i].strategy)) for i in range(sp.n_families)]

    def close(self):
        if getattr(self, "_h", None):
            lib().chm_free_scenario(self._h)
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

    def score_plans(self, first, count, out=None, stream=None):
        """chm_score_plans into a torch int64 CUDA tensor (allocated here unless given)"""
        import torch
        if out is None:
            out = torch.empty(count, dtype=torch.int64, device="cuda")
        assert out.is_cuda and out.dtype == torch.int64 and out.numel() >= count and out.is_contiguous()
        _check(lib().chm_score_plans(self._h, first, count, C.c_void_p(out.data_ptr()), _stream_ptr(stream)))
        return out

    def score_ranks(self, strategy, d_ranks, out=None, stream=None):
        """chm_score_ranks; d_ranks is a contiguous CUDA tensor holding uint64 ranks (dtype int64 or uint64)"""
        import torch
        n = d_ranks.numel()
        assert d_ranks.is_cuda and d_ranks.element_size() == 8 and d_ranks.is_contiguous()
        if out is None:
            out = torch.empty(n, dtype=torch.int64, device="cuda")
        _check(lib().chm_score_ranks(self._h, strategy, C.c_void_p(d_ranks.data_ptr()), n,
                                     C.c_void_p(out.data_ptr()), _stream_ptr(stream)))
        return out

    def search_best(self, mask=7, stream=None):
        b = Best()
        rc = _check(lib().chm_search_best(self._h, mask, C.byref(b), _stream_ptr(stream)),
                    allowed=(ERR_NO_FEASIBLE, ERR_UNRECOVERABLE))
        return rc, _best_dict(b)

    def search_best_static(self, mask=7, stream=None):
        """chm_search_best_static: chm_search_best with its scratch in the library's fixed device array"""
        b = Best()
        rc = _check(lib().chm_search_best_static(self._h, mask, C.byref(b), _stream_ptr(stream)),
                    allowed=(ERR_NO_FEASIBLE, ERR_UNRECOVERABLE, ERR_LIMIT))
        return rc, _best_dict(b)

    def search_range(self, strategy, first, count, stream=None):
        b = Best()
        rc = _check(lib().chm_search_range(self._h, strategy, first, count, C.byref(b), _stream_ptr(stream)),
                    allowed=(ERR_NO_FEASIBLE, ERR_UNRECOVERABLE))
        return rc, _best_dict(b)

    def rank_partitions(self, strategy, d_cuts, out=None, stream=None):
        """chm_rank_partitions: (n, stages-1) uint8 CUDA tensor of cut positions -> int64 tensor of ranks"""
        import torch
        assert d_cuts.is_cuda and d_cuts.dtype == torch.uint8 and d_cuts.is_contiguous() and d_cuts.dim() == 2
        assert d_cuts.shape[1] == self.family(strategy)["stages"] - 1
        n = d_cuts.shape[0]
        if out is None:
            out = torch.empty(n, dtype=torch.int64, device="cuda")
        _check(lib().chm_rank_partitions(self._h, strategy, C.c_void_p(d_cuts.data_ptr()), n,
                                         C.c_void_p(out.data_ptr()), _stream_ptr(stream)))
        return out

    def search_ranks(self, strategy, d_ranks, costs=None, stream=None):
        """chm_search_ranks: argmin over explicit partition ranks held in a CUDA tensor"""
        b = Best()
        pos = C.c_uint64()
        n = d_ranks.numel()
        assert d_ranks.is_cuda and d_ranks.element_size() == 8 and d_ranks.is_contiguous()
        cp = C.c_void_p(costs.data_ptr()) if costs is not None else None
        rc = _check(lib().chm_search_ranks(self._h, strategy, C.c_void_p(d_ranks.data_ptr()), n, cp, C.byref(b),
                                           C.byref(pos), _stream_ptr(stream)),
                    allowed=(ERR_NO_FEASIBLE, ERR_UNRECOVERABLE))
        return rc, _best_dict(b), int(pos.value)

    def search_cuts(self, strategy, d_cuts, costs=None, stream=None):
        """chm_search_cuts: argmin over explicit partitions given as an (n, stages-1) uint8 CUDA tensor of cut positions"""
        import torch
        b = Best()
        pos = C.c_uint64()
        assert d_cuts.is_cuda and d_cuts.dtype == torch.uint8 and d_cuts.is_contiguous() and d_cuts.dim() == 2
        assert d_cuts.shape[1] == self.family(strategy)["stages"] - 1
        cp = C.c_void_p(costs.data_ptr()) if costs is not None else None
        rc = _check(lib().chm_search_cuts(self._h, strategy, C.c_void_p(d_cuts.data_ptr()), d_cuts.shape[0], cp, C.byref(b),
                                          C.byref(pos), _stream_ptr(stream)),
                    allowed=(ERR_NO_FEASIBLE, ERR_UNRECOVERABLE))
        return rc, _best_dict(b), int(pos.value)

    def decode_plan(self, index):
        b = Best()
        _check(lib().chm_decode_plan(self._h, index, C.byref(b)))
        return _best_dict(b)

    def family_classes(self, strategy):
        """[(stages, micro-batches)] of the distinct pipelines one plan of the strategy evaluates"""
        n = C.c_int32()
        ln, mb = (C.c_int32 * 16)(), (C.c_int32 * 16)()
        _check(lib().chm_family_classes(self._h, strategy, C.byref(n), ln, mb))
        return [(int(ln[i]), int(mb[i])) for i in range(n.value)]

    def reroute_shape(self):
        """[(surviving peers, valid reroute vectors)] per stage that lost nodes"""
        n = C.c_int32()
        peers, vecs = (C.c_int32 * 4)(), (C.c_uint64 * 4)()
        _check(lib().chm_reroute_shape(self._h, C.byref(n), peers, vecs))
        return [(int(peers[a]), int(vecs[a])) for a in range(n.value)]

    def transfer_plan(self, part_rank, pipeline, stream=None):
        """chm_transfer_plan: (fault-free stage of every surviving node, new stage it hosts, MiB fetched in total)"""
        n, mib = C.c_int32(), C.c_int64()
        node_stage, stage_of_node = (C.c_uint8 * 32)(), (C.c_uint8 * 32)()
        _check(lib().chm_transfer_plan(self._h, C.c_uint64(part_rank), pipeline, C.byref(n), C.byref(node_stage), C.byref(stage_of_node),
                                       C.byref(mib), _stream_ptr(stream)))
        return [int(node_stage[i]) for i in range(n.value)], [int(stage_of_node[i]) for i in range(n.value)], int(mib.value)

    def set_timing(self, on=True):
        _check(lib().chm_set_timing(self._h, 1 if on else 0))

    def set_filter_compaction(self, mode=-1):
        """chm_set_filter_compaction: -1 automatic, 0 off, 1 on; returns the sampled share of partitions that fit, per strategy"""
        share = (C.c_float * 3)()
        _check(lib().chm_set_filter_compaction(self._h, mode, share))
        return [float(x) for x in share]

    def set_bounded_search(self, on=True):
        """chm_set_bounded_search: skip partitions whose lower bound of the cost lies above the best cost found so far"""
        _check(lib().chm_set_bounded_search(self._h, int(on)))

    def get_timing(self):
        t = Timing()
        _check(lib().chm_get_timing(self._h, C.byref(t)))
        return {"family_ms": [float(x) for x in t.family_ms], "total_ms": float(t.total_ms),
                "partitions": [int(x) for x in t.partitions], "evaluations": [int(x) for x in t.evaluations], "feasible": [int(x) for x in t.feasible],
                "evaluated": [int(x) for x in t.evaluated]}
