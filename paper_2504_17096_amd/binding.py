"""Thin ctypes binding of libsailor.so (same names as include/sailor.h).

Argument marshalling only: every step of plan evaluation and selection runs in the
library's HIP kernels.  torch is used by callers for device memory and streams; this
module accepts raw device pointers (ints) or torch tensors.  There is no CPU fallback:
a missing library raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsailor.so")

SAILOR_OK, SAILOR_EINVAL, SAILOR_ENOMEM, SAILOR_EDEVICE, SAILOR_ERANGE, SAILOR_ENOFEASIBLE = \
    0, -1, -2, -3, -4, -5
MAX_THROUGHPUT, MIN_COST = 0, 1
MASK_OOM, MASK_OVER_QUOTA, MASK_BATCH_INDIVISIBLE, MASK_TP_EXCEEDS_NODE, MASK_CONSTRAINT = \
    1, 2, 4, 8, 32
MAX_K = 4096

EXPORTS = ["sailor_plan_create", "sailor_plan_destroy", "sailor_plan_set_avail",
           "sailor_plan_num_candidates", "sailor_plan_decode", "sailor_eval_batch",
           "sailor_best_plan", "sailor_topk", "sailor_plan_set_scratch", "sailor_plan_set_timing",
           "sailor_plan_last_timing", "sailor_plan_last_counts", "sailor_simulate_1f1b",
           "sailor_simulate_1f1b_static", "sailor_plan_set_incremental", "sailor_plan_last_scan",
           "sailor_search", "sailor_eval_placements", "sailor_eval_replica_placements",
           "sailor_set_scan_unit_parts"]


class SailorError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: sailor_status {status}")
        self.status = status


class sailor_problem(C.Structure):
    _fields_ = [
        ("n_layers", C.c_int32), ("n_types", C.c_int32), ("n_zones", C.c_int32),
        ("n_mb", C.c_int32), ("n_tp", C.c_int32), ("n_dp", C.c_int32), ("n_pp", C.c_int32),
        ("max_segments", C.c_int32), ("seg3_max_pp", C.c_int32), ("uniform_layers", C.c_int32),
        ("per_segment_tp", C.c_int32), ("n_bw_coef", C.c_int32),
        ("mixed_types", C.c_int32),
        ("global_batch", C.c_int64),
        ("mb_values", C.c_void_p), ("tp_values", C.c_void_p), ("dp_values", C.c_void_p),
        ("pp_values", C.c_void_p), ("n_partitions", C.c_void_p), ("partition_layers", C.c_void_p),
        ("layer_params", C.c_void_p),
        ("embed_params", C.c_uint64), ("head_params", C.c_uint64),
        ("bytes_per_param", C.c_uint32), ("grad_bytes_per_param", C.c_uint32),
        ("t_fwd", C.c_void_p), ("t_bwd", C.c_void_p), ("t_upd", C.c_void_p),
        ("act_store_bytes", C.c_void_p), ("p2p_bytes", C.c_void_p),
        ("mem_capacity", C.c_void_p), ("mem_reserved", C.c_void_p),
        ("gpus_per_node", C.c_void_p), ("price_per_hour", C.c_void_p),
        ("avail", C.c_void_p), ("bandwidth", C.c_void_p), ("egress_per_byte", C.c_void_p),
        ("bw_poly", C.c_void_p),
    ]


class sailor_constraint(C.Structure):
    _fields_ = [("bound", C.c_double), ("has_bound", C.c_int32)]


class sailor_result(C.Structure):
    _fields_ = [
        ("index", C.c_uint64), ("peak_mem_bytes", C.c_uint64),
        ("iter_time_s", C.c_double), ("cost_per_iter", C.c_double),
        ("mask", C.c_uint32),
        ("pp", C.c_int32), ("tp", C.c_int32), ("dp", C.c_int32), ("mb", C.c_int32),
        ("pp_index", C.c_int32), ("tp_index", C.c_int32), ("dp_index", C.c_int32),
        ("mb_index", C.c_int32), ("partition", C.c_int32), ("n_segments", C.c_int32),
        ("cut", C.c_int32 * 2), ("pool", C.c_int32 * 3),
        ("seg_tp", C.c_int32 * 3), ("seg_tp_index", C.c_int32 * 3),
        ("zone", C.c_int32 * 3), ("type_a", C.c_int32 * 3), ("type_b", C.c_int32 * 3),
    ]


MAX_STAGES = 256


class sailor_search_options(C.Structure):
    _fields_ = [("beam_width", C.c_int32), ("max_runs", C.c_int32), ("use_incumbent", C.c_int32),
                ("incumbent", C.c_double), ("allow_split", C.c_int32), ("stage_tp", C.c_int32)]


class sailor_stage_plan(C.Structure):
    _fields_ = [("found", C.c_int32), ("exact", C.c_int32),
                ("pp", C.c_int32), ("tp", C.c_int32), ("dp", C.c_int32), ("mb", C.c_int32),
                ("pp_index", C.c_int32), ("tp_index", C.c_int32), ("dp_index", C.c_int32),
                ("mb_index", C.c_int32), ("partition", C.c_int32), ("mask", C.c_uint32),
                ("peak_mem_bytes", C.c_uint64),
                ("iter_time_s", C.c_double), ("cost_per_iter", C.c_double),
                ("eval_time_s", C.c_double), ("eval_cost", C.c_double),
                ("expanded", C.c_uint64), ("incumbent_used", C.c_int32), ("incumbent", C.c_double),
                ("pool", C.c_int32 * MAX_STAGES), ("pool_b", C.c_int32 * MAX_STAGES),
                ("stage_tp_index", C.c_int32 * MAX_STAGES)]


@dataclass
class StagePlan:
    """Result of sailor_search: one pool per stage."""
    found: bool
    exact: bool
    pp: int
    tp: int
    dp: int
    mb: int
    pp_index: int
    tp_index: int
    dp_index: int
    mb_index: int
    partition: int
    mask: int
    peak_mem_bytes: int
    iter_time_s: float
    cost_per_iter: float
    eval_time_s: float
    eval_cost: float
    expanded: int
    incumbent: Optional[float]
    pools: Tuple[int, ...]
    pools_b: Tuple[int, ...] = ()
    tps: Tuple[int, ...] = ()      # index of every stage's TP degree


@dataclass
class Result:
    index: int
    peak_mem_bytes: int
    iter_time_s: float
    cost_per_iter: float
    mask: int
    pp: int
    tp: int
    dp: int
    mb: int
    pp_index: int
    tp_index: int
    dp_index: int
    mb_index: int
    partition: int
    n_segments: int
    cut: Tuple[int, int]
    pool: Tuple[int, int, int]
    seg_tp: Tuple[int, int, int] = (0, 0, 0)
    seg_tp_index: Tuple[int, int, int] = (-1, -1, -1)
    zone: Tuple[int, int, int] = (-1, -1, -1)
    type_a: Tuple[int, int, int] = (-1, -1, -1)
    type_b: Tuple[int, int, int] = (-1, -1, -1)


def _result(r: sailor_result) -> Result:
    return Result(r.index, r.peak_mem_bytes, r.iter_time_s, r.cost_per_iter, r.mask, r.pp, r.tp,
                  r.dp, r.mb, r.pp_index, r.tp_index, r.dp_index, r.mb_index, r.partition,
                  r.n_segments, tuple(r.cut), tuple(r.pool), tuple(r.seg_tp), tuple(r.seg_tp_index), tuple(r.zone), tuple(r.type_a),
                  tuple(r.type_b))


_lib = None


def load_library() -> C.CDLL:
    """Loads libsailor.so; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with "
                          "`python -m paper_2504_17096_amd.build` (hipcc, gfx950)")
    lib = C.CDLL(LIB_PATH)
    P = C.c_void_p
    lib.sailor_plan_create.argtypes = [C.POINTER(sailor_problem), C.POINTER(P)]
    lib.sailor_plan_destroy.argtypes = [P]
    lib.sailor_plan_set_avail.argtypes = [P, P]
    lib.sailor_plan_num_candidates.argtypes = [P, C.POINTER(C.c_uint64)]
    lib.sailor_plan_decode.argtypes = [P, C.c_uint64, C.POINTER(sailor_result)]
    lib.sailor_eval_batch.argtypes = [P, C.c_uint64, C.c_uint64, P, C.c_int,
                                      C.POINTER(sailor_constraint), P, P, P, P, P]
    lib.sailor_best_plan.argtypes = [P, C.c_int, C.POINTER(sailor_constraint),
                                     C.POINTER(sailor_result), P]
    lib.sailor_topk.argtypes = [P, C.c_int, C.POINTER(sailor_constraint), C.c_int32,
                                C.POINTER(sailor_result), C.POINTER(C.c_int32), P]
    lib.sailor_plan_set_scratch.argtypes = [P, C.c_uint32, C.c_uint32]
    lib.sailor_plan_set_timing.argtypes = [P, C.c_int32]
    lib.sailor_plan_last_timing.argtypes = [P, C.POINTER(C.c_float), C.POINTER(C.c_float)]
    lib.sailor_simulate_1f1b.argtypes = [P, C.c_uint64, P, P, P, P]
    lib.sailor_simulate_1f1b_static.argtypes = [P, C.c_uint64, P, P, P, P]
    lib.sailor_plan_set_incremental.argtypes = [P, C.c_int32]
    lib.sailor_plan_last_scan.argtypes = [P, C.POINTER(C.c_uint32), C.POINTER(C.c_uint32)]
    lib.sailor_set_scan_unit_parts.argtypes = [C.c_int32]
    lib.sailor_search.argtypes = [P, C.c_int, C.POINTER(sailor_constraint),
                                  C.POINTER(sailor_search_options), C.POINTER(sailor_stage_plan), P]
    lib.sailor_eval_placements.argtypes = [P, C.c_uint64, P, P, P, P, C.c_uint32, C.c_int,
                                           C.POINTER(sailor_constraint), P, P, P, P, P]
    lib.sailor_eval_replica_placements.argtypes = [P, C.c_uint64, P, P, C.c_uint64, P, C.c_uint32, C.c_int,
                                                   C.POINTER(sailor_constraint), P, P, P, P, P]
    lib.sailor_plan_last_counts.argtypes = [P, C.POINTER(C.c_uint32), C.POINTER(C.c_uint32),
                                            C.POINTER(C.c_uint32)]
    for name in EXPORTS:
        getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def marshal_problem(prob):
    """Problem object -> (sailor_problem, list of arrays that must stay alive)."""
    keep = []

    def arr(a, dtype):
        a = np.ascontiguousarray(a, dtype=dtype)
        keep.append(a)
        return a.ctypes.data

    s = sailor_problem()
    s.n_layers, s.n_types, s.n_zones = prob.n_layers, prob.n_types, prob.n_zones
    s.n_mb, s.n_tp = len(prob.mb_values), len(prob.tp_values)
    s.n_dp, s.n_pp = len(prob.dp_values), len(prob.pp_values)
    s.max_segments, s.seg3_max_pp = prob.max_segments, prob.seg3_max_pp
    s.uniform_layers = 1 if prob.uniform_layers else 0
    s.per_segment_tp = 1 if getattr(prob, "per_segment_tp", False) else 0
    s.mixed_types = 1 if getattr(prob, "mixed_types", False) else 0
    s.global_batch = prob.global_batch
    s.mb_values = arr(prob.mb_values, np.int32)
    s.tp_values = arr(prob.tp_values, np.int32)
    s.dp_values = arr(prob.dp_values, np.int32)
    s.pp_values = arr(prob.pp_values, np.int32)
    s.n_partitions = arr(prob.n_partitions, np.int32)
    s.partition_layers = arr(prob.partition_layers, np.int32)
    s.layer_params = arr(prob.layer_params, np.uint64)
    s.embed_params, s.head_params = int(prob.embed_params), int(prob.head_params)
    s.bytes_per_param, s.grad_bytes_per_param = prob.bytes_per_param, prob.grad_bytes_per_param
    s.t_fwd = arr(prob.t_fwd, np.float64)
    s.t_bwd = arr(prob.t_bwd, np.float64)
    s.t_upd = arr(prob.t_upd, np.float64)
    s.act_store_bytes = arr(prob.act_store_bytes, np.uint64)
    s.p2p_bytes = arr(prob.p2p_bytes, np.uint64)
    s.mem_capacity = arr(prob.mem_capacity, np.uint64)
    s.mem_reserved = arr(prob.mem_reserved, np.uint64)
    s.gpus_per_node = arr(prob.gpus_per_node, np.int32)
    s.price_per_hour = arr(prob.price_per_hour, np.float64)
    s.avail = arr(prob.avail, np.int32)
    s.bandwidth = arr(prob.bandwidth, np.float64)
    s.egress_per_byte = (arr(prob.egress_per_byte, np.float64)
                         if prob.egress_per_byte is not None else None)
    poly = getattr(prob, "bw_poly", None)
    s.n_bw_coef = 0 if poly is None else int(np.asarray(poly).shape[-1])
    s.bw_poly = arr(poly, np.float64) if poly is not None else None
    return s, keep


def _ptr(x) -> Optional[int]:
    """Device pointer of a torch tensor, an int, or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _constraint(bound: Optional[float]):
    if bound is None:
        return None
    return C.byref(sailor_constraint(float(bound), 1))


def set_scan_unit_parts(n: int) -> None:
    """sailor_set_scan_unit_parts: 0 = cut scan pieces by measured time, n = into n parts each."""
    rc = load_library().sailor_set_scan_unit_parts(n)
    if rc != SAILOR_OK:
        raise SailorError(rc, "sailor_set_scan_unit_parts")


class Plan:
    """Owns one sailor_plan*.  Method names follow the C entry points."""

    def __init__(self, prob):
        self._lib = load_library()
        s, keep = marshal_problem(prob)
        h = C.c_void_p()
        rc = self._lib.sailor_plan_create(C.byref(s), C.byref(h))
        del keep
        if rc != SAILOR_OK:
            raise SailorError(rc, "sailor_plan_create")
        self._h = h

    def destroy(self):
        if getattr(self, "_h", None):
            self._lib.sailor_plan_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def set_avail(self, avail) -> None:
        a = np.ascontiguousarray(avail, dtype=np.int32)
        rc = self._lib.sailor_plan_set_avail(self._h, a.ctypes.data)
        if rc != SAILOR_OK:
            raise SailorError(rc, "sailor_plan_set_avail")

    def num_candidates(self) -> int:
        out = C.c_uint64()
        rc = self._lib.sailor_plan_num_candidates(self._h, C.byref(out))
        if rc != SAILOR_OK:
            raise SailorError(rc, "sailor_plan_num_candidates")
        return int(out.value)

    def decode(self, index: int) -> Result:
        r = sailor_result()
        rc = self._lib.sailor_plan_decode(self._h, index, C.byref(r))
        if rc != SAILOR_OK:
            raise SailorError(rc, "sailor_plan_decode")
        return _result(r)

    def eval_batch(self, first: int, count: int, d_indices=None, objective: int = MAX_THROUGHPUT,
                   bound: Optional[float] = None, d_time=None, d_cost=None, d_mem=None,
                   d_mask=None, stream: int = 0) -> None:
        rc = self._lib.sailor_eval_batch(self._h, first, count, _ptr(d_indices), objective,
                                         _constraint(bound), _ptr(d_time), _ptr(d_cost),
                                         _ptr(d_mem), _ptr(d_mask), stream or None)
        if rc != SAILOR_OK:
            raise SailorError(rc, "sailor_eval_batch")

    def best_plan(self, objective: int = MAX_THROUGHPUT, bound: Optional[float] = None,
                  stream: int = 0) -> Optional[Result]:
        """The best valid plan, or None when no candidate is valid."""
        r = sailor_result()
        rc = self._lib.sailor_best_plan(self._h, objective, _constraint(bound), C.byref(r),
                                        stream or None)
        if rc == SAILOR_ENOFEASIBLE:
            return None
        if rc != SAILOR_OK:
            raise SailorError(rc, "sailor_best_plan")
        return _result(r)

    def topk(self, k: int, objective: int = MAX_THROUGHPUT, bound: Optional[float] = None,
             stream: int = 0) -> List[Result]:
        buf = (sailor_result * k)()
        n = C.c_int32(0)
        rc = self._lib.sailor_topk(self._h, objective, _constraint(bound), k, buf, C.byref(n),
                                   stream or None)
        if rc == SAILOR_ENOFEASIBLE:
            return []
        if rc != SAILOR_OK:
            raise SailorError(rc, "sailor_topk")
        return [_result(buf[i]) for i in range(n.value)]

    def set_scratch(self, max_survivors: int, max_refined: int) -> None:
        rc = self._lib.sailor_plan_set_scratch(self._h, max_survivors, max_refined)
        if rc != SAILOR_OK:
            raise SailorError(rc, "sailor_plan_set_scratch")

    def set_timing(self, mode: int) -> None:
        rc = self._lib.sailor_plan_set_timing(self._h, mode)
        if rc != SAILOR_OK:
            raise SailorError(rc, "sailor_plan_set_timing")

    def topk_raw(self, k: int, objective: int, bound: Optional[float], buf, stream: int = 0) -> int:
        """sailor_topk into a caller-kept (sailor_result * k) array; returns n_found."""
        n = C.c_int32(0)
        rc = self._lib.sailor_topk(self._h, objective, _constraint(bound), k, buf, C.byref(n),
                                   stream or None)
        if rc not in (SAILOR_OK, SAILOR_ENOFEASIBLE):
            raise SailorError(rc, "sailor_topk")
        return n.value

    def last_timing(self) -> Tuple[float, float]:
        """(total ms, dominant-kernel ms) of the last call, from HIP events (see set_timing)."""
        t, s = C.c_float(), C.c_float()
        rc = self._lib.sailor_plan_last_timing(self._h, C.byref(t), C.byref(s))
        if rc != SAILOR_OK:
            raise SailorError(rc, "sailor_plan_last_timing")
        return t.value, s.value

    def last_counts(self) -> Tuple[int, int, int]:
        """(survivors of the fp32 threshold, candidates re-evaluated in fp64, valid ones
        among them) of the last successful best_plan / topk."""
        a, b, c = C.c_uint32(), C.c_uint32(), C.c_uint32()
        rc = self._lib.sailor_plan_last_counts(self._h, C.byref(a), C.byref(b), C.byref(c))
        if rc != SAILOR_OK:
            raise SailorError(rc, "sailor_plan_last_counts")
        return a.value, b.value, c.value

    def search(self, beam_width: int, objective: int = MAX_THROUGHPUT, bound: Optional[float] = None,
               max_runs: int = 0, incumbent=None, stream: int = 0, allow_split: bool = False,
               stage_tp: bool = False) -> StagePlan:
        """sailor_search.  incumbent: None, a float, or "flat" (the library takes the best plan
        of the flat space).  The returned plan has found = False when nothing valid exists."""
        o = sailor_search_options(beam_width, max_runs, 0, 0.0, 1 if allow_split else 0,
                                  1 if stage_tp else 0)
        if incumbent == "flat":
            o.use_incumbent = 2
        elif incumbent is not None:
            o.use_incumbent, o.incumbent = 1, float(incumbent)
        r = sailor_stage_plan()
        rc = self._lib.sailor_search(self._h, objective, _constraint(bound), C.byref(o), C.byref(r),
                                     stream or None)
        if rc not in (SAILOR_OK, SAILOR_ENOFEASIBLE):
            raise SailorError(rc, "sailor_search")
        return StagePlan(bool(r.found), bool(r.exact), r.pp, r.tp, r.dp, r.mb, r.pp_index, r.tp_index,
                         r.dp_index, r.mb_index, r.partition, r.mask, r.peak_mem_bytes, r.iter_time_s,
                         r.cost_per_iter, r.eval_time_s, r.eval_cost, r.expanded,
                         r.incumbent if r.incumbent_used else None, tuple(r.pool[:r.pp]),
                         tuple(r.pool_b[:r.pp]), tuple(r.stage_tp_index[:r.pp]))

    def eval_placements(self, count: int, d_desc, d_pools, pool_stride: int,
                        objective: int = MAX_THROUGHPUT, bound: Optional[float] = None, d_time=None,
                        d_cost=None, d_mem=None, d_mask=None, stream: int = 0, d_pools_b=None,
                        d_tps=None) -> None:
        """sailor_eval_placements; device tensors: int32 [count][5], int32 [count][pool_stride]
        (and optionally the pools of the other half of every stage's replicas, the TP index
        of every stage, or both), float64 / float64 / int64 / int32 outputs."""
        rc = self._lib.sailor_eval_placements(self._h, count, _ptr(d_desc), _ptr(d_pools),
                                              _ptr(d_pools_b), _ptr(d_tps), pool_stride,
                                              objective, _constraint(bound), _ptr(d_time), _ptr(d_cost),
                                              _ptr(d_mem), _ptr(d_mask), stream or None)
        if rc != SAILOR_OK:
            raise SailorError(rc, "sailor_eval_placements")

    def eval_replica_placements(self, count: int, d_desc, d_pools, stride: int,
                                objective: int = MAX_THROUGHPUT, bound: Optional[float] = None, d_time=None,
                                d_cost=None, d_mem=None, d_mask=None, stream: int = 0, d_tps=None,
                                tps_stride: int = 0) -> None:
        """sailor_eval_replica_placements; device tensors: int32 [count][5], int32 [count][stride] with
        the pool of replica r of stage i at i * D + r (optionally int32 [count][tps_stride], the TP
        index of every stage), float64 / float64 / int64 / int32 outputs."""
        rc = self._lib.sailor_eval_replica_placements(self._h, count, _ptr(d_desc), _ptr(d_pools), stride,
                                                      _ptr(d_tps), tps_stride,
                                                      objective, _constraint(bound), _ptr(d_time),
                                                      _ptr(d_cost), _ptr(d_mem), _ptr(d_mask), stream or None)
        if rc != SAILOR_OK:
            raise SailorError(rc, "sailor_eval_replica_placements")

    def set_incremental(self, on: bool) -> None:
        rc = self._lib.sailor_plan_set_incremental(self._h, 1 if on else 0)
        if rc != SAILOR_OK:
            raise SailorError(rc, "sailor_plan_set_incremental")

    def last_scan(self) -> Tuple[int, int]:
        """(pieces of the space the last selection evaluated, pieces in total)."""
        a, b = C.c_uint32(), C.c_uint32()
        rc = self._lib.sailor_plan_last_scan(self._h, C.byref(a), C.byref(b))
        if rc != SAILOR_OK:
            raise SailorError(rc, "sailor_plan_last_scan")
        return a.value, b.value

    def simulate_1f1b(self, count: int, d_indices, d_event=None, d_closed=None, stream: int = 0) -> None:
        """sailor_simulate_1f1b; the arrays are device tensors (uint64 / int64 indices, float64)."""
        rc = self._lib.sailor_simulate_1f1b(self._h, count, _ptr(d_indices), _ptr(d_event),
                                            _ptr(d_closed), stream or None)
        if rc != SAILOR_OK:
            raise SailorError(rc, "sailor_simulate_1f1b")

    def simulate_1f1b_static(self, count: int, d_indices, d_event=None, d_closed=None,
                             stream: int = 0) -> None:
        """sailor_simulate_1f1b_static: the same schedule with its working set in the library's
        static device array (no allocation inside the call)."""
        rc = self._lib.sailor_simulate_1f1b_static(self._h, count, _ptr(d_indices), _ptr(d_event),
                                                   _ptr(d_closed), stream or None)
        if rc != SAILOR_OK:
            raise SailorError(rc, "sailor_simulate_1f1b_static")
