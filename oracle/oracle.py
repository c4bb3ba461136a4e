"""ctypes front end of the CPU oracle -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg import this.  It
marshals a problem object (any object with the attribute names of the C struct in
sailor_oracle.h) and calls the plain C implementation; it contains no arithmetic of
the method itself.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import List, Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# the mutation tests point this at a copy of the sources with a planted mistake
_DIR = os.environ.get("SAILOR_ORACLE_DIR", _HERE)
_SRC = os.path.join(_DIR, "sailor_oracle.c")
_SRC_SEARCH = os.path.join(_DIR, "sailor_search_oracle.c")
_LIB = os.path.join(_DIR, "libsailor_oracle.so")

MAX_THROUGHPUT, MIN_COST = 0, 1
BIT_OOM, BIT_QUOTA, BIT_BATCH, BIT_TP_NODE, BIT_CONSTRAINT = 1, 2, 4, 8, 32


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no intrinsics)."""
    deps = [_SRC, _SRC_SEARCH, os.path.join(_DIR, "sailor_oracle.h")]
    stale = not os.path.exists(_LIB) or any(os.path.getmtime(_LIB) < os.path.getmtime(d) for d in deps)
    if force or stale:
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-Wall", "-shared", "-fPIC", "-o", _LIB,
                               _SRC, _SRC_SEARCH, "-lpthread", "-lm"])
    return _LIB


class _Problem(C.Structure):
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


class _Config(C.Structure):
    _fields_ = [("pp", C.c_int32), ("pp_idx", C.c_int32), ("n_segments", C.c_int32),
                ("partition", C.c_int32), ("cut", C.c_int32 * 2), ("pool", C.c_int32 * 3),
                ("dp", C.c_int32), ("tp", C.c_int32), ("mb", C.c_int32),
                ("dp_idx", C.c_int32), ("tp_idx", C.c_int32), ("mb_idx", C.c_int32),
                ("seg_tp", C.c_int32 * 3), ("seg_tp_idx", C.c_int32 * 3)]


class _Eval(C.Structure):
    _fields_ = [("index", C.c_uint64), ("mask", C.c_uint32), ("peak_mem", C.c_uint64),
                ("iter_time", C.c_double), ("cost", C.c_double)]


@dataclass
class Config:
    pp: int
    pp_idx: int
    n_segments: int
    partition: int
    cut: tuple
    pool: tuple
    dp: int
    tp: int
    mb: int
    dp_idx: int
    tp_idx: int
    mb_idx: int
    seg_tp: tuple = (0, 0, 0)
    seg_tp_idx: tuple = (-1, -1, -1)


class _SearchResult(C.Structure):
    _fields_ = [("found", C.c_int32), ("truncated", C.c_int32), ("pp_idx", C.c_int32),
                ("partition", C.c_int32), ("tp_idx", C.c_int32), ("dp_idx", C.c_int32),
                ("mb_idx", C.c_int32), ("pp", C.c_int32), ("expanded", C.c_uint64),
                ("key", C.c_double), ("iter_time", C.c_double), ("cost", C.c_double),
                ("pools", C.c_int32 * 256), ("pools_b", C.c_int32 * 256), ("tps", C.c_int32 * 256)]


class _SearchOpts(C.Structure):
    _fields_ = [("beam_width", C.c_int32), ("max_runs", C.c_int32), ("has_incumbent", C.c_int32),
                ("incumbent", C.c_double), ("allow_split", C.c_int32), ("stage_tp", C.c_int32)]


@dataclass
class StagePlan:
    """A plan whose stages choose their pools freely."""
    pp_idx: int
    partition: int
    tp_idx: int
    dp_idx: int
    mb_idx: int
    pools: tuple
    key: float
    iter_time: float
    cost: float
    truncated: bool = False
    expanded: int = 0
    pools_b: tuple = ()
    tps: tuple = ()      # index of every stage's TP degree


@dataclass
class Eval:
    index: int
    mask: int
    peak_mem: int
    iter_time: float
    cost: float


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = C.CDLL(build())
        lib.so_create.restype = C.c_void_p
        lib.so_create.argtypes = [C.POINTER(_Problem)]
        lib.so_destroy.argtypes = [C.c_void_p]
        lib.so_num_candidates.restype = C.c_uint64
        lib.so_num_candidates.argtypes = [C.c_void_p]
        lib.so_decode.argtypes = [C.c_void_p, C.c_uint64, C.POINTER(_Config)]
        lib.so_encode.argtypes = [C.c_void_p, C.POINTER(_Config), C.POINTER(C.c_uint64)]
        lib.so_enumerate.restype = C.c_uint64
        lib.so_enumerate.argtypes = [C.c_void_p, C.POINTER(_Config), C.c_uint64]
        lib.so_simulate_1f1b.argtypes = [C.c_void_p, C.c_uint64, C.POINTER(C.c_double),
                                         C.POINTER(C.c_double)]
        lib.so_eval_one.argtypes = [C.c_void_p, C.c_uint64, C.c_int, C.c_int, C.c_double,
                                    C.POINTER(_Eval)]
        lib.so_eval_batch.argtypes = [C.c_void_p, C.c_uint64, C.c_uint64, C.c_void_p, C.c_int,
                                      C.c_int, C.c_double, C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_int]
        lib.so_best.argtypes = [C.c_void_p, C.c_uint64, C.c_uint64, C.c_int, C.c_int, C.c_double,
                                C.c_int, C.POINTER(_Eval)]
        lib.so_topk.argtypes = [C.c_void_p, C.c_uint64, C.c_uint64, C.c_int, C.c_int, C.c_double,
                                C.c_int, C.c_int, C.POINTER(_Eval)]
        lib.so_eval_assignment.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                           C.c_void_p, C.c_int, C.c_int, C.c_double, C.POINTER(_Eval)]
        lib.so_eval_split_assignment.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                                 C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_double,
                                                 C.POINTER(_Eval)]
        lib.so_eval_split_assignment_tp.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p,
                                                    C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_double,
                                                    C.POINTER(_Eval)]
        lib.so_eval_assignment_tp.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p,
                                              C.c_void_p, C.c_int, C.c_int, C.c_double, C.POINTER(_Eval)]
        lib.so_eval_replica_assignment.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                                   C.c_void_p, C.c_int, C.c_int, C.c_double, C.POINTER(_Eval)]
        lib.so_eval_replica_assignment_tp.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p,
                                                      C.c_void_p, C.c_int, C.c_int, C.c_double, C.POINTER(_Eval)]
        lib.so_search_exhaustive.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_double, C.c_int, C.c_int,
                                             C.c_int, C.POINTER(_SearchResult)]
        lib.so_search_prefix_bound_tp.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p,
                                                  C.c_void_p, C.c_int, C.c_int, C.POINTER(C.c_double),
                                                  C.POINTER(C.c_double)]
        lib.so_search_prefix_bound_split_tp.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int,
                                                        C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int,
                                                        C.POINTER(C.c_double), C.POINTER(C.c_double)]
        lib.so_search_beam.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_double, C.POINTER(_SearchOpts),
                                       C.POINTER(_SearchResult)]
        lib.so_search_prefix_bound.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                               C.c_void_p, C.c_int, C.c_int, C.POINTER(C.c_double),
                                               C.POINTER(C.c_double)]
        _lib = lib
    return _lib


def _stage_plan(r: _SearchResult) -> Optional[StagePlan]:
    if not r.found:
        return None
    return StagePlan(r.pp_idx, r.partition, r.tp_idx, r.dp_idx, r.mb_idx, tuple(r.pools[:r.pp]),
                     r.key, r.iter_time, r.cost, bool(r.truncated), int(r.expanded),
                     tuple(r.pools_b[:r.pp]), tuple(r.tps[:r.pp]))


def _cfg(c: _Config) -> Config:
    return Config(c.pp, c.pp_idx, c.n_segments, c.partition, tuple(c.cut), tuple(c.pool),
                  c.dp, c.tp, c.mb, c.dp_idx, c.tp_idx, c.mb_idx, tuple(c.seg_tp), tuple(c.seg_tp_idx))


def _ev(e: _Eval) -> Eval:
    return Eval(e.index, e.mask, e.peak_mem, e.iter_time, e.cost)


class Oracle:
    """One problem bound to the C oracle.  Keeps the numpy arrays alive."""

    def __init__(self, prob):
        lib = _load()
        self._keep = []

        def arr(a, dtype):
            a = np.ascontiguousarray(a, dtype=dtype)
            self._keep.append(a)
            return a.ctypes.data

        s = _Problem()
        s.n_layers, s.n_types, s.n_zones = prob.n_layers, prob.n_types, prob.n_zones
        s.n_mb, s.n_tp, s.n_dp, s.n_pp = (len(prob.mb_values), len(prob.tp_values),
                                          len(prob.dp_values), len(prob.pp_values))
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
        s.bytes_per_param = prob.bytes_per_param
        s.grad_bytes_per_param = prob.grad_bytes_per_param
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
        self._struct = s
        self._prob = prob
        self._lib = lib
        self._ctx = lib.so_create(C.byref(s))
        if not self._ctx:
            raise ValueError("oracle rejected the problem")

    def close(self):
        if self._ctx:
            self._lib.so_destroy(self._ctx)
            self._ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def num_candidates(self) -> int:
        return int(self._lib.so_num_candidates(self._ctx))

    def decode(self, index: int) -> Config:
        c = _Config()
        if self._lib.so_decode(self._ctx, index, C.byref(c)) != 0:
            raise IndexError(index)
        return _cfg(c)

    def encode(self, cfg: Config) -> int:
        c = _Config()
        c.pp, c.pp_idx, c.n_segments, c.partition = cfg.pp, cfg.pp_idx, cfg.n_segments, cfg.partition
        c.cut[0], c.cut[1] = cfg.cut
        c.pool[0], c.pool[1], c.pool[2] = cfg.pool
        c.dp, c.tp, c.mb = cfg.dp, cfg.tp, cfg.mb
        c.dp_idx, c.tp_idx, c.mb_idx = cfg.dp_idx, cfg.tp_idx, cfg.mb_idx
        for j in range(3):
            c.seg_tp[j], c.seg_tp_idx[j] = cfg.seg_tp[j], cfg.seg_tp_idx[j]
        out = C.c_uint64()
        if self._lib.so_encode(self._ctx, C.byref(c), C.byref(out)) != 0:
            raise ValueError("invalid config")
        return int(out.value)

    def enumerate(self, max_out: Optional[int] = None) -> List[Config]:
        n = self.num_candidates if max_out is None else max_out
        buf = (_Config * n)()
        total = self._lib.so_enumerate(self._ctx, buf, n)
        return [_cfg(buf[i]) for i in range(min(n, total))]

    def enumerate_count(self) -> int:
        return int(self._lib.so_enumerate(self._ctx, None, 0))

    def eval_one(self, index: int, objective: int = MAX_THROUGHPUT,
                 bound: Optional[float] = None) -> Eval:
        e = _Eval()
        rc = self._lib.so_eval_one(self._ctx, index, objective, bound is not None,
                                   0.0 if bound is None else bound, C.byref(e))
        if rc != 0:
            raise IndexError(index)
        return _ev(e)

    def simulate_1f1b(self, index: int) -> Tuple[float, float]:
        """(event-by-event makespan, closed-form T_pp) of one pipeline of the plan."""
        a, b = C.c_double(), C.c_double()
        if self._lib.so_simulate_1f1b(self._ctx, index, C.byref(a), C.byref(b)) < 0:
            raise IndexError(index)
        return a.value, b.value

    def eval_batch(self, first: int = 0, count: Optional[int] = None, indices=None,
                   objective: int = MAX_THROUGHPUT, bound: Optional[float] = None,
                   n_threads: int = 1):
        """Returns (time f64, cost f64, mem u64, mask u32) arrays."""
        if indices is not None:
            indices = np.ascontiguousarray(indices, dtype=np.uint64)
            count = len(indices)
        elif count is None:
            count = self.num_candidates - first
        t = np.empty(count, np.float64)
        c = np.empty(count, np.float64)
        m = np.empty(count, np.uint64)
        k = np.empty(count, np.uint32)
        rc = self._lib.so_eval_batch(self._ctx, first, count,
                                     None if indices is None else indices.ctypes.data,
                                     objective, bound is not None, 0.0 if bound is None else bound,
                                     t.ctypes.data, c.ctypes.data, m.ctypes.data, k.ctypes.data,
                                     n_threads)
        if rc != 0:
            raise IndexError((first, count))
        return t, c, m, k

    def eval_assignment(self, pp_idx: int, partition: int, dp_idx: int, mb_idx: int, tp_idx: int,
                        pools, objective: int = MAX_THROUGHPUT, bound: Optional[float] = None) -> Eval:
        a = np.ascontiguousarray(pools, dtype=np.int32)
        e = _Eval()
        rc = self._lib.so_eval_assignment(self._ctx, pp_idx, partition, dp_idx, mb_idx, tp_idx,
                                          a.ctypes.data, objective, bound is not None,
                                          0.0 if bound is None else bound, C.byref(e))
        if rc != 0:
            raise ValueError("assignment out of range")
        return _ev(e)

    def eval_assignment_tp(self, pp_idx: int, partition: int, dp_idx: int, mb_idx: int, tps, pools,
                           objective: int = MAX_THROUGHPUT, bound: Optional[float] = None) -> Eval:
        """A plan with a pool and a TP index per stage."""
        a = np.ascontiguousarray(pools, dtype=np.int32)
        t = np.ascontiguousarray(tps, dtype=np.int32)
        assert len(a) == len(t)
        e = _Eval()
        rc = self._lib.so_eval_assignment_tp(self._ctx, pp_idx, partition, dp_idx, mb_idx, t.ctypes.data,
                                             a.ctypes.data, objective, bound is not None,
                                             0.0 if bound is None else bound, C.byref(e))
        if rc != 0:
            raise ValueError("assignment out of range")
        return _ev(e)

    def eval_split_assignment(self, pp_idx: int, partition: int, dp_idx: int, mb_idx: int, tp_idx: int,
                              pools_a, pools_b, objective: int = MAX_THROUGHPUT,
                              bound: Optional[float] = None) -> Eval:
        a = np.ascontiguousarray(pools_a, dtype=np.int32)
        b = np.ascontiguousarray(pools_b, dtype=np.int32)
        e = _Eval()
        rc = self._lib.so_eval_split_assignment(self._ctx, pp_idx, partition, dp_idx, mb_idx, tp_idx,
                                                a.ctypes.data, b.ctypes.data, objective,
                                                bound is not None, 0.0 if bound is None else bound,
                                                C.byref(e))
        if rc != 0:
            raise ValueError("assignment out of range")
        return _ev(e)

    def eval_split_assignment_tp(self, pp_idx: int, partition: int, dp_idx: int, mb_idx: int, tp_idx,
                                 pools_a, pools_b, objective: int = MAX_THROUGHPUT,
                                 bound: Optional[float] = None) -> Eval:
        """Two pools and a TP index per stage (tp_idx: one index per stage)."""
        t = np.ascontiguousarray(tp_idx, dtype=np.int32)
        a = np.ascontiguousarray(pools_a, dtype=np.int32)
        b = np.ascontiguousarray(pools_b, dtype=np.int32)
        e = _Eval()
        rc = self._lib.so_eval_split_assignment_tp(self._ctx, pp_idx, partition, dp_idx, mb_idx,
                                                   t.ctypes.data, a.ctypes.data, b.ctypes.data, objective,
                                                   bound is not None, 0.0 if bound is None else bound,
                                                   C.byref(e))
        if rc != 0:
            raise ValueError("assignment out of range")
        return _ev(e)

    def eval_replica_assignment(self, pp_idx: int, partition: int, dp_idx: int, mb_idx: int, tp_idx: int,
                                pools, objective: int = MAX_THROUGHPUT, bound: Optional[float] = None) -> Eval:
        """pools: [P][D], the pool of every replica of every stage."""
        a = np.ascontiguousarray(pools, dtype=np.int32)
        assert a.shape == (int(self._prob.pp_values[pp_idx]), int(self._prob.dp_values[dp_idx]))
        e = _Eval()
        rc = self._lib.so_eval_replica_assignment(self._ctx, pp_idx, partition, dp_idx, mb_idx, tp_idx,
                                                  a.ctypes.data, objective, bound is not None,
                                                  0.0 if bound is None else bound, C.byref(e))
        if rc != 0:
            raise ValueError("assignment out of range")
        return _ev(e)


    def eval_replica_assignment_tp(self, pp_idx: int, partition: int, dp_idx: int, mb_idx: int, tp_idx,
                                   pools, objective: int = MAX_THROUGHPUT,
                                   bound: Optional[float] = None) -> Eval:
        """pools: [P][D], the pool of every replica of every stage; tp_idx: [P], a TP index per stage."""
        a = np.ascontiguousarray(pools, dtype=np.int32)
        t = np.ascontiguousarray(tp_idx, dtype=np.int32)
        assert a.shape == (int(self._prob.pp_values[pp_idx]), int(self._prob.dp_values[dp_idx]))
        assert t.shape == (a.shape[0],)
        e = _Eval()
        rc = self._lib.so_eval_replica_assignment_tp(self._ctx, pp_idx, partition, dp_idx, mb_idx,
                                                     t.ctypes.data, a.ctypes.data, objective,
                                                     bound is not None, 0.0 if bound is None else bound,
                                                     C.byref(e))
        if rc != 0:
            raise ValueError("assignment out of range")
        return _ev(e)
    def search_exhaustive(self, objective: int = MAX_THROUGHPUT, bound: Optional[float] = None,
                          max_runs: int = 0, allow_split: bool = False,
                          stage_tp: bool = False) -> Optional[StagePlan]:
        r = _SearchResult()
        rc = self._lib.so_search_exhaustive(self._ctx, objective, bound is not None,
                                            0.0 if bound is None else bound, max_runs,
                                            1 if allow_split else 0, 1 if stage_tp else 0, C.byref(r))
        if rc != 0:
            raise ValueError("the search does not cover this problem")
        return _stage_plan(r)

    def search_beam(self, beam_width: int, objective: int = MAX_THROUGHPUT,
                    bound: Optional[float] = None, max_runs: int = 0,
                    incumbent: Optional[float] = None, allow_split: bool = False,
                    stage_tp: bool = False) -> Optional[StagePlan]:
        r = _SearchResult()
        o = _SearchOpts(beam_width, max_runs, incumbent is not None,
                        0.0 if incumbent is None else incumbent, 1 if allow_split else 0,
                        1 if stage_tp else 0)
        rc = self._lib.so_search_beam(self._ctx, objective, bound is not None,
                                      0.0 if bound is None else bound, C.byref(o), C.byref(r))
        if rc != 0:
            raise ValueError("the search does not cover this problem")
        self.last_search = (bool(r.truncated), int(r.expanded))
        return _stage_plan(r)

    def prefix_bound(self, pp_idx: int, partition: int, dp_idx: int, mb_idx: int, tp_idx: int,
                     pools, n_placed: int, objective: int = MAX_THROUGHPUT):
        """(lower bound on T_iter, on C_iter) of the completions of the first n_placed stages'
        placement, or None when the prefix itself is not admissible."""
        a = np.ascontiguousarray(pools, dtype=np.int32)
        t, c = C.c_double(), C.c_double()
        rc = self._lib.so_search_prefix_bound(self._ctx, pp_idx, partition, dp_idx, mb_idx, tp_idx,
                                              a.ctypes.data, n_placed, objective, C.byref(t), C.byref(c))
        return None if rc != 0 else (t.value, c.value)

    def prefix_bound_tp(self, pp_idx: int, partition: int, dp_idx: int, mb_idx: int, tps, pools,
                        n_placed: int, objective: int = MAX_THROUGHPUT):
        """prefix_bound for a placement with a TP index per stage."""
        a = np.ascontiguousarray(pools, dtype=np.int32)
        tt = np.ascontiguousarray(tps, dtype=np.int32)
        t, c = C.c_double(), C.c_double()
        rc = self._lib.so_search_prefix_bound_tp(self._ctx, pp_idx, partition, dp_idx, mb_idx, tt.ctypes.data,
                                                 a.ctypes.data, n_placed, objective, C.byref(t), C.byref(c))
        return None if rc != 0 else (t.value, c.value)

    def prefix_bound_split_tp(self, pp_idx: int, partition: int, dp_idx: int, mb_idx: int, tps, pools_a,
                              pools_b, n_placed: int, objective: int = MAX_THROUGHPUT):
        """prefix_bound for a placement with two pools and a TP index per stage."""
        a = np.ascontiguousarray(pools_a, dtype=np.int32)
        b = np.ascontiguousarray(pools_b, dtype=np.int32)
        tt = np.ascontiguousarray(tps, dtype=np.int32)
        t, c = C.c_double(), C.c_double()
        rc = self._lib.so_search_prefix_bound_split_tp(self._ctx, pp_idx, partition, dp_idx, mb_idx,
                                                       tt.ctypes.data, a.ctypes.data, b.ctypes.data, n_placed,
                                                       objective, C.byref(t), C.byref(c))
        return None if rc != 0 else (t.value, c.value)

    def best(self, objective: int = MAX_THROUGHPUT, bound: Optional[float] = None,
             first: int = 0, count: Optional[int] = None, n_threads: int = 1) -> Optional[Eval]:
        if count is None:
            count = self.num_candidates - first
        e = _Eval()
        ok = self._lib.so_best(self._ctx, first, count, objective, bound is not None,
                               0.0 if bound is None else bound, n_threads, C.byref(e))
        return _ev(e) if ok else None

    def topk(self, k: int, objective: int = MAX_THROUGHPUT, bound: Optional[float] = None,
             first: int = 0, count: Optional[int] = None, n_threads: int = 1) -> List[Eval]:
        if count is None:
            count = self.num_candidates - first
        buf = (_Eval * k)()
        n = self._lib.so_topk(self._ctx, first, count, objective, bound is not None,
                              0.0 if bound is None else bound, k, n_threads, buf)
        return [_ev(buf[i]) for i in range(n)]
