"""Seeded synthetic planning problems (inputs only).

This module draws the *inputs* of the planner: profiled per-layer times, memory
tables, GPU availability per (zone, type), the zone-to-zone bandwidth matrix,
prices and the lists of parallelism degrees.  It holds none of the planner's or
simulator's arithmetic, so both the HIP path and the CPU oracle may be fed from it.

The shapes follow the workloads of the paper's evaluation (Sec. 5: OPT-350M and
GPT-Neo-2.7B-like transformer stacks on A100/V100-like mixes over several zones);
the numbers are synthetic stand-ins for the paper's real profiles (Sec. 4.1), which
are not public.

Random numbers come from one counter-based generator, SplitMix64 (Steele, Lea,
Flood, "Fast splittable pseudorandom number generators", OOPSLA 2014): state
advances by the 64-bit golden-ratio increment and is finalised by two xor-shift
multiplies.  Normal deviates use the Box-Muller transform on two uniforms.
All draws happen in a fixed, documented order, so a seed fixes the problem.

Units everywhere: seconds, bytes, bytes/second, $/hour, $/byte.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import List, Optional

import numpy as np

_MASK64 = (1 << 64) - 1


class SplitMix64:
    """SplitMix64 stream; `seed` is the initial state."""

    def __init__(self, seed: int):
        self.state = seed & _MASK64

    def next_u64(self) -> int:
        self.state = (self.state + 0x9E3779B97F4A7C15) & _MASK64
        z = self.state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
        return z ^ (z >> 31)

    def uniform(self) -> float:
        """Uniform in [0, 1) with 53 random bits."""
        return (self.next_u64() >> 11) * (1.0 / (1 << 53))

    def uniform_range(self, lo: float, hi: float) -> float:
        return lo + (hi - lo) * self.uniform()

    def randint(self, lo: int, hi: int) -> int:
        """Uniform integer in [lo, hi] (inclusive)."""
        return lo + int(self.uniform() * (hi - lo + 1))

    def normal(self) -> float:
        """Standard normal by Box-Muller (uses two uniforms, returns one deviate)."""
        u1 = 1.0 - self.uniform()  # (0, 1]
        u2 = self.uniform()
        return math.sqrt(-2.0 * math.log(u1)) * math.cos(2.0 * math.pi * u2)

    def lognormal(self, median: float, sigma: float) -> float:
        return median * math.exp(sigma * self.normal())


@dataclass
class Problem:
    """One planning problem; field names follow the C-ABI problem struct.

    Arrays are C-contiguous numpy arrays of the stated dtype and shape
    (G = n_types, Z = n_zones, Lc = n_layers if not uniform_layers else 1).
    """
    n_layers: int
    n_types: int
    n_zones: int
    mb_values: np.ndarray          # int32 [n_mb], ascending
    tp_values: np.ndarray          # int32 [n_tp], ascending
    dp_values: np.ndarray          # int32 [n_dp], ascending
    pp_values: np.ndarray          # int32 [n_pp], ascending
    max_segments: int              # 1, 2 or 3
    seg3_max_pp: int               # a third segment only for pp <= this
    global_batch: int
    n_partitions: np.ndarray       # int32 [n_pp]
    partition_layers: np.ndarray   # int32, concatenated rows of pp_values[i] layer counts
    layer_params: np.ndarray       # uint64 [n_layers]
    embed_params: int
    head_params: int
    bytes_per_param: int
    grad_bytes_per_param: int
    uniform_layers: bool
    t_fwd: np.ndarray              # float64 [G][n_mb][n_tp][Lc]
    t_bwd: np.ndarray              # float64 [G][n_mb][n_tp][Lc]
    t_upd: np.ndarray              # float64 [G][n_tp][Lc]
    act_store_bytes: np.ndarray    # uint64 [n_mb][n_tp]
    p2p_bytes: np.ndarray          # uint64 [n_mb]
    mem_capacity: np.ndarray       # uint64 [G]
    mem_reserved: np.ndarray       # uint64 [G]
    gpus_per_node: np.ndarray      # int32 [G]
    price_per_hour: np.ndarray     # float64 [G]
    avail: np.ndarray              # int32 [Z][G]
    bandwidth: np.ndarray          # float64 [Z][Z], bytes/s
    egress_per_byte: Optional[np.ndarray] = None  # float64 [Z][Z] or None (= zeros)
    per_segment_tp: bool = False   # every segment carries its own TP digit
    mixed_types: bool = False      # a segment's replicas may be split over two GPU types
    bw_poly: Optional[np.ndarray] = None  # float64 [Z][Z][n_coef]: bandwidth over log2(message
                                          # bytes), lowest power first; None = constant
    name: str = ""
    notes: dict = field(default_factory=dict)

    @property
    def n_mb(self) -> int:
        return len(self.mb_values)

    @property
    def n_tp(self) -> int:
        return len(self.tp_values)

    @property
    def n_dp(self) -> int:
        return len(self.dp_values)

    @property
    def n_pp(self) -> int:
        return len(self.pp_values)

    def with_per_segment_tp(self, on: bool = True) -> "Problem":
        return replace(self, per_segment_tp=bool(on))

    def with_mixed_types(self, on: bool = True) -> "Problem":
        return replace(self, mixed_types=bool(on))

    def with_bw_poly(self, poly: Optional[np.ndarray]) -> "Problem":
        return replace(self, bw_poly=None if poly is None
                       else np.ascontiguousarray(poly, dtype=np.float64))

    def with_avail(self, avail: np.ndarray) -> "Problem":
        return replace(self, avail=np.ascontiguousarray(avail, dtype=np.int32))


GIB = 1 << 30


def _divisors(n: int) -> List[int]:
    return [d for d in range(1, n + 1) if n % d == 0]


def _pow2_upto(n: int) -> List[int]:
    out, v = [], 1
    while v <= n:
        out.append(v)
        v *= 2
    return out


def _uniform_split(n_layers: int, pp: int) -> List[int]:
    base, rem = divmod(n_layers, pp)
    return [base + (1 if i < rem else 0) for i in range(pp)]


def _random_composition(rng: SplitMix64, n_layers: int, pp: int) -> List[int]:
    """pp positive layer counts summing to n_layers: pp-1 distinct cut points by a
    partial Fisher-Yates shuffle of 1..n_layers-1."""
    cuts = list(range(1, n_layers))
    for i in range(pp - 1):
        j = rng.randint(i, len(cuts) - 1)
        cuts[i], cuts[j] = cuts[j], cuts[i]
    chosen = sorted(cuts[:pp - 1])
    edges = [0] + chosen + [n_layers]
    return [edges[i + 1] - edges[i] for i in range(pp)]


def _partitions(rng: Optional[SplitMix64], n_layers: int, pp_values, per_pp: int):
    """Exactly per_pp rows for every pp.  Row 0 is the uniform split; the others are
    distinct random compositions while distinct ones exist (pp = 1 and pp = n_layers
    have a single composition: their rows repeat, which yields exact duplicate plans
    that the lowest-index tie rule resolves)."""
    n_part, rows = [], []
    for pp in pp_values:
        seen = [tuple(_uniform_split(n_layers, pp))]
        limit = min(per_pp, math.comb(n_layers - 1, pp - 1))
        while len(seen) < limit:
            c = tuple(_random_composition(rng, n_layers, pp))
            if c not in seen:
                seen.append(c)
        while len(seen) < per_pp:
            seen.append(seen[len(seen) % limit])
        n_part.append(len(seen))
        for c in seen:
            rows.extend(c)
    return np.asarray(n_part, np.int32), np.asarray(rows, np.int32)


def _transformer_problem(*, name, seed, n_layers, hidden, seq, vocab, n_zones, type_mult,
                         caps_gib, prices, tp_list, mb_list, dp_max, global_batch,
                         max_segments, seg3_max_pp, partitions_per_pp, avail_fn, bw_fn,
                         egress_inter, notes):
    rng = SplitMix64(seed)
    G, Z = len(type_mult), n_zones
    pp_values = _divisors(n_layers)
    dp_values = _pow2_upto(dp_max)
    n_mb, n_tp = len(mb_list), len(tp_list)

    # draw order: (1) times fwd then bwd per (g, mb, tp), (2) update times per (g, tp),
    # (3) availability, (4) bandwidth, (5) partitions.
    base = 1.0e-3 * (hidden / 1024.0) ** 2
    t_fwd = np.zeros((G, n_mb, n_tp, 1))
    t_bwd = np.zeros((G, n_mb, n_tp, 1))
    for g in range(G):
        for m, mb in enumerate(mb_list):
            for t, tp in enumerate(tp_list):
                med = base * mb / tp * type_mult[g]
                t_fwd[g, m, t, 0] = rng.lognormal(med, 0.1)
                t_bwd[g, m, t, 0] = rng.lognormal(med, 0.1)
    t_upd = np.zeros((G, n_tp, 1))
    for g in range(G):
        for t, tp in enumerate(tp_list):
            t_upd[g, t, 0] = rng.lognormal(0.1 * base / tp * type_mult[g], 0.1)
    avail = np.asarray(avail_fn(rng), np.int32).reshape(Z, G)
    bandwidth = np.asarray(bw_fn(rng), np.float64).reshape(Z, Z)
    n_part, part_rows = _partitions(rng, n_layers, pp_values, partitions_per_pp)

    layer_params = np.full(n_layers, 12 * hidden * hidden + 13 * hidden, np.uint64)
    act = np.zeros((n_mb, n_tp), np.uint64)
    for m, mb in enumerate(mb_list):
        for t, tp in enumerate(tp_list):
            # 10 + 24/tp bytes per token per hidden unit, kept integral
            act[m, t] = mb * seq * hidden * 10 + (mb * seq * hidden * 24) // tp
    p2p = np.asarray([mb * seq * hidden * 2 for mb in mb_list], np.uint64)
    egress = None
    if egress_inter is not None:
        egress = np.full((Z, Z), float(egress_inter))
        np.fill_diagonal(egress, 0.0)

    return Problem(
        n_layers=n_layers, n_types=G, n_zones=Z,
        mb_values=np.asarray(mb_list, np.int32), tp_values=np.asarray(tp_list, np.int32),
        dp_values=np.asarray(dp_values, np.int32), pp_values=np.asarray(pp_values, np.int32),
        max_segments=max_segments, seg3_max_pp=seg3_max_pp, global_batch=global_batch,
        n_partitions=n_part, partition_layers=part_rows,
        layer_params=layer_params,
        embed_params=vocab * hidden + seq * hidden, head_params=vocab * hidden,
        bytes_per_param=16, grad_bytes_per_param=2, uniform_layers=True,
        t_fwd=t_fwd, t_bwd=t_bwd, t_upd=t_upd,
        act_store_bytes=act, p2p_bytes=p2p,
        mem_capacity=np.asarray([c * GIB for c in caps_gib], np.uint64),
        mem_reserved=np.full(G, GIB, np.uint64),
        gpus_per_node=np.full(G, 8, np.int32),
        price_per_hour=np.asarray(prices, np.float64),
        avail=avail, bandwidth=bandwidth, egress_per_byte=egress,
        name=name, notes=dict(notes, seed=seed, hidden=hidden, seq=seq, vocab=vocab),
    )


GBIT = 1.0e9 / 8.0  # bytes/s in one Gb/s


def _bw_matrix(rng: SplitMix64, Z: int, intra_gbit: float, lo: float, hi: float):
    bw = np.zeros((Z, Z))
    for a in range(Z):
        for b in range(Z):
            bw[a, b] = intra_gbit * GBIT if a == b else rng.uniform_range(lo, hi) * GBIT
    return bw


def config1(seed: int = 1) -> Problem:
    """OPT-350M-like, one zone, 16 x type A (40 GiB, 2.9 $/h) + 16 x type B (16 GiB, 1.9 $/h)."""
    return _transformer_problem(
        name="cfg1", seed=seed, n_layers=24, hidden=1024, seq=2048, vocab=50272, n_zones=1,
        type_mult=[1.0, 2.2], caps_gib=[40, 16], prices=[2.9, 1.9],
        tp_list=[1, 2, 4], mb_list=[1, 2, 4, 8], dp_max=32, global_batch=256,
        max_segments=2, seg3_max_pp=0, partitions_per_pp=1,
        avail_fn=lambda r: [[16, 16]],
        bw_fn=lambda r: _bw_matrix(r, 1, 100.0, 5.0, 20.0),
        egress_inter=None, notes={"objective": "max throughput (and min cost)"})


def config2(seed: int = 2) -> Problem:
    """Same model, 2 zones x 2 types, 32 GPUs per (zone, type), inter-zone 5-20 Gb/s."""
    return _transformer_problem(
        name="cfg2", seed=seed, n_layers=24, hidden=1024, seq=2048, vocab=50272, n_zones=2,
        type_mult=[1.0, 2.2], caps_gib=[40, 16], prices=[2.9, 1.9],
        tp_list=[1, 2, 4], mb_list=[1, 2, 4, 8], dp_max=64, global_batch=256,
        max_segments=2, seg3_max_pp=0, partitions_per_pp=1,
        avail_fn=lambda r: [[32, 32], [32, 32]],
        bw_fn=lambda r: _bw_matrix(r, 2, 100.0, 5.0, 20.0),
        egress_inter=2.0e-11,
        notes={"objective": "max throughput s.t. cost <= 1.2 x cheapest feasible"})


def config3(seed: int = 3, seg3_max_pp: int = 8) -> Problem:
    """GPT-2.7B-like, 4 zones x 3 types (80/40/16 GiB), 0-128 GPUs per (zone, type)."""
    Z, G = 4, 3
    return _transformer_problem(
        name="cfg3", seed=seed, n_layers=32, hidden=2560, seq=2048, vocab=50272, n_zones=Z,
        type_mult=[0.6, 1.0, 2.2], caps_gib=[80, 40, 16], prices=[4.0, 2.9, 1.9],
        tp_list=[1, 2, 4, 8], mb_list=[1, 2, 4, 8, 16], dp_max=128, global_batch=2048,
        max_segments=3 if seg3_max_pp >= 3 else 2, seg3_max_pp=seg3_max_pp, partitions_per_pp=1,
        avail_fn=lambda r: [[r.randint(0, 128) for _ in range(G)] for _ in range(Z)],
        bw_fn=lambda r: _bw_matrix(r, Z, 100.0, 5.0, 20.0),
        egress_inter=2.0e-11, notes={"objective": "max throughput"})


def config4(seed: int = 4, seg3_max_pp: int = 4) -> Problem:
    """OPT-30B-like, 5 zones x 4 types, up to 256 GPUs each, 8 layer splits per pp."""
    Z, G = 5, 4
    return _transformer_problem(
        name="cfg4", seed=seed, n_layers=48, hidden=7168, seq=2048, vocab=50272, n_zones=Z,
        type_mult=[0.6, 1.0, 2.2, 4.0], caps_gib=[80, 40, 24, 16], prices=[4.0, 2.9, 2.2, 1.9],
        tp_list=[1, 2, 4, 8], mb_list=[1, 2, 4, 8, 16], dp_max=256, global_batch=2048,
        max_segments=3 if seg3_max_pp >= 3 else 2, seg3_max_pp=seg3_max_pp, partitions_per_pp=8,
        avail_fn=lambda r: [[r.randint(0, 256) for _ in range(G)] for _ in range(Z)],
        bw_fn=lambda r: _bw_matrix(r, Z, 100.0, 5.0, 20.0),
        egress_inter=2.0e-11,
        notes={"objective": "min cost s.t. throughput floor; max throughput s.t. budget; top-64"})


def config4_dense(seed: int = 4) -> Problem:
    """The fourth workload with resources that never bind: 100 000 GPUs in every pool and GPU
    memory no plan can exhaust, so that nearly every candidate is a valid plan (only batch
    divisibility rules some out) and an evaluator cannot gain from discarding invalid ones."""
    p = config4(seed)
    return replace(p, name="cfg4_dense", avail=np.full_like(p.avail, 100_000),
                   mem_capacity=np.full_like(p.mem_capacity, 10 ** 15))


def config5_snapshots(base: Problem, n_snapshots: int = 64, seed: int = 5) -> List[np.ndarray]:
    """Availability stream for a cluster: every (zone, type) count follows a +-25 %
    multiplicative random walk clamped to [0, 128]; each zone is, independently per
    snapshot, dropped (all its counts read 0) with probability 0.05 while the walk
    state underneath is kept."""
    rng = SplitMix64(seed)
    Z, G = base.n_zones, base.n_types
    state = base.avail.astype(np.int64).copy()
    out = []
    for _ in range(n_snapshots):
        for z in range(Z):
            for g in range(G):
                f = 1.0 + rng.uniform_range(-0.25, 0.25)
                state[z, g] = min(128, max(0, int(math.floor(state[z, g] * f + 0.5))))
        snap = state.copy()
        for z in range(Z):
            if rng.uniform() < 0.05:
                snap[z, :] = 0
        out.append(snap.astype(np.int32))
    return out


def node_events(base: Problem, n_snapshots: int = 64, seed: int = 7) -> List[np.ndarray]:
    """Availability stream in which one (zone, type) pool changes per snapshot: a few nodes of
    one type join or leave one zone (the 16 -> 20 GPU reconfiguration of Sec. 5.5 is of this
    kind), 4 to 16 GPUs at a time, clamped to [0, 256]."""
    rng = SplitMix64(seed)
    Z, G = base.n_zones, base.n_types
    state = base.avail.astype(np.int64).copy()
    out = []
    for _ in range(n_snapshots):
        z, g = rng.randint(0, Z - 1), rng.randint(0, G - 1)
        step = 4 * rng.randint(1, 4)
        if rng.uniform() < 0.5:
            step = -step
        state[z, g] = min(256, max(0, int(state[z, g]) + step))
        out.append(state.astype(np.int32).copy())
    return out


def bandwidth_poly(prob: Problem, seed: int = 6) -> np.ndarray:
    """Seeded message-size profile of every link: a quadratic in log2(bytes) through
    (1 KiB, 2-8 % of the peak), (1 MiB, 40-70 %) and (128 MiB, the peak), the shape
    of a measured collective-bandwidth curve.  Returns [Z][Z][3], lowest power first."""
    rng = SplitMix64(seed)
    Z = prob.n_zones
    out = np.zeros((Z, Z, 3))
    xs = np.array([10.0, 20.0, 27.0])
    vand = np.stack([xs ** 0, xs, xs ** 2], axis=1)
    for a in range(Z):
        for b in range(Z):
            peak = float(prob.bandwidth[a, b])
            ys = np.array([rng.uniform_range(0.02, 0.08), rng.uniform_range(0.4, 0.7), 1.0]) * peak
            out[a, b] = np.linalg.solve(vand, ys)
    return out


def tiny_problem(seed: int, *, n_layers: int = 6, n_types: int = 2, n_zones: int = 2,
                 max_segments: int = 3, seg3_max_pp: int = 4, uniform_layers: bool = False,
                 partitions_per_pp: int = 3, with_egress: bool = True) -> Problem:
    """A small random problem with non-uniform layers, sized for brute force."""
    rng = SplitMix64(seed)
    G, Z, L = n_types, n_zones, n_layers
    mb_list, tp_list, dp_list = [1, 2, 4], [1, 2, 4], [1, 2, 4, 8]
    pp_values = _divisors(L)
    Lc = 1 if uniform_layers else L
    mult = [rng.uniform_range(0.5, 3.0) for _ in range(G)]
    t_fwd = np.zeros((G, 3, 3, Lc))
    t_bwd = np.zeros((G, 3, 3, Lc))
    t_upd = np.zeros((G, 3, Lc))
    for g in range(G):
        for m, mb in enumerate(mb_list):
            for t, tp in enumerate(tp_list):
                for l in range(Lc):
                    t_fwd[g, m, t, l] = rng.lognormal(1e-3 * mb / tp * mult[g], 0.3)
                    t_bwd[g, m, t, l] = rng.lognormal(2e-3 * mb / tp * mult[g], 0.3)
        for t, tp in enumerate(tp_list):
            for l in range(Lc):
                t_upd[g, t, l] = rng.lognormal(2e-4 / tp * mult[g], 0.3)
    layer_params = np.asarray([rng.randint(1_000_000, 60_000_000) for _ in range(L)], np.uint64)
    act = np.zeros((3, 3), np.uint64)
    for m, mb in enumerate(mb_list):
        for t, tp in enumerate(tp_list):
            act[m, t] = mb * rng.randint(30_000_000, 60_000_000) // tp + 1_000_003
    p2p = np.asarray([mb * rng.randint(2_000_000, 9_000_000) for mb in mb_list], np.uint64)
    caps = np.asarray([rng.randint(1, 6) * GIB // 2 for _ in range(G)], np.uint64)
    res = np.asarray([rng.randint(0, 200_000_000) for _ in range(G)], np.uint64)
    node = np.asarray([rng.randint(1, 3) * 2 for _ in range(G)], np.int32)
    price = np.asarray([rng.uniform_range(0.5, 5.0) for _ in range(G)])
    avail = np.asarray([[rng.randint(0, 24) for _ in range(G)] for _ in range(Z)], np.int32)
    bw = np.zeros((Z, Z))
    for a in range(Z):
        for b in range(Z):
            bw[a, b] = rng.uniform_range(5.0, 12.0) * 1e9 if a == b else rng.uniform_range(0.3, 2.0) * 1e9
    egress = None
    if with_egress:
        egress = np.zeros((Z, Z))
        for a in range(Z):
            for b in range(Z):
                if a != b:
                    egress[a, b] = rng.uniform_range(1e-11, 9e-11)
    n_part, rows = _partitions(rng, L, pp_values, partitions_per_pp)
    return Problem(
        n_layers=L, n_types=G, n_zones=Z,
        mb_values=np.asarray(mb_list, np.int32), tp_values=np.asarray(tp_list, np.int32),
        dp_values=np.asarray(dp_list, np.int32), pp_values=np.asarray(pp_values, np.int32),
        max_segments=max_segments, seg3_max_pp=seg3_max_pp, global_batch=16,
        n_partitions=n_part, partition_layers=rows, layer_params=layer_params,
        embed_params=rng.randint(0, 40_000_000), head_params=rng.randint(0, 40_000_000),
        bytes_per_param=16, grad_bytes_per_param=2, uniform_layers=uniform_layers,
        t_fwd=t_fwd, t_bwd=t_bwd, t_upd=t_upd, act_store_bytes=act, p2p_bytes=p2p,
        mem_capacity=caps, mem_reserved=res, gpus_per_node=node, price_per_hour=price,
        avail=avail, bandwidth=bw, egress_per_byte=egress, name=f"tiny{seed}",
        notes={"seed": seed})
