"""Pins of the oracle's mixed replicas: the D replicas of a stage split over two GPU types of
one zone (the D tuples of the plan, Sec. 4.2; the slower replica is the straggler, Sec. 4.3).

Expected values come from the plain-type mode (pinned elsewhere), from hand-written formulas
and from Python-integer bookkeeping written here.
"""
import itertools
import math

import numpy as np
import pytest

from oracle.oracle import (BIT_BATCH, BIT_OOM, BIT_QUOTA, BIT_TP_NODE, MAX_THROUGHPUT, MIN_COST,
                           Oracle)
from paper_2504_17096_amd import workloads as W
from tests.helpers import GIB, make_problem


def extended_types(G):
    """(a, b) per extended type: the plain ones, then the pairs a < b in lexicographic order."""
    return [(a, a) for a in range(G)] + list(itertools.combinations(range(G), 2))


def expected_count(p):
    GX = len(extended_types(p.n_types))
    ZG = p.n_zones * GX
    total = 0
    for ip, P in enumerate(p.pp_values):
        for s in (1, 2, 3):
            if s > p.max_segments or s > P or (s == 3 and P > p.seg3_max_pp):
                continue
            tps = p.n_tp ** s if p.per_segment_tp else p.n_tp
            total += (p.n_mb * p.n_dp * tps) * math.comb(int(P) - 1, s - 1) * ZG * (ZG - 1) ** (s - 1) * int(
                p.n_partitions[ip])
    return total


@pytest.mark.parametrize("seed,types", [(1, 2), (2, 3)])
def test_space_count_bijection_and_pool_numbering(seed, types):
    p = W.tiny_problem(seed, n_layers=4, n_types=types, partitions_per_pp=1).with_mixed_types()
    o = Oracle(p)
    n = o.num_candidates
    assert n == expected_count(p) == o.enumerate_count()
    assert n > Oracle(p.with_mixed_types(False)).num_candidates
    GX = len(extended_types(types))
    seen = set()
    for c, cfg in enumerate(o.enumerate()):
        assert o.decode(c) == cfg and o.encode(cfg) == c
        pools = cfg.pool[:cfg.n_segments]
        assert all(0 <= a < p.n_zones * GX for a in pools)
        assert all(pools[j] != pools[j + 1] for j in range(len(pools) - 1))
        key = (cfg.pp, cfg.n_segments, cfg.partition, cfg.cut[:cfg.n_segments - 1], pools, cfg.dp,
               cfg.seg_tp[:cfg.n_segments], cfg.mb)
        assert key not in seen
        seen.add(key)


def test_one_gpu_type_has_nothing_to_mix():
    p = W.tiny_problem(6, n_zones=2, n_types=1)
    a, b = Oracle(p).eval_batch(), Oracle(p.with_mixed_types()).eval_batch()
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


def test_plain_types_evaluate_as_without_the_flag():
    base = W.tiny_problem(5)
    G = base.n_types
    GX = len(extended_types(G))
    o0, o1 = Oracle(base), Oracle(base.with_mixed_types())
    hits = 0
    for c in range(o1.num_candidates):
        g = o1.decode(c)
        pools = g.pool[:g.n_segments]
        if any(a % GX >= G for a in pools):
            continue
        # the same plan in the plain numbering: zone * G + type
        plain = tuple((a // GX) * G + a % GX for a in pools) + (-1,) * (3 - g.n_segments)
        g0 = type(g)(**{**g.__dict__, "pool": plain})
        c0 = o0.encode(g0)
        for obj, bound in ((MAX_THROUGHPUT, None), (MIN_COST, 2.0)):
            x, y = o1.eval_one(c, obj, bound), o0.eval_one(c0, obj, bound)
            assert (x.mask, x.peak_mem) == (y.mask, y.peak_mem)
            assert (x.iter_time == y.iter_time and x.cost == y.cost) or math.isinf(y.iter_time)
        hits += 1
    assert hits == o0.num_candidates


def two_type_problem(**kw):
    # type 0 fast and dear, type 1 slow and cheap; one zone
    tf = np.zeros((2, 1, 2, 1))
    tf[0, 0, :, 0] = [4e-3, 2e-3]
    tf[1, 0, :, 0] = [6e-3, 5e-3]
    args = dict(n_layers=4, n_types=2, mb_list=(1,), tp_list=(1, 2), dp_list=(1, 2, 4), pp_list=[1, 2],
                global_batch=8, max_segments=2, t_fwd=tf, t_bwd=2 * tf, price=np.array([3.0, 1.0]),
                t_upd=np.array([1e-4, 1e-4, 3e-4, 2e-4]).reshape(2, 2, 1), layer_params=1_000_000,
                act=1000, bw=1e9)
    args.update(kw)
    return make_problem(**args).with_mixed_types()


def test_mixed_stage_runs_at_the_pace_of_its_slower_type_and_pays_the_mean_price():
    p = two_type_problem()
    o = Oracle(p)
    checked = 0
    for c in range(o.num_candidates):
        g = o.decode(c)
        if g.n_segments != 1 or g.pool[0] != 2 or g.dp % 2:  # extended type 2 = the pair (0, 1)
            continue
        e = o.eval_one(c)
        nl = 4 // g.pp
        t = nl * 3 * p.t_fwd[1, 0, g.tp_idx, 0]                      # the slow type, fwd + bwd
        nb = 8 // g.dp
        shard = -(-(nl * 1_000_000) // g.tp)
        ring = 2 * (g.dp - 1) / g.dp * shard * 2 / 1e9
        upd = nl * max(p.t_upd[0, g.tp_idx, 0], p.t_upd[1, g.tp_idx, 0])
        T = (nb + g.pp - 1) * t + ring + upd
        assert e.mask == 0 and e.iter_time == pytest.approx(T, rel=1e-13)
        rent = g.pp * g.dp * g.tp * 0.5 * (3.0 + 1.0)                # $ per hour
        assert e.cost == pytest.approx(rent / 3600 * T, rel=1e-13)
        checked += 1
    assert checked == 2 * 2 * 2  # pp x tp x even dp


def test_the_straggler_is_chosen_per_stage():
    # non-uniform layers: type 0 is slower on the first layers, type 1 on the last ones
    L = 4
    tf = np.zeros((2, 1, 1, L)); tf[0, 0, 0] = [5, 5, 1, 1]; tf[1, 0, 0] = [2, 2, 4, 4]
    p = make_problem(n_layers=L, n_types=2, mb_list=(1,), tp_list=(1,), dp_list=(2,), pp_list=[2],
                     global_batch=4, t_fwd=tf * 1e-3, t_bwd=0.0, uniform_layers=False,
                     layer_params=0).with_mixed_types()
    o = Oracle(p)
    c = next(c for c in range(o.num_candidates) if o.decode(c).pool[0] == 2)
    # stage 0 (layers 0, 1): max(10, 4) = 10 ms ; stage 1 (layers 2, 3): max(2, 8) = 8 ms ; N_b = 2
    assert o.eval_one(c).iter_time == pytest.approx((10e-3 + 8e-3) + 1 * 10e-3, rel=1e-13)
    ev, closed = o.simulate_1f1b(c)
    assert closed == pytest.approx(28e-3, rel=1e-13) and ev <= closed


def test_both_types_must_fit_memory_and_node_and_odd_degrees_cannot_be_halved():
    p = two_type_problem(cap=np.array([64 * GIB, 24_000_000], np.uint64), node=np.array([8, 1]),
                         layer_params=1_000_000, bytes_per_param=16)
    o = Oracle(p)
    for c in range(o.num_candidates):
        g, e = o.decode(c), o.eval_one(c)
        if e.mask == BIT_BATCH:
            continue
        kinds = [a for a in g.pool[:g.n_segments]]
        uses_small = any(a in (1, 2) for a in kinds)   # plain type 1 or the pair
        assert bool(e.mask & BIT_TP_NODE) == (uses_small and g.tp > 1)
        # a worker holds nl layers x 16 MB / tp (+ 1 000 B x in-flight x nl activations)
        oom = False
        for i in range(g.pp):
            seg = 0 if i < g.cut[0] else 1
            nl = 4 // g.pp
            m = -(-(nl * 1_000_000) // g.tp) * 16 + min(g.pp - i, 8 // g.dp) * nl * 1000
            oom |= g.pool[seg] in (1, 2) and m > 24_000_000
        assert bool(e.mask & BIT_OOM) == oom
        if any(a == 2 for a in kinds) and g.dp % 2:
            assert e.mask & BIT_QUOTA


@pytest.mark.parametrize("seed", [3, 8])
def test_every_real_pool_holds_what_all_segments_take_from_it(seed):
    p = W.tiny_problem(seed, n_types=3, n_zones=2).with_mixed_types().with_per_segment_tp()
    avail = p.avail.copy()
    avail[:] = np.random.default_rng(seed).integers(2, 14, avail.shape)
    p = p.with_avail(avail)
    o = Oracle(p)
    xt = extended_types(3)
    GX = len(xt)
    rng = np.random.default_rng(seed)
    shared = 0
    for c in rng.integers(0, o.num_candidates, 8000):
        c = int(c)
        g, e = o.decode(c), o.eval_one(c)
        if e.mask == BIT_BATCH:
            continue
        half = {}
        odd = False
        for i in range(g.pp):
            seg = 0 if i < g.cut[0] else 1 if i < g.cut[1] else 2
            z, (a, b) = g.pool[seg] // GX, xt[g.pool[seg] % GX]
            if a == b:
                half[(z, a)] = half.get((z, a), 0) + 2 * g.seg_tp[seg]
            else:
                half[(z, a)] = half.get((z, a), 0) + g.seg_tp[seg]
                half[(z, b)] = half.get((z, b), 0) + g.seg_tp[seg]
                odd |= g.dp % 2 == 1
        over = odd or any(h * g.dp > 2 * int(p.avail[z, t]) for (z, t), h in half.items())
        assert bool(e.mask & BIT_QUOTA) == over
        # plans whose segments draw on one real pool together
        pools_of = [set((g.pool[j] // GX, t) for t in xt[g.pool[j] % GX]) for j in range(g.n_segments)]
        shared += any(pools_of[i] & pools_of[j] for i in range(len(pools_of)) for j in range(i))
    assert shared > 500


def test_twin_types_behave_like_one_type_with_two_half_quotas():
    # two identical types: a mixed stage equals a plain one, but takes half from each pool
    p = make_problem(n_layers=4, n_types=2, mb_list=(1,), tp_list=(1, 2), dp_list=(2, 4), pp_list=[2],
                     global_batch=8, max_segments=1, avail=np.array([[8, 8]]), layer_params=3_000_000,
                     bw=1e9).with_mixed_types()
    o = Oracle(p)
    by = {}
    for c in range(o.num_candidates):
        g = o.decode(c)
        by[(g.pool[0], g.dp, g.tp)] = o.eval_one(c)
    for dp in (2, 4):
        for tp in (1, 2):
            plain, mixed = by[(0, dp, tp)], by[(2, dp, tp)]
            assert (mixed.iter_time, mixed.cost, mixed.peak_mem) == (plain.iter_time, plain.cost, plain.peak_mem)
            assert bool(plain.mask & BIT_QUOTA) == (2 * dp * tp > 8)   # two stages on one pool
            assert bool(mixed.mask & BIT_QUOTA) == (2 * dp * tp > 16)  # half of it on each


@pytest.mark.parametrize("objective,bound", [(MAX_THROUGHPUT, None), (MAX_THROUGHPUT, 0.02), (MIN_COST, None)])
def test_a_superset_of_plans_never_has_a_worse_optimum(objective, bound):
    base = W.tiny_problem(21, n_types=3)
    a = Oracle(base).best(objective, bound)
    b = Oracle(base.with_mixed_types()).best(objective, bound)
    key = (lambda e: e.iter_time) if objective == MAX_THROUGHPUT else (lambda e: e.cost)
    if a is not None:
        assert b is not None and key(b) <= key(a) * (1 + 1e-12)


def test_scarce_fast_gpus_make_a_mixed_plan_the_best():
    # 2 fast GPUs and 2 slow ones: D = 4 only fits when the replicas are split over both types
    tf = np.zeros((2, 1, 1, 1)); tf[0] = 1e-3; tf[1] = 1.2e-3
    p = make_problem(n_layers=2, n_types=2, mb_list=(1,), tp_list=(1,), dp_list=(1, 2, 4), pp_list=[1],
                     global_batch=64, t_fwd=tf, t_bwd=2 * tf, avail=np.array([[2, 2]]),
                     layer_params=1000, bw=1e11)
    best_plain = Oracle(p).best()
    o = Oracle(p.with_mixed_types())
    best = o.best()
    assert o.decode(best.index).pool[0] == 2 and o.decode(best.index).dp == 4
    assert best.iter_time < best_plain.iter_time
