"""Pins of the oracle's per-segment tensor parallelism (the plan tuple of Sec. 4.2 lets
every stage carry its own TP degree; H1 makes that a property of the GPU type the stage
runs on, so here every contiguous segment -- one pool -- has its own TP digit).

The mode is tied to the shared-TP mode (pinned elsewhere) where the two must agree, and
to closed forms / Python integers where the TP degrees differ between segments.
"""
import itertools
import math

import numpy as np
import pytest

from oracle.oracle import (BIT_BATCH, BIT_OOM, BIT_QUOTA, BIT_TP_NODE, MAX_THROUGHPUT, MIN_COST,
                           Oracle)
from paper_2504_17096_amd import workloads as W
from tests.helpers import make_problem


def expected_count(p):
    """pp, segment count, cut points, an ordered pool per segment (neighbours distinct),
    a TP degree per segment, a partition and (dp, mb)."""
    ZG = p.n_zones * p.n_types
    total = 0
    for ip, P in enumerate(p.pp_values):
        for s in (1, 2, 3):
            if s > p.max_segments or s > P or (s == 3 and P > p.seg3_max_pp):
                continue
            cuts = math.comb(int(P) - 1, s - 1)
            pools = ZG * (ZG - 1) ** (s - 1)
            total += (p.n_mb * p.n_dp * p.n_tp ** s) * cuts * pools * int(p.n_partitions[ip])
    return total


@pytest.mark.parametrize("seed", [1, 2])
def test_space_bijection_count_and_uniqueness(seed):
    p = W.tiny_problem(seed, n_layers=4, partitions_per_pp=2).with_per_segment_tp()
    o = Oracle(p)
    n = o.num_candidates
    assert n == expected_count(p) == o.enumerate_count()
    assert n > Oracle(p.with_per_segment_tp(False)).num_candidates
    seen = set()
    for c, cfg in enumerate(o.enumerate()):
        assert o.decode(c) == cfg and o.encode(cfg) == c
        s = cfg.n_segments
        assert cfg.seg_tp[0] == cfg.tp and cfg.seg_tp_idx[0] == cfg.tp_idx
        assert all(cfg.seg_tp[j] == p.tp_values[cfg.seg_tp_idx[j]] for j in range(s))
        assert cfg.seg_tp[s:] == (0,) * (3 - s) and cfg.seg_tp_idx[s:] == (-1,) * (3 - s)
        key = (cfg.pp, s, cfg.partition, cfg.cut[:s - 1], cfg.pool[:s], cfg.seg_tp[:s], cfg.dp, cfg.mb)
        assert key not in seen
        seen.add(key)


def test_digit_order():
    # mb fastest, then segment 1's tp, dp, its pool; then segment 2's pool and tp
    p = make_problem(n_layers=4, n_types=2, n_zones=2, max_segments=2, pp_list=[2]).with_per_segment_tp()
    o = Oracle(p)
    n_mb, n_tp, n_dp, ZG = p.n_mb, p.n_tp, p.n_dp, 4
    inner = n_mb * n_tp * n_dp * ZG
    one_seg = inner  # the s = 1 block comes first
    base = o.decode(one_seg)
    assert base.n_segments == 2 and base.pool[:2] == (0, 1) and base.seg_tp_idx[:2] == (0, 0)
    assert o.decode(one_seg + inner).pool[:2] == (0, 2)
    nxt = o.decode(one_seg + inner * (ZG - 1))
    assert nxt.pool[:2] == (0, 1) and nxt.seg_tp_idx[:2] == (0, 1)


def test_equal_degrees_reproduce_the_shared_tp_mode_bit_for_bit():
    base = W.tiny_problem(5)
    o_shared, o_seg = Oracle(base), Oracle(base.with_per_segment_tp())
    hits = 0
    for c in range(o_seg.num_candidates):
        g = o_seg.decode(c)
        if len(set(g.seg_tp[:g.n_segments])) != 1:
            continue
        c0 = o_shared.encode(g)
        for obj, bound in ((MAX_THROUGHPUT, None), (MIN_COST, 3.0)):
            a, b = o_seg.eval_one(c, obj, bound), o_shared.eval_one(c0, obj, bound)
            assert (a.mask, a.peak_mem, a.iter_time, a.cost) == (b.mask, b.peak_mem, b.iter_time, b.cost) \
                or (math.isinf(a.iter_time) and a.mask == b.mask)
        hits += 1
    assert hits == o_shared.num_candidates


def stage_table(p, g):
    """(layers, first layer, segment, type, zone, tp, tp index) of every stage."""
    row0 = sum(int(p.n_partitions[i]) * int(p.pp_values[i]) for i in range(g.pp_idx))
    nl = [int(x) for x in p.partition_layers[row0 + g.partition * g.pp: row0 + (g.partition + 1) * g.pp]]
    out, first = [], 0
    for i in range(g.pp):
        seg = 0 if i < g.cut[0] else 1 if i < g.cut[1] else 2
        a = g.pool[seg]
        out.append((nl[i], first, seg, a % p.n_types, a // p.n_types, g.seg_tp[seg], g.seg_tp_idx[seg]))
        first += nl[i]
    return out


@pytest.mark.parametrize("seed", [3, 9])
def test_memory_quota_and_node_bits_against_python_integers(seed):
    p = W.tiny_problem(seed).with_per_segment_tp()
    o = Oracle(p)
    n = o.num_candidates
    mixed = 0
    for c in np.random.default_rng(seed).integers(0, n, 6000):
        c = int(c)
        g, e = o.decode(c), o.eval_one(c)
        if int(p.global_batch) % (g.dp * g.mb):
            assert e.mask == BIT_BATCH
            continue
        nb = int(p.global_batch) // (g.dp * g.mb)
        mem, oom, node, need = [], False, False, {}
        for i, (nl, first, seg, gt, z, tp, ti) in enumerate(stage_table(p, g)):
            params = sum(int(x) for x in p.layer_params[first:first + nl])
            params += int(p.embed_params) if i == 0 else 0
            params += int(p.head_params) if i == g.pp - 1 else 0
            m = -(-params // tp) * int(p.bytes_per_param) + min(g.pp - i, nb) * nl * int(
                p.act_store_bytes[g.mb_idx, ti]) + int(p.mem_reserved[gt])
            mem.append(m)
            oom |= m > int(p.mem_capacity[gt])
            node |= tp > int(p.gpus_per_node[gt])
            need[(z, gt)] = need.get((z, gt), 0) + g.dp * tp
        quota = any(v > int(p.avail[z, gt]) for (z, gt), v in need.items())
        assert e.peak_mem == max(mem)
        assert bool(e.mask & BIT_OOM) == oom
        assert bool(e.mask & BIT_TP_NODE) == node
        assert bool(e.mask & BIT_QUOTA) == quota
        mixed += len(set(g.seg_tp[:g.n_segments])) > 1
    assert mixed > 1000


def two_type_problem(**kw):
    # type 0: fast with TP, type 1: no TP speed-up; one zone, no transfers
    tf = np.zeros((2, 1, 3, 1))
    tf[0, 0, :, 0] = [8e-3, 4e-3, 2e-3]
    tf[1, 0, :, 0] = [6e-3, 5e-3, 4.5e-3]
    args = dict(n_layers=4, n_types=2, mb_list=(1,), tp_list=(1, 2, 4), dp_list=(1, 2), pp_list=[2],
                global_batch=8, max_segments=2, t_fwd=tf, t_bwd=2 * tf, price=np.array([3.0, 1.0]),
                layer_params=1_000_000, act=np.array([[400, 200, 100]], np.uint64))
    args.update(kw)
    return make_problem(**args).with_per_segment_tp()


def test_time_sync_and_cost_with_different_degrees_by_hand():
    p = two_type_problem(bw=1e9, t_upd=np.arange(6, dtype=np.float64).reshape(2, 3, 1) * 1e-4)
    o = Oracle(p)
    checked = 0
    for c in range(o.num_candidates):
        g = o.decode(c)
        if g.n_segments != 2:
            continue
        e = o.eval_one(c)
        (ta, tb), (ia, ib) = g.seg_tp[:2], g.seg_tp_idx[:2]
        ga, gb = g.pool[0], g.pool[1]  # one zone: pool = type
        nb = 8 // g.dp
        t = [3 * 2 * p.t_fwd[ga, 0, ia, 0], 3 * 2 * p.t_fwd[gb, 0, ib, 0]]  # 2 layers, fwd + bwd
        t_pp = sum(t) + (nb - 1) * max(t)
        shard = [-(-2_000_000 // ta), -(-2_000_000 // tb)]
        sync = 0.0 if g.dp == 1 else max(2 * (g.dp - 1) / g.dp * s * 2 / 1e9 for s in shard)
        upd = max(2 * p.t_upd[ga, ia, 0], 2 * p.t_upd[gb, ib, 0])
        T = t_pp + sync + upd
        assert e.iter_time == pytest.approx(T, rel=1e-13)
        dollars = g.dp * (ta * p.price_per_hour[ga] + tb * p.price_per_hour[gb])
        assert e.cost == pytest.approx(dollars / 3600 * T, rel=1e-13)
        checked += 1
    assert checked == 2 * 3 * 3 * 2  # pool orders x tp1 x tp2 x dp


def test_each_segment_is_held_to_its_own_node_size_and_quota():
    p = two_type_problem(node=np.array([4, 1]), avail=np.array([[8, 2]]))
    o = Oracle(p)
    for c in range(o.num_candidates):
        g, e = o.decode(c), o.eval_one(c)
        tp_on = {}
        for j in range(g.n_segments):
            tp_on[g.pool[j]] = g.seg_tp[j]
        assert bool(e.mask & BIT_TP_NODE) == (tp_on.get(1, 1) > 1)
        stages = 2 if g.n_segments == 1 else 1
        over = any(stages * g.dp * t > (8, 2)[a] for a, t in tp_on.items())
        assert bool(e.mask & BIT_QUOTA) == over


def test_third_segment_back_on_the_first_pool_adds_both_degrees_to_its_quota():
    p = make_problem(n_layers=3, n_types=2, mb_list=(1,), tp_list=(1, 2), dp_list=(2,), pp_list=[3],
                     global_batch=2, max_segments=3, seg3_max_pp=3,
                     avail=np.array([[5, 8]])).with_per_segment_tp()
    o = Oracle(p)
    seen = 0
    for c in range(o.num_candidates):
        g = o.decode(c)
        if g.n_segments == 3 and g.pool == (0, 1, 0):
            # pool 0 gives D * (tp1 + tp3) GPUs
            assert bool(o.eval_one(c).mask & BIT_QUOTA) == (2 * (g.seg_tp[0] + g.seg_tp[2]) > 5)
            seen += 1
    assert seen == 8


@pytest.mark.parametrize("objective,bound", [(MAX_THROUGHPUT, None), (MAX_THROUGHPUT, 0.02), (MIN_COST, None)])
def test_a_superset_of_plans_never_has_a_worse_optimum(objective, bound):
    base = W.tiny_problem(21)
    a = Oracle(base).best(objective, bound)
    b = Oracle(base.with_per_segment_tp()).best(objective, bound)
    key = (lambda e: e.iter_time) if objective == MAX_THROUGHPUT else (lambda e: e.cost)
    if a is not None:
        assert b is not None and key(b) <= key(a) * (1 + 1e-12)


def test_selection_against_a_full_sort():
    p = W.tiny_problem(4).with_per_segment_tp()
    o = Oracle(p)
    for objective in (MAX_THROUGHPUT, MIN_COST):
        t, cst, mem, mask = o.eval_batch(objective=objective)
        key = t if objective == MAX_THROUGHPUT else cst
        ok = np.flatnonzero(mask == 0)
        order = ok[np.lexsort((ok, key[ok]))]
        top = o.topk(16, objective)
        assert [e.index for e in top] == order[:16].tolist()
        lo = key[ok].min()
        first = ok[key[ok] <= lo * (1 + 1e-5)][0]
        assert o.best(objective).index == first
