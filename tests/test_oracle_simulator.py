"""Pins of the oracle's simulator (Sec. 4.3: memory, iteration time, cost) against
closed forms, a discrete-event 1F1B schedule, limits, invariants and big-integer
arithmetic.  None of these re-uses the oracle's own formula on its own output.
"""
import math
from dataclasses import replace

import numpy as np
import pytest

from oracle.oracle import (BIT_BATCH, BIT_CONSTRAINT, BIT_OOM, BIT_QUOTA, BIT_TP_NODE,
                           MAX_THROUGHPUT, MIN_COST, Oracle)
from paper_2504_17096_amd import workloads as W
from tests.helpers import GIB, find_index, make_problem


# ---------------------------------------------------------------- 1F1B makespan

def one_f_one_b_makespan(fwd, bwd, n_micro):
    """Discrete-event 1F1B: stage i runs min(P-1-i, M) warm-up forwards, then
    alternates one forward / one backward, then drains its backwards.  A forward
    waits for the previous stage's forward of that microbatch, a backward for the
    next stage's backward."""
    P, M = len(fwd), n_micro
    order = []
    for i in range(P):
        w = min(P - 1 - i, M)
        ops = [("F", m) for m in range(w)]
        for j in range(M - w):
            ops.append(("F", w + j))
            ops.append(("B", j))
        ops += [("B", m) for m in range(M - w, M)]
        order.append(ops)
    done = {}
    pos = [0] * P
    free = [0.0] * P
    progressed = True
    while progressed:
        progressed = False
        for i in range(P):
            while pos[i] < len(order[i]):
                kind, m = order[i][pos[i]]
                if kind == "F":
                    dep = 0.0 if i == 0 else done.get(("F", i - 1, m))
                else:
                    dep = done.get(("F", i, m)) if i == P - 1 else done.get(("B", i + 1, m))
                if dep is None:
                    break
                start = max(free[i], dep)
                free[i] = start + (fwd[i] if kind == "F" else bwd[i])
                done[(kind, i, m)] = free[i]
                pos[i] += 1
                progressed = True
    assert all(pos[i] == len(order[i]) for i in range(P))
    return max(free)


@pytest.mark.parametrize("P,M,tf,tb", [(1, 5, 1.0, 2.0), (4, 1, 1.0, 2.0), (4, 8, 1.0, 2.0),
                                       (8, 3, 0.5, 0.75), (6, 16, 2.0, 3.0)])
def test_discrete_event_schedule_has_the_textbook_makespan(P, M, tf, tb):
    assert one_f_one_b_makespan([tf] * P, [tb] * P, M) == pytest.approx((M + P - 1) * (tf + tb), rel=1e-12)


@pytest.mark.parametrize("pp,dp,mb", [(1, 1, 1), (2, 2, 4), (4, 1, 2), (8, 4, 1), (4, 4, 4), (8, 1, 4)])
def test_homogeneous_pipeline_closed_form_and_event_schedule(pp, dp, mb):
    # one GPU type, no transfers: T = (N_b + P - 1) (t_f + t_b) n_layers_per_stage + all-reduce
    L, B, tf, tb = 8, 32, 1.3e-3, 2.9e-3
    params, gb, bw = 3_000_001, 2, 1.0e9
    p = make_problem(n_layers=L, global_batch=B, t_fwd=tf, t_bwd=tb, layer_params=params,
                     grad_bytes=gb, bw=bw, tp_list=(1, 2))
    o = Oracle(p)
    for tp in (1, 2):
        c = find_index(o, pp=pp, dp=dp, mb=mb, tp=tp)
        e = o.eval_one(c)
        nb = B // (dp * mb)
        per_stage = (L // pp) * (tf + tb)
        shard = -(-(params * (L // pp)) // tp)
        ring = 2.0 * (dp - 1) / dp * shard * gb / bw
        assert e.mask == 0
        assert e.iter_time == pytest.approx((nb + pp - 1) * per_stage + ring, rel=1e-13)
        des = one_f_one_b_makespan([(L // pp) * tf] * pp, [(L // pp) * tb] * pp, nb)
        assert e.iter_time - ring == pytest.approx(des, rel=1e-12)


def test_single_stage_and_single_microbatch_limits():
    # P = 1 -> N_b t ; N_b = 1 -> sum of the stage times (heterogeneous stages)
    L = 6
    tf = np.zeros((1, 1, 1, L)); tb = np.zeros((1, 1, 1, L))
    tf[0, 0, 0] = [1, 2, 3, 4, 5, 6]; tb[0, 0, 0] = [2, 1, 2, 1, 2, 1]
    p = make_problem(n_layers=L, mb_list=(4,), tp_list=(1,), dp_list=(1, 2), global_batch=8,
                     t_fwd=tf * 1e-3, t_bwd=tb * 1e-3, uniform_layers=False, layer_params=0)
    o = Oracle(p)
    e = o.eval_one(find_index(o, pp=1, dp=1))
    assert e.iter_time == pytest.approx(2 * 30e-3, rel=1e-13)          # N_b = 2, t = 30 ms
    e = o.eval_one(find_index(o, pp=3, dp=2))
    assert e.iter_time == pytest.approx(30e-3, rel=1e-13)              # N_b = 1
    e = o.eval_one(find_index(o, pp=3, dp=1))
    # stage times 6, 10, 14 ms; N_b = 2: sum + (N_b - 1) * straggler
    assert e.iter_time == pytest.approx(30e-3 + 14e-3, rel=1e-13)


def test_straggler_sets_the_steady_phase():
    # slowing a non-straggler stage by eps moves T only through the sum term;
    # slowing the straggler moves it N_b times
    L = 4
    base = np.full((1, 1, 1, L), 1e-3)
    base[0, 0, 0, 2] = 5e-3
    eps = 1e-4

    def t_iter(tf):
        p = make_problem(n_layers=L, mb_list=(1,), tp_list=(1,), dp_list=(1,), global_batch=10,
                         t_fwd=tf, t_bwd=0.0, uniform_layers=False, layer_params=0)
        o = Oracle(p)
        return o.eval_one(find_index(o, pp=4)).iter_time

    t0 = t_iter(base)
    slow_other = base.copy(); slow_other[0, 0, 0, 0] += eps
    slow_strag = base.copy(); slow_strag[0, 0, 0, 2] += eps
    assert t_iter(slow_other) - t0 == pytest.approx(eps, rel=1e-9)
    assert t_iter(slow_strag) - t0 == pytest.approx(10 * eps, rel=1e-9)


def test_event_schedule_brackets_on_heterogeneous_pipelines():
    # the closed form is the definition; the schedule is reported beside it.  What always
    # holds for the schedule: a microbatch passes every stage, the slowest stage runs every
    # microbatch, and nothing is slower than one microbatch after the other.
    rng = np.random.default_rng(5)
    for _ in range(50):
        P, M = int(rng.integers(2, 7)), int(rng.integers(1, 12))
        f = rng.uniform(0.5, 2.0, P); b = rng.uniform(0.5, 3.0, P)
        closed = float(np.sum(f + b) + (M - 1) * np.max(f + b))
        des = one_f_one_b_makespan(list(f), list(b), M)
        assert max(np.sum(f + b), M * np.max(f + b)) * (1 - 1e-12) <= des <= M * np.sum(f + b) * (1 + 1e-12)
        assert 0.6 < closed / des < 1.4


# ---------------------------------------------------------------- transfers between stages

def test_two_stage_cross_zone_transfer_by_hand():
    # P = 2, stage 0 in zone 0, stage 1 in zone 1, asymmetric links
    bw = np.array([[8e9, 1e9], [2e9, 8e9]])
    p2p, tf, tb = 4_000_000, 1e-3, 2e-3
    p = make_problem(n_layers=2, n_zones=2, max_segments=2, mb_list=(1,), tp_list=(1,),
                     dp_list=(1,), global_batch=5, t_fwd=tf, t_bwd=tb, p2p=p2p, bw=bw,
                     layer_params=0)
    o = Oracle(p)
    c = next(c for c in range(o.num_candidates)
             if o.decode(c).pool[:2] == (0, 1) and o.decode(c).pp == 2)
    e = o.eval_one(c)
    t0 = tf + tb + p2p / 1e9      # sends activations 0 -> 1
    t1 = tf + tb + p2p / 2e9      # sends gradients 1 -> 0
    assert e.iter_time == pytest.approx(t0 + t1 + 4 * max(t0, t1), rel=1e-13)
    # same pipeline inside one zone: both transfers over the intra-zone link
    c_in = next(c for c in range(o.num_candidates)
                if o.decode(c).pp == 2 and o.decode(c).n_segments == 1 and o.decode(c).pool[0] == 0)
    e_in = o.eval_one(c_in)
    ti = tf + tb + p2p / 8e9
    assert e_in.iter_time == pytest.approx(2 * ti + 4 * ti, rel=1e-13)
    assert e.iter_time > e_in.iter_time


def test_interior_stages_pay_two_transfers_and_infinite_bandwidth_removes_them():
    p2p, tf, tb, bwv = 1_000_000, 1e-3, 1e-3, 1e9
    kw = dict(n_layers=4, mb_list=(1,), tp_list=(1,), dp_list=(1,), global_batch=3,
              t_fwd=tf, t_bwd=tb, p2p=p2p, layer_params=0)
    o = Oracle(make_problem(bw=bwv, **kw))
    e = o.eval_one(find_index(o, pp=4))
    x = p2p / bwv
    stage = [tf + tb + x, tf + tb + 2 * x, tf + tb + 2 * x, tf + tb + x]
    assert e.iter_time == pytest.approx(sum(stage) + 2 * max(stage), rel=1e-13)
    o_inf = Oracle(make_problem(bw=1e300, **kw))
    assert o_inf.eval_one(find_index(o_inf, pp=4)).iter_time == pytest.approx(
        (3 + 4 - 1) * (tf + tb), rel=1e-13)


# ---------------------------------------------------------------- gradient all-reduce

@pytest.mark.parametrize("tp", [1, 2, 4])
def test_ring_all_reduce_alone(tp):
    # no compute, no transfers: T_iter is the all-reduce of the largest stage shard
    params, gb, bwv = 7_000_003, 2, 3.0e9
    p = make_problem(n_layers=4, mb_list=(1,), tp_list=(1, 2, 4), dp_list=(1, 2, 4, 8, 16, 32),
                     global_batch=32, t_fwd=0.0, t_bwd=0.0, layer_params=params, grad_bytes=gb,
                     bw=bwv, embed=11, head=5)
    o = Oracle(p)
    shard = -(-(2 * params + 11) // tp)   # pp = 2: stage 0 carries the embedding
    prev = None
    for dp in (1, 2, 4, 8, 16, 32):
        t = o.eval_one(find_index(o, pp=2, dp=dp, tp=tp)).iter_time
        assert t == pytest.approx(2.0 * (dp - 1) / dp * shard * gb / bwv, rel=1e-13)
        if dp == 1:
            assert t == 0.0
        if prev is not None:
            assert t > prev          # grows with D ...
        prev = t
    assert prev < 2.0 * shard * gb / bwv    # ... towards 2 S / BW from below
    o_fast = Oracle(replace(p, bandwidth=p.bandwidth * 2))
    assert o_fast.eval_one(find_index(o_fast, pp=2, dp=8, tp=tp)).iter_time == pytest.approx(
        0.5 * o.eval_one(find_index(o, pp=2, dp=8, tp=tp)).iter_time, rel=1e-13)


def test_update_time_is_the_slowest_stage():
    tu = np.zeros((1, 1, 6)); tu[0, 0] = [1, 1, 1, 5, 1, 1]
    p = make_problem(n_layers=6, mb_list=(1,), tp_list=(1,), dp_list=(1,), global_batch=1,
                     t_fwd=0.0, t_bwd=0.0, t_upd=tu * 1e-3, uniform_layers=False, layer_params=0)
    o = Oracle(p)
    assert o.eval_one(find_index(o, pp=1)).iter_time == pytest.approx(10e-3, rel=1e-13)
    assert o.eval_one(find_index(o, pp=3)).iter_time == pytest.approx(6e-3, rel=1e-13)
    assert o.eval_one(find_index(o, pp=6)).iter_time == pytest.approx(5e-3, rel=1e-13)


# ---------------------------------------------------------------- memory

@pytest.mark.parametrize("pp,tp,mb,dp", [(1, 1, 1, 1), (2, 2, 2, 1), (4, 4, 4, 2), (8, 1, 2, 4), (8, 2, 1, 1)])
def test_memory_closed_form_uniform_split(pp, tp, mb, dp):
    # embed = head = reserved = 0: M_model = params / (tp pp) * 16; stage 0 holds the
    # most in-flight microbatches, so it attains the peak
    L, B, params, act = 8, 64, 4_194_304, 1_000_000
    p = make_problem(n_layers=L, global_batch=B, layer_params=params, mb_list=(1, 2, 4),
                     tp_list=(1, 2, 4), dp_list=(1, 2, 4), act=np.array(
                         [[act * m // t for t in (1, 2, 4)] for m in (1, 2, 4)]))
    o = Oracle(p)
    e = o.eval_one(find_index(o, pp=pp, tp=tp, mb=mb, dp=dp))
    nb = B // (dp * mb)
    m_model = params * L // (tp * pp) * 16
    assert (params * L) % (tp * pp) == 0
    m_act = min(pp, nb) * (L // pp) * (act * mb // tp)
    assert e.peak_mem == m_model + m_act


def test_memory_monotone_in_microbatch_and_tp():
    p = W.config1()
    o = Oracle(p)
    t, c, mem, mask = o.eval_batch()
    cfgs = [o.decode(i) for i in range(o.num_candidates)]
    table = {}
    for i, g in enumerate(cfgs):
        if mask[i] & BIT_BATCH:
            continue
        table[(g.pp, g.n_segments, g.partition, g.cut, g.pool, g.dp, g.tp_idx, g.mb_idx)] = int(mem[i])
    checked = 0
    for (pp, s, q, cut, pool, dp, it, im), m in table.items():
        up_tp = table.get((pp, s, q, cut, pool, dp, it + 1, im))
        if up_tp is not None:
            assert up_tp <= m
            checked += 1
    assert checked > 1000
    # more microbatch -> more activation bytes per in-flight microbatch, at a fixed number
    # of microbatches per pipeline (dp halves as mb doubles)
    by = {}
    for i, g in enumerate(cfgs):
        if not mask[i] & BIT_BATCH:
            by[(g.pp, g.n_segments, g.cut, g.pool, g.tp, g.dp * g.mb, g.mb)] = int(mem[i])
    inc = 0
    for (pp, s, cut, pool, tp, prod, mb), m in by.items():
        other = by.get((pp, s, cut, pool, tp, prod, mb * 2))
        if other is not None:
            assert other >= m
            inc += 1
    assert inc > 500


def big_int_memory(p, g):
    """Exact Python-integer bytes of every stage of plan g (Sec. 4.3 memory model)."""
    row0 = sum(int(p.n_partitions[i]) * int(p.pp_values[i]) for i in range(g.pp_idx))
    nl = [int(x) for x in p.partition_layers[row0 + g.partition * g.pp: row0 + (g.partition + 1) * g.pp]]
    nb = int(p.global_batch) // (g.dp * g.mb)
    out, first = [], 0
    for i in range(g.pp):
        seg = 0 if i < g.cut[0] else 1 if i < g.cut[1] else 2
        gt = g.pool[seg] % p.n_types
        params = sum(int(x) for x in p.layer_params[first:first + nl[i]])
        params += int(p.embed_params) if i == 0 else 0
        params += int(p.head_params) if i == g.pp - 1 else 0
        shard = (params + g.tp - 1) // g.tp
        m = shard * int(p.bytes_per_param) + min(g.pp - i, nb) * nl[i] * int(
            p.act_store_bytes[g.mb_idx, g.tp_idx]) + int(p.mem_reserved[gt])
        out.append((m, int(p.mem_capacity[gt])))
        first += nl[i]
    return out


@pytest.mark.parametrize("make,n_samples", [(W.config1, None), (W.config2, 4000), (W.config4, 3000),
                                            (lambda: W.tiny_problem(7), None)])
def test_memory_bytes_against_python_integers(make, n_samples):
    p = make()
    o = Oracle(p)
    n = o.num_candidates
    idx = range(n) if n_samples is None else np.random.default_rng(1).integers(0, n, n_samples)
    for c in idx:
        c = int(c)
        g = o.decode(c)
        e = o.eval_one(c)
        if int(p.global_batch) % (g.dp * g.mb):
            assert e.mask == BIT_BATCH and e.peak_mem == 0 and math.isinf(e.iter_time)
            continue
        stages = big_int_memory(p, g)
        assert e.peak_mem == max(m for m, _ in stages) < 2 ** 63
        assert bool(e.mask & BIT_OOM) == any(m > cap for m, cap in stages)


def test_stage_zero_attains_the_peak_on_a_uniform_pipeline():
    p = make_problem(n_layers=8, global_batch=64, act=5_000_000, layer_params=1_000_000)
    o = Oracle(p)
    for c in range(o.num_candidates):
        g = o.decode(c)
        e = o.eval_one(c)
        if e.mask & BIT_BATCH:
            continue
        assert e.peak_mem == big_int_memory(p, g)[0][0]


# ---------------------------------------------------------------- cost

def test_cost_homogeneous_and_price_scaling():
    p = make_problem(n_layers=8, price=2.5, egress=None)
    o = Oracle(p)
    o2 = Oracle(replace(p, price_per_hour=p.price_per_hour * 3.0))
    for c in range(0, o.num_candidates, 7):
        g, e = o.decode(c), o.eval_one(c)
        if e.mask & BIT_BATCH:
            continue
        n_gpu = g.pp * g.dp * g.tp
        assert e.cost == pytest.approx(n_gpu * 2.5 / 3600.0 * e.iter_time, rel=1e-13)
        assert o2.eval_one(c).cost == pytest.approx(3.0 * e.cost, rel=1e-13)


def test_cross_zone_traffic_is_charged_per_boundary_and_direction():
    Z = 2
    eg = np.array([[0.0, 3e-11], [5e-11, 0.0]])
    kw = dict(n_layers=4, n_zones=Z, max_segments=2, mb_list=(2,), tp_list=(1,), dp_list=(2,),
              global_batch=16, p2p=1_000_000, bw=1e9, price=1.0)
    o0 = Oracle(make_problem(egress=None, **kw))
    o1 = Oracle(make_problem(egress=eg, **kw))
    hits = 0
    for c in range(o0.num_candidates):
        g = o0.decode(c)
        e0, e1 = o0.eval_one(c), o1.eval_one(c)
        assert e0.iter_time == e1.iter_time
        if g.n_segments == 1:
            assert e1.cost == e0.cost          # same zone: no egress
        else:
            # B / mb microbatches cross the single boundary in each direction
            extra = (16 // 2) * 1_000_000 * (3e-11 + 5e-11)
            assert e1.cost - e0.cost == pytest.approx(extra, rel=1e-9)
            hits += 1
    assert hits > 0
    # with equal bandwidth everywhere and zero egress a two-zone plan costs what the
    # one-zone plan of the same shape costs
    one = o0.eval_one(find_index(o0, pp=4, n_segments=1)).cost
    two = o0.eval_one(find_index(o0, pp=4, n_segments=2)).cost
    assert one == pytest.approx(two, rel=1e-13)


def test_cost_does_not_fall_when_dp_doubles_on_a_fixed_pipeline():
    # doubling D doubles the GPUs but does not halve the time (H4, Sec. 4.2.1)
    p = W.config1()
    o = Oracle(p)
    t, c, mem, mask = o.eval_batch()
    by = {}
    for i in range(o.num_candidates):
        g = o.decode(i)
        if not mask[i] & BIT_BATCH:
            by[(g.pp, g.n_segments, g.cut, g.pool, g.tp, g.mb, g.dp)] = (t[i], c[i])
    n = 0
    for (pp, s, cut, pool, tp, mb, dp), (ti, ci) in by.items():
        nxt = by.get((pp, s, cut, pool, tp, mb, dp * 2))
        if nxt:
            assert nxt[0] > 0.5 * ti * (1 - 1e-12)
            assert nxt[1] >= ci * (1 - 1e-12)
            n += 1
    assert n > 1000


# ---------------------------------------------------------------- feasibility bits

def test_batch_divisibility_tp_node_and_quota_bits():
    p = make_problem(n_layers=4, n_types=2, mb_list=(1, 3), tp_list=(1, 2, 4), dp_list=(1, 2, 4),
                     global_batch=8, node=np.array([2, 8]), avail=np.array([[3, 64]]),
                     max_segments=2)
    o = Oracle(p)
    for c in range(o.num_candidates):
        g, e = o.decode(c), o.eval_one(c)
        if 8 % (g.dp * g.mb):
            assert e.mask == BIT_BATCH
            continue
        types = {a % 2 for a in g.pool[:g.n_segments]}
        assert bool(e.mask & BIT_TP_NODE) == (g.tp > 2 and 0 in types)  # tp = node size is fine
        stages = {0: 0, 1: 0}
        for i in range(g.pp):
            seg = 0 if i < g.cut[0] else 1
            stages[g.pool[seg]] += 1
        over = stages[0] * g.dp * g.tp > 3 or stages[1] * g.dp * g.tp > 64
        assert bool(e.mask & BIT_QUOTA) == over


def test_third_segment_returning_to_the_first_pool_shares_its_quota():
    p = make_problem(n_layers=3, n_types=2, mb_list=(1,), tp_list=(1,), dp_list=(2,),
                     pp_list=[3], global_batch=2, max_segments=3, seg3_max_pp=3,
                     avail=np.array([[3, 8]]))
    o = Oracle(p)
    seen = 0
    for c in range(o.num_candidates):
        g = o.decode(c)
        if g.n_segments == 3 and g.pool == (0, 1, 0):
            # pool 0 hosts two stages x D = 2 -> 4 GPUs > 3
            assert o.eval_one(c).mask & BIT_QUOTA
            seen += 1
        if g.n_segments == 3 and g.pool == (1, 0, 1):
            assert not o.eval_one(c).mask & BIT_QUOTA
            seen += 1
    assert seen == 2


def test_raising_availability_or_capacity_never_removes_a_feasible_plan():
    p = W.tiny_problem(11)
    o = Oracle(p)
    m0 = o.eval_batch()[3]
    more = p.avail.copy(); more[0, 0] += 5; more[-1, -1] += 1
    m1 = Oracle(p.with_avail(more)).eval_batch()[3]
    assert not np.any((m0 & BIT_QUOTA == 0) & (m1 & BIT_QUOTA != 0))
    assert np.array_equal(m0 & ~np.uint32(BIT_QUOTA), m1 & ~np.uint32(BIT_QUOTA))
    bigger = replace(p, mem_capacity=p.mem_capacity + np.uint64(GIB))
    m2 = Oracle(bigger).eval_batch()[3]
    assert not np.any((m0 & BIT_OOM == 0) & (m2 & BIT_OOM != 0))
    assert np.any((m0 & BIT_OOM != 0) & (m2 & BIT_OOM == 0))


def test_constraint_bit_follows_the_objective():
    p = W.tiny_problem(3)
    o = Oracle(p)
    t, c, _, m = o.eval_batch()
    ok = (m & BIT_BATCH) == 0
    budget = float(np.median(c[ok]))
    mt = o.eval_batch(objective=MAX_THROUGHPUT, bound=budget)[3]
    assert np.array_equal((mt & BIT_CONSTRAINT) != 0, ok & (c > budget))
    floor = float(np.median(1.0 / t[ok]))
    mc = o.eval_batch(objective=MIN_COST, bound=floor)[3]
    assert np.array_equal((mc & BIT_CONSTRAINT) != 0, ok & (1.0 / t < floor))
    assert np.array_equal(mt & ~np.uint32(BIT_CONSTRAINT), m)


# ---------------------------------------------------------------- invariances

def test_iteration_time_never_rises_with_bandwidth():
    p = W.tiny_problem(5)
    o = Oracle(p)
    t0 = o.eval_batch()[0]
    for a in range(p.n_zones):
        for b in range(p.n_zones):
            bw = p.bandwidth.copy(); bw[a, b] *= 1.7
            t1 = Oracle(replace(p, bandwidth=bw)).eval_batch()[0]
            fin = np.isfinite(t0)
            assert np.all(t1[fin] <= t0[fin] * (1 + 1e-15))
            assert np.any(t1[fin] < t0[fin])
