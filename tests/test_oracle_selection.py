"""Pins of the oracle's plan selection (Sec. 4.2: sort by the objective, return the
best valid plan) by brute force on small spaces and by monotonicity."""
from dataclasses import replace

import numpy as np
import pytest

from oracle.oracle import BIT_CONSTRAINT, MAX_THROUGHPUT, MIN_COST, Oracle
from paper_2504_17096_amd import workloads as W
from tests.helpers import make_problem

TOL = 1e-5


def brute_best(key, mask):
    ok = np.flatnonzero(mask == 0)
    if len(ok) == 0:
        return None
    vmin = key[ok].min()
    return int(ok[key[ok] <= vmin * (1 + TOL)][0])


def brute_topk(key, mask, k):
    ok = np.flatnonzero(mask == 0)
    order = np.lexsort((ok, key[ok]))
    return [int(i) for i in ok[order][:k]]


@pytest.mark.parametrize("seed", range(1, 9))
@pytest.mark.parametrize("objective", [MAX_THROUGHPUT, MIN_COST])
def test_best_and_topk_against_full_sort(seed, objective):
    p = W.tiny_problem(seed)
    o = Oracle(p)
    t, c, mem, mask = o.eval_batch(objective=objective)
    key = t if objective == MAX_THROUGHPUT else c
    for bound in (None, "median"):
        b = None
        if bound == "median":
            ok = mask == 0
            if not ok.any():
                continue
            b = float(np.median(c[ok])) if objective == MAX_THROUGHPUT else float(np.median(1.0 / t[ok]))
            mask_b = o.eval_batch(objective=objective, bound=b)[3]
        else:
            mask_b = mask
        want = brute_best(key, mask_b)
        for threads in (1, 3):
            got = o.best(objective=objective, bound=b, n_threads=threads)
            assert (got.index if got else None) == want
            top = o.topk(10, objective=objective, bound=b, n_threads=threads)
            assert [e.index for e in top] == brute_topk(key, mask_b, 10)
        if got:
            assert got.mask == 0 and got.peak_mem == mem[want]
            assert got.iter_time == t[want] and got.cost == c[want]


def test_near_ties_go_to_the_lowest_index():
    # two GPU types whose times differ by 4e-6 relative: the slower one comes first in
    # index order and must win; at 4e-5 it must not
    for rel, expect_first in ((4e-6, True), (4e-5, False)):
        tf = np.zeros((2, 1, 1, 1)); tf[0] = 1e-3 * (1 + rel); tf[1] = 1e-3
        p = make_problem(n_layers=2, n_types=2, mb_list=(1,), tp_list=(1,), dp_list=(1,),
                         pp_list=[1], global_batch=4, t_fwd=tf, t_bwd=0.0, layer_params=0)
        o = Oracle(p)
        assert o.num_candidates == 2
        best = o.best()
        assert best.index == (0 if expect_first else 1)
        # top-k stays strictly sorted by (key, index)
        assert [e.index for e in o.topk(2)] == [1, 0]


def test_tolerance_is_relative_to_the_minimum_not_chained():
    # keys 1+1.6e-5, 1+0.8e-5, 1 in index order: index 1 is within 1e-5 of the minimum,
    # index 0 is not (although it is within 1e-5 of index 1)
    tf = np.zeros((3, 1, 1, 1)); tf[:, 0, 0, 0] = [1 + 1.6e-5, 1 + 0.8e-5, 1.0]
    p = make_problem(n_layers=1, n_types=3, mb_list=(1,), tp_list=(1,), dp_list=(1,), pp_list=[1],
                     global_batch=1, t_fwd=tf, t_bwd=0.0, layer_params=0)
    assert Oracle(p).best().index == 1


def test_no_feasible_plan():
    p = make_problem(n_layers=2, avail=0)
    o = Oracle(p)
    assert o.best() is None and o.topk(5) == []


def test_looser_budget_and_more_gpus_never_hurt():
    p = W.config1()
    o = Oracle(p)
    cheapest = o.best(objective=MIN_COST)
    prev = None
    for factor in (1.0 + 1e-9, 1.1, 1.2, 1.5, 3.0):
        b = o.best(objective=MAX_THROUGHPUT, bound=cheapest.cost * factor)
        assert b is not None and b.cost <= cheapest.cost * factor
        if prev is not None:
            assert b.iter_time <= prev * (1 + TOL)
        prev = b.iter_time
    unconstrained = o.best(objective=MAX_THROUGHPUT).iter_time
    assert unconstrained <= prev * (1 + TOL)
    fewer = Oracle(p.with_avail(p.avail // 2)).best(objective=MAX_THROUGHPUT).iter_time
    assert unconstrained <= fewer * (1 + TOL)


def test_best_dp_follows_the_link_speed_and_time_is_affine_in_one_over_dp():
    # sync time grows with D while compute time shrinks (H3): both the microbatch count
    # B / (D mb) and the ring factor 2 (D - 1) / D are affine in 1 / D, so is T_iter, and
    # the best D sits at an end of the list chosen by the intra-zone link speed
    kw = dict(n_layers=4, mb_list=(1,), tp_list=(1,), dp_list=(1, 2, 4, 8, 16, 32),
              pp_list=[2], global_batch=32, layer_params=50_000_000, t_fwd=1e-3, t_bwd=2e-3)
    slow, fast = Oracle(make_problem(bw=2e8, **kw)), Oracle(make_problem(bw=2e11, **kw))
    assert slow.decode(slow.best().index).dp == 1
    assert fast.decode(fast.best().index).dp == 32
    for o in (slow, fast):
        t = {o.decode(c).dp: o.eval_one(c).iter_time for c in range(o.num_candidates)}
        for d in (1, 2, 4, 8):
            assert t[d] - t[2 * d] == pytest.approx(2 * (t[2 * d] - t[4 * d]), rel=1e-9)


def test_relabelling_zones_keeps_the_optimum_value():
    p = W.tiny_problem(4, n_zones=3, n_layers=4)
    perm = [2, 0, 1]
    q = replace(p, avail=p.avail[perm].copy(),
                bandwidth=p.bandwidth[np.ix_(perm, perm)].copy(),
                egress_per_byte=p.egress_per_byte[np.ix_(perm, perm)].copy())
    for objective in (MAX_THROUGHPUT, MIN_COST):
        a, b = Oracle(p).best(objective=objective), Oracle(q).best(objective=objective)
        ka = a.iter_time if objective == MAX_THROUGHPUT else a.cost
        kb = b.iter_time if objective == MAX_THROUGHPUT else b.cost
        assert ka == pytest.approx(kb, rel=1e-12)


def test_two_pass_budget_workflow_of_the_second_workload():
    # cheapest feasible plan first, then max throughput under 1.2 x its cost
    p = W.config2()
    o = Oracle(p)
    cheapest = o.best(objective=MIN_COST, n_threads=4)
    best = o.best(objective=MAX_THROUGHPUT, bound=1.2 * cheapest.cost, n_threads=4)
    assert best.mask == 0 and best.cost <= 1.2 * cheapest.cost
    t, c, _, m = o.eval_batch(objective=MAX_THROUGHPUT, bound=1.2 * cheapest.cost, n_threads=4)
    assert best.index == brute_best(t, m)
    assert np.count_nonzero(m & BIT_CONSTRAINT) > 0
