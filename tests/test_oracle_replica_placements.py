"""Pins of the oracle's evaluation of plans in which every replica of every stage names its pool
(the D tuples of a stage, Sec. 4.2; T_iter = max over the pipelines + T_sync + T_update,
Sec. 4.3): reduction to the two already pinned evaluators, cases by hand, invariances."""
import numpy as np
import pytest

from oracle.oracle import MAX_THROUGHPUT, MIN_COST, Oracle
from paper_2504_17096_amd import workloads as W
from tests.helpers import make_problem

BIT_OOM, BIT_QUOTA, BIT_BATCH, BIT_TP_NODE = 1, 2, 4, 8


def _same(a, b, rel=1e-13):
    assert (a.mask, a.peak_mem) == (b.mask, b.peak_mem)
    if np.isinf(b.iter_time):
        assert np.isinf(a.iter_time) and np.isinf(a.cost)
    else:
        assert a.iter_time == pytest.approx(b.iter_time, rel=rel) and a.cost == pytest.approx(b.cost, rel=rel)


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_replicas_that_agree_reduce_to_the_evaluators_with_one_or_two_pools_per_stage(seed):
    prob = W.tiny_problem(seed, n_types=2 + seed % 2, n_zones=2 + seed % 2, seg3_max_pp=64)
    orc = Oracle(prob)
    rng = np.random.default_rng(seed)
    zg = prob.n_zones * prob.n_types
    checked = 0
    for _ in range(1200):
        ip = int(rng.integers(0, len(prob.pp_values)))
        P = int(prob.pp_values[ip])
        q, it = int(rng.integers(0, prob.n_partitions[ip])), int(rng.integers(0, len(prob.tp_values)))
        idp, im = int(rng.integers(0, len(prob.dp_values))), int(rng.integers(0, len(prob.mb_values)))
        D = int(prob.dp_values[idp])
        # a few runs of pools rather than white noise, so that valid plans are not rare
        cuts = np.sort(rng.integers(0, P + 1, int(rng.integers(0, 3))))
        pa = rng.integers(0, zg, len(cuts) + 1)[np.searchsorted(cuts, np.arange(P), side="right")]
        pb = np.where(rng.random(P) < 0.5, pa, rng.integers(0, zg, P))
        for objective, bound in ((MAX_THROUGHPUT, None), (MIN_COST, 0.5)):
            one = np.repeat(pa[:, None], D, axis=1)
            _same(orc.eval_replica_assignment(ip, q, idp, im, it, one, objective, bound),
                  orc.eval_assignment(ip, q, idp, im, it, pa, objective, bound))
            if D % 2 == 0:  # the first half of the replicas on one pool, the second half on another
                two = np.concatenate([np.repeat(pa[:, None], D // 2, axis=1), np.repeat(pb[:, None], D // 2, axis=1)], axis=1)
                want = orc.eval_split_assignment(ip, q, idp, im, it, pa, pb, objective, bound)
                tight = bound is not None and np.isfinite(want.iter_time) and abs(1.0 / want.iter_time / bound - 1) < 1e-9
                if not tight:
                    _same(orc.eval_replica_assignment(ip, q, idp, im, it, two, objective, bound), want)
                checked += want.mask == 0
    assert checked > 20


def _three_zones(**kw):
    # one stage of one layer, TP 1, 6 microbatches in all; three zones of one GPU type
    bw = np.array([[1e10, 4e8, 9e8], [5e8, 2e10, 2e8], [3e8, 6e8, 3e10]])
    eg = np.array([[0.0, 1e-9, 2e-9], [3e-9, 0.0, 4e-9], [5e-9, 6e-9, 0.0]])
    args = dict(n_layers=1, n_types=1, n_zones=3, mb_list=(1,), tp_list=(1,), dp_list=(3,), pp_list=[1],
                global_batch=6, t_fwd=1e-3, t_bwd=2e-3, t_upd=4e-4, p2p=0, bw=bw, egress=eg,
                layer_params=3_000_000, price=np.array([3600.0]), avail=2)
    args.update(kw)
    return make_problem(**args)


def test_a_ring_through_three_zones_by_hand():
    orc = Oracle(_three_zones())
    e = orc.eval_replica_assignment(0, 0, 0, 0, 0, [[0, 1, 2]])
    # 2 microbatches per pipeline of 3 ms; ring 2 * 2/3 * 6 MB = 8 MB over 0->1, 1->2, 2->0: the
    # slowest is 1->2 at 0.2 GB/s; every ring link crosses zones and is paid in its direction
    T = 2 * 3e-3 + 8e6 / 2e8 + 4e-4
    assert e.mask == 0 and e.iter_time == pytest.approx(T, rel=1e-14)
    assert e.cost == pytest.approx(3 * T + 8e6 * (1e-9 + 4e-9 + 5e-9), rel=1e-14)
    # the other way round the ring uses the other three links: 0->2, 2->1, 1->0, slowest 1->0 at 0.5 GB/s
    back = orc.eval_replica_assignment(0, 0, 0, 0, 0, [[0, 2, 1]])
    assert back.iter_time == pytest.approx(2 * 3e-3 + 8e6 / 5e8 + 4e-4, rel=1e-14)
    assert back.cost == pytest.approx(3 * back.iter_time + 8e6 * (2e-9 + 6e-9 + 3e-9), rel=1e-14)
    # a rotation of the replicas is the same ring and the same pipelines
    rot = orc.eval_replica_assignment(0, 0, 0, 0, 0, [[1, 2, 0]])
    assert rot.iter_time == pytest.approx(e.iter_time, rel=1e-14) and rot.cost == pytest.approx(e.cost, rel=1e-14)
    # two replicas in zone 0, one in zone 1: links 0->0, 0->1, 1->0; zone 0 gives two GPUs, not three
    un = orc.eval_replica_assignment(0, 0, 0, 0, 0, [[0, 0, 1]])
    assert un.mask == 0 and un.iter_time == pytest.approx(2 * 3e-3 + 8e6 / 4e8 + 4e-4, rel=1e-14)
    assert un.cost == pytest.approx(3 * un.iter_time + 8e6 * (1e-9 + 3e-9), rel=1e-14)
    assert orc.eval_replica_assignment(0, 0, 0, 0, 0, [[0, 0, 0]]).mask == BIT_QUOTA


def test_which_replicas_form_a_pipeline_matters():
    # two stages, D = 2, two types in one zone: type 1 takes three times as long.  Replica r of
    # every stage is pipeline r: (fast, fast) and (slow, slow) wait for the all-slow pipeline;
    # (fast, slow) and (slow, fast) have one slow stage each
    tf = np.zeros((2, 1, 1, 1)); tf[:, 0, 0, 0] = (1e-3, 3e-3)
    p = make_problem(n_layers=2, n_types=2, n_zones=1, mb_list=(1,), tp_list=(1,), dp_list=(2,), pp_list=[2],
                     global_batch=8, t_fwd=tf, t_bwd=0.0, layer_params=0, p2p=0, price=np.array([3.0, 1.0]))
    orc = Oracle(p)
    straight = orc.eval_replica_assignment(0, 0, 0, 0, 0, [[0, 1], [0, 1]])
    crossed = orc.eval_replica_assignment(0, 0, 0, 0, 0, [[0, 1], [1, 0]])
    assert straight.iter_time == pytest.approx((3e-3 + 3e-3) + 3 * 3e-3, rel=1e-14)
    assert crossed.iter_time == pytest.approx((1e-3 + 3e-3) + 3 * 3e-3, rel=1e-14)
    # the same four GPUs either way: two at each price
    assert straight.cost == pytest.approx((3.0 + 1.0) * 2 / 3600.0 * straight.iter_time, rel=1e-14)
    assert crossed.cost == pytest.approx((3.0 + 1.0) * 2 / 3600.0 * crossed.iter_time, rel=1e-14)


def test_uneven_splits_count_what_every_pool_gives():
    # D = 4 at TP 2: three replicas on pool 0 and one on pool 1 take 6 and 2 GPUs per stage
    p = make_problem(n_layers=2, n_types=2, n_zones=1, mb_list=(1,), tp_list=(2,), dp_list=(4,), pp_list=[2],
                     global_batch=8, layer_params=10_000_000, avail=np.array([[12, 4]]), node=np.array([2, 2], np.int32),
                     cap=np.array([8 << 30, 1 << 30], np.uint64), act=0)
    orc = Oracle(p)
    ok = orc.eval_replica_assignment(0, 0, 0, 0, 0, [[0, 0, 0, 1], [0, 0, 0, 1]])
    assert ok.mask == 0 and ok.peak_mem == 5_000_000 * 16
    assert orc.eval_replica_assignment(0, 0, 0, 0, 0, [[0, 0, 1, 1], [0, 0, 0, 1]]).mask == BIT_QUOTA  # pool 1: 6 of 4
    assert Oracle(p.with_avail(np.array([[11, 4]]))).eval_replica_assignment(
        0, 0, 0, 0, 0, [[0, 0, 0, 1], [0, 0, 0, 1]]).mask == BIT_QUOTA
    # one replica's type alone can break memory or the node size
    from dataclasses import replace
    small = replace(p, mem_capacity=np.array([8 << 30, 64 << 20], np.uint64))
    assert Oracle(small).eval_replica_assignment(0, 0, 0, 0, 0, [[0, 0, 0, 1], [0, 0, 1, 0]]).mask == BIT_OOM
    narrow = replace(p, gpus_per_node=np.array([2, 1], np.int32))
    assert Oracle(narrow).eval_replica_assignment(0, 0, 0, 0, 0, [[1, 0, 0, 0], [0, 0, 0, 1]]).mask == BIT_TP_NODE
    # a batch that D x mb does not divide
    odd = replace(p, global_batch=10)
    e = Oracle(odd).eval_replica_assignment(0, 0, 0, 0, 0, [[0, 0, 0, 1], [0, 0, 0, 1]])
    assert e.mask == BIT_BATCH and np.isinf(e.iter_time)


def test_pipelines_pay_for_their_own_crossings():
    # two stages, D = 2, two zones: pipeline 0 stays in zone 0, pipeline 1 goes from zone 0 to zone 1
    bw = np.array([[1e9, 1e8], [2e8, 1e9]])
    p = make_problem(n_layers=2, n_types=1, n_zones=2, mb_list=(1,), tp_list=(1,), dp_list=(2,), pp_list=[2],
                     global_batch=8, t_fwd=1e-3, t_bwd=2e-3, p2p=1_000_000, bw=bw, layer_params=0,
                     price=3600.0, avail=4, egress=np.array([[0.0, 1e-9], [3e-9, 0.0]]))
    e = Oracle(p).eval_replica_assignment(0, 0, 0, 0, 0, [[0, 0], [0, 1]])
    ms = 1e-3
    a = [3 * ms + 1 * ms, 3 * ms + 1 * ms]
    b = [3 * ms + 10 * ms, 3 * ms + 5 * ms]  # forward 0 -> 1 at 0.1 GB/s, backward 1 -> 0 at 0.2 GB/s
    T = max(sum(a) + 3 * max(a), sum(b) + 3 * max(b))
    assert e.mask == 0 and e.iter_time == pytest.approx(T, rel=1e-14)
    assert e.cost == pytest.approx(4 * T + 4 * 1e6 * 4e-9, rel=1e-14)  # no gradients: no ring traffic


# ------------------------------------------------------------------ a TP degree per stage as well

@pytest.mark.parametrize("seed", [4, 5, 6])
def test_with_a_degree_per_stage_agreeing_replicas_reduce_to_the_pinned_evaluators(seed):
    # all replicas of a stage on one pool: the evaluation with a pool and a TP degree per stage;
    # the halves on two pools: the one with two pools and a degree per stage; one degree for all
    # stages: the evaluation above -- each pinned on its own
    prob = W.tiny_problem(seed, n_types=2 + seed % 2, n_zones=2 + seed % 2, seg3_max_pp=64)
    orc = Oracle(prob)
    rng = np.random.default_rng(seed)
    zg = prob.n_zones * prob.n_types
    checked = mixed = 0
    for _ in range(1200):
        ip = int(rng.integers(0, len(prob.pp_values)))
        P = int(prob.pp_values[ip])
        q = int(rng.integers(0, prob.n_partitions[ip]))
        idp, im = int(rng.integers(0, len(prob.dp_values))), int(rng.integers(0, len(prob.mb_values)))
        D = int(prob.dp_values[idp])
        cuts = np.sort(rng.integers(0, P + 1, int(rng.integers(0, 3))))
        pa = rng.integers(0, zg, len(cuts) + 1)[np.searchsorted(cuts, np.arange(P), side="right")]
        pb = np.where(rng.random(P) < 0.5, pa, rng.integers(0, zg, P))
        tps = rng.integers(0, len(prob.tp_values), len(cuts) + 1)[np.searchsorted(cuts, np.arange(P), side="right")]
        any_pools = rng.integers(0, zg, (P, D))
        it = int(rng.integers(0, len(prob.tp_values)))
        for objective, bound in ((MAX_THROUGHPUT, None), (MIN_COST, 0.5)):
            one = np.repeat(pa[:, None], D, axis=1)
            _same(orc.eval_replica_assignment_tp(ip, q, idp, im, tps, one, objective, bound),
                  orc.eval_assignment_tp(ip, q, idp, im, tps, pa, objective, bound))
            a = orc.eval_replica_assignment(ip, q, idp, im, it, any_pools, objective, bound)
            b = orc.eval_replica_assignment_tp(ip, q, idp, im, np.full(P, it), any_pools, objective, bound)
            assert (a.mask, a.peak_mem) == (b.mask, b.peak_mem)
            assert (a.iter_time, a.cost) == (b.iter_time, b.cost) or np.isinf(a.iter_time)
            if D % 2 == 0:
                two = np.concatenate([np.repeat(pa[:, None], D // 2, axis=1), np.repeat(pb[:, None], D // 2, axis=1)], axis=1)
                want = orc.eval_split_assignment_tp(ip, q, idp, im, tps, pa, pb, objective, bound)
                tight = bound is not None and np.isfinite(want.iter_time) and abs(1.0 / want.iter_time / bound - 1) < 1e-9
                if not tight:
                    _same(orc.eval_replica_assignment_tp(ip, q, idp, im, tps, two, objective, bound), want)
                # (times and costs are compared whether or not the plan is valid)
                checked += np.isfinite(want.iter_time)
                mixed += np.isfinite(want.iter_time) and len(set(tps)) > 1
    assert checked > 200 and mixed > 50


def test_uneven_split_with_two_degrees_by_hand():
    # two stages, D = 4: stage 0 at TP 2 (three replicas on pool 0, one on pool 1), stage 1 at TP 1
    # (two and two).  GPUs: pool 0 gives 3 x 2 + 2 x 1 = 8, pool 1 gives 1 x 2 + 2 x 1 = 4.
    tf = np.zeros((2, 1, 2, 1)); tf[0, 0, :, 0] = (2e-3, 1e-3); tf[1, 0, :, 0] = (6e-3, 3e-3)
    p = make_problem(n_layers=2, n_types=2, n_zones=1, mb_list=(1,), tp_list=(1, 2), dp_list=(4,), pp_list=[2],
                     global_batch=8, t_fwd=tf, t_bwd=0.0, layer_params=10_000_000, p2p=0, act=0,
                     avail=np.array([[8, 4]]), node=np.array([2, 2], np.int32), price=np.array([3600.0, 1800.0]),
                     bw=1e9, grad_bytes=2)
    orc = Oracle(p)
    pools = [[0, 0, 0, 1], [0, 1, 0, 1]]
    e = orc.eval_replica_assignment_tp(0, 0, 0, 0, [1, 0], pools)
    assert e.mask == 0
    # memory: stage 0 holds half of its parameters (80 MB), stage 1 all of them (160 MB)
    assert e.peak_mem == 10_000_000 * 16
    # pipelines (2 microbatches each): r0 (1 + 2) ms, r1 (1 + 6), r2 (1 + 2), r3 (3 + 6); the last is the slowest
    t_pp = (3e-3 + 6e-3) + 1 * 6e-3
    # rings inside the one zone at 1 GB/s: stage 0 2 * 3/4 * 10 MB, stage 1 2 * 3/4 * 20 MB
    t_sync = 1.5 * 20e6 / 1e9
    assert e.iter_time == pytest.approx(t_pp + t_sync, rel=1e-14)
    # rent in $/s: stage 0 three replicas of 2 GPUs at 1 and one at 0.5, stage 1 two of 1 GPU at each price
    assert e.cost == pytest.approx((3 * 2 * 1.0 + 1 * 2 * 0.5 + 2 * 1.0 + 2 * 0.5) * e.iter_time, rel=1e-14)
    # one GPU fewer in either pool breaks the quota; with degree 1 for stage 0 it still fits
    for avail in ([[7, 4]], [[8, 3]]):
        short = Oracle(p.with_avail(np.array(avail)))
        assert short.eval_replica_assignment_tp(0, 0, 0, 0, [1, 0], pools).mask == BIT_QUOTA
        assert short.eval_replica_assignment_tp(0, 0, 0, 0, [0, 0], pools).mask == 0
    # the other way round (stage 1 at TP 2) pool 1 would have to give 1 + 2 x 2 = 5
    assert orc.eval_replica_assignment_tp(0, 0, 0, 0, [0, 1], pools).mask == BIT_QUOTA
