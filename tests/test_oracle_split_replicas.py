"""Pins of the oracle's evaluation of plans whose stages split their replicas over two pools,
also of different zones (the D tuples of a stage, Sec. 4.2; max over pipelines and the
all-reduce over the slowest link, Sec. 4.3)."""
import numpy as np
import pytest

from oracle.oracle import BIT_OOM, BIT_QUOTA, BIT_TP_NODE, MAX_THROUGHPUT, MIN_COST, Oracle
from paper_2504_17096_amd import workloads as W
from tests.helpers import GIB, make_problem


def _tiny(seed, **kw):
    kw.setdefault("seg3_max_pp", 64)
    return W.tiny_problem(seed, **kw)


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_unsplit_stages_reduce_to_the_plain_evaluation(seed):
    prob = _tiny(seed, n_types=2, n_zones=2 + seed % 2)
    orc = Oracle(prob)
    rng = np.random.default_rng(seed)
    zg = prob.n_zones * prob.n_types
    for _ in range(600):
        ip = int(rng.integers(0, len(prob.pp_values)))
        P = int(prob.pp_values[ip])
        args = (ip, int(rng.integers(0, prob.n_partitions[ip])), int(rng.integers(0, len(prob.dp_values))),
                int(rng.integers(0, len(prob.mb_values))), int(rng.integers(0, len(prob.tp_values))))
        pools = rng.integers(0, zg, P)
        for objective, bound in ((MAX_THROUGHPUT, None), (MIN_COST, 3.0)):
            a = orc.eval_assignment(*args, pools, objective, bound)
            b = orc.eval_split_assignment(*args, pools, pools, objective, bound)
            assert (a.mask, a.peak_mem) == (b.mask, b.peak_mem)
            if np.isfinite(a.iter_time):
                assert b.iter_time == pytest.approx(a.iter_time, rel=1e-13)
                assert b.cost == pytest.approx(a.cost, rel=1e-13)


def _two_zone(**kw):
    # 2 stages of 1 layer, one GPU type, D = 2 replicas, 4 microbatches per pipeline:
    # fwd 1 ms + bwd 2 ms per layer; links: zone 0 fast (1 GB/s), zone 1 slow inside (0.5 GB/s),
    # 0.1 GB/s from 0 to 1 and 0.2 GB/s back; 1 MB activations; 1e6 parameters x 2 B gradients
    bw = np.array([[1e9, 1e8], [2e8, 5e8]])
    args = dict(n_layers=2, n_types=1, n_zones=2, mb_list=(1,), tp_list=(1,), dp_list=(2,), pp_list=[2],
                global_batch=8, t_fwd=1e-3, t_bwd=2e-3, t_upd=5e-4, p2p=1_000_000, bw=bw,
                layer_params=1_000_000, price=3600.0, avail=4,
                egress=np.array([[0.0, 1e-9], [3e-9, 0.0]]))
    args.update(kw)
    return make_problem(**args)


def test_two_zones_by_hand():
    orc = Oracle(_two_zone())
    # stage 0 split over zones (0, 1), stage 1 in zone 0 for both halves
    e = orc.eval_split_assignment(0, 0, 0, 0, 0, [0, 0], [1, 0])
    assert e.mask == 0
    ms = 1e-3
    # pipelines through the first pools: zone 0 -> zone 0
    a = [3 * ms + 1 * ms, 3 * ms + 1 * ms]
    # through the second pools: zone 1 -> zone 0: forward over 1->0 (0.2 GB/s: 5 ms), backward
    # over 0->1 (0.1 GB/s: 10 ms)
    b = [3 * ms + 5 * ms, 3 * ms + 10 * ms]
    t_pp = max(sum(a) + 3 * max(a), sum(b) + 3 * max(b))
    # ring of stage 0 through both zones: slowest link 0.1 GB/s, 2 (D-1)/D x 2 MB = 2 MB
    t_sync = max(2e6 / 1e8, 2e6 / 1e9)
    T = t_pp + t_sync + 5e-4
    assert e.iter_time == pytest.approx(T, rel=1e-13)
    # rent: 2 stages x 2 replicas at 1 $/s; traffic: the second kind of pipeline (1 replica)
    # crosses once, 4 microbatches x 1 MB both ways at 4e-9 $/B, and stage 0's ring 2 MB x 4e-9
    assert e.cost == pytest.approx(4 * T + 4 * 1e6 * 4e-9 + 2e6 * 4e-9, rel=1e-13)
    # without the split: no slow link anywhere
    plain = orc.eval_split_assignment(0, 0, 0, 0, 0, [0, 0], [0, 0])
    assert plain.iter_time == pytest.approx(2 * 4 * ms + 3 * 4 * ms + 2e6 / 1e9 + 5e-4, rel=1e-13)
    assert plain.cost == pytest.approx(4 * plain.iter_time, rel=1e-13)
    # the all-reduce takes the slowest of the four links, whichever it is
    for slow in ((0, 0), (1, 1), (0, 1), (1, 0)):
        bw = np.full((2, 2), 1e9)
        bw[slow] = 1e7
        e2 = Oracle(_two_zone(bw=bw, p2p=0)).eval_split_assignment(0, 0, 0, 0, 0, [0, 0], [1, 0])
        assert e2.iter_time == pytest.approx(2 * 3 * ms + 3 * 3 * ms + 2e6 / 1e7 + 5e-4, rel=1e-13)


def test_identical_zones_make_the_split_invisible():
    # two zones with the same links everywhere and free traffic: where a stage's halves sit
    # does not matter
    orc = Oracle(_two_zone(bw=np.full((2, 2), 1e9), egress=None))
    base = orc.eval_split_assignment(0, 0, 0, 0, 0, [0, 0], [0, 0])
    for a, b in (([0, 0], [1, 1]), ([0, 1], [1, 0]), ([1, 0], [0, 0])):
        e = orc.eval_split_assignment(0, 0, 0, 0, 0, a, b)
        assert e.mask == 0 and e.iter_time == base.iter_time and e.cost == base.cost


def test_two_types_in_one_zone_the_slower_pipeline_counts():
    # type 1 is slower in stage 0, type 0 in stage 1 (non-uniform layers): per pipeline the sums
    # differ from the per-stage maxima that the flat space's pairs of types use
    tf = np.zeros((2, 1, 1, 2)); tf[0, 0, 0] = [1e-3, 4e-3]; tf[1, 0, 0] = [3e-3, 1e-3]
    p = make_problem(n_layers=2, n_types=2, n_zones=1, mb_list=(1,), tp_list=(1,), dp_list=(2,), pp_list=[2],
                     global_batch=4, t_fwd=tf, t_bwd=0.0, uniform_layers=False, layer_params=0, p2p=0)
    orc = Oracle(p)
    e = orc.eval_split_assignment(0, 0, 0, 0, 0, [0, 0], [1, 1])
    pipe_a, pipe_b = [1e-3, 4e-3], [3e-3, 1e-3]
    want = max(sum(pipe_a) + 1 * max(pipe_a), sum(pipe_b) + 1 * max(pipe_b))
    assert e.iter_time == pytest.approx(want, rel=1e-13)
    flat = Oracle(p.with_mixed_types())
    # the flat space's pair (type 0, type 1) on both stages: every stage at its slower type
    cands = [c for c in range(flat.num_candidates)
             if flat.decode(c).pool[0] == 2 and flat.decode(c).n_segments == 1 and flat.decode(c).pp == 2]
    stage_max = flat.eval_one(cands[0]).iter_time
    assert stage_max == pytest.approx((3e-3 + 4e-3) + 4e-3, rel=1e-13) and e.iter_time < stage_max
    # crossed halves: stage 0 on (0, 1), stage 1 on (1, 0): each pipeline gets both slow stages or none
    x = orc.eval_split_assignment(0, 0, 0, 0, 0, [0, 1], [1, 0])
    assert x.iter_time == pytest.approx(max(1e-3 + 1e-3 + 1e-3, 3e-3 + 4e-3 + 4e-3), rel=1e-13)


def test_quota_memory_and_node_size_of_both_halves():
    p = _two_zone(avail=np.array([[3], [1]]), dp_list=(1, 2, 4), global_batch=8)
    orc = Oracle(p)
    # D = 2: stage 0 split (one replica per zone), stage 1 in zone 0: zone 0 holds 1 + 2, zone 1 one
    assert orc.eval_split_assignment(0, 0, 1, 0, 0, [0, 0], [1, 0]).mask == 0
    # both stages split: zone 1 would hold two
    assert orc.eval_split_assignment(0, 0, 1, 0, 0, [0, 0], [1, 1]).mask == BIT_QUOTA
    # D = 4: zone 0 would hold 2 + 4
    assert orc.eval_split_assignment(0, 0, 2, 0, 0, [0, 0], [1, 0]).mask == BIT_QUOTA
    # D = 1 cannot be halved
    assert orc.eval_split_assignment(0, 0, 0, 0, 0, [0, 0], [1, 0]).mask & BIT_QUOTA
    assert orc.eval_split_assignment(0, 0, 0, 0, 0, [0, 0], [0, 0]).mask == 0
    # two types: the smaller memory and the smaller node of the two halves decide
    q = make_problem(n_layers=2, n_types=2, n_zones=1, mb_list=(1,), tp_list=(1, 4), dp_list=(2,), pp_list=[1],
                     global_batch=4, layer_params=100_000_000, cap=np.array([8 * GIB, 2 * GIB], np.uint64),
                     node=np.array([8, 2], np.int32), act=0)
    oq = Oracle(q)
    assert oq.eval_split_assignment(0, 0, 0, 0, 0, [0], [0]).mask == 0
    e = oq.eval_split_assignment(0, 0, 0, 0, 0, [0], [1])
    assert e.mask == BIT_OOM and e.peak_mem == 200_000_000 * 16
    assert oq.eval_split_assignment(0, 0, 0, 0, 1, [0], [1]).mask == BIT_TP_NODE


def test_a_stage_on_two_types_pays_both_prices_and_waits_for_the_slower_update():
    # one stage, D = 2, one replica on each of two types of one zone: type 1 is twice as slow in
    # compute and in its optimizer step and costs a third; 2 microbatches per pipeline
    tf = np.zeros((2, 1, 1, 1)); tf[:, 0, 0, 0] = (1e-3, 2e-3)
    tu = np.zeros((2, 1, 1)); tu[:, 0, 0] = (3e-4, 6e-4)
    p = make_problem(n_layers=1, n_types=2, n_zones=1, mb_list=(1,), tp_list=(1,), dp_list=(2,), pp_list=[1],
                     global_batch=4, t_fwd=tf, t_bwd=0.0, t_upd=tu, layer_params=0, p2p=0,
                     price=np.array([3600.0, 1200.0]))
    orc = Oracle(p)
    for a, b in (([0], [1]), ([1], [0])):
        e = orc.eval_split_assignment(0, 0, 0, 0, 0, a, b)
        T = 2 * 2e-3 + 6e-4                  # the slower kind of pipeline, then the slower update
        assert e.mask == 0 and e.iter_time == pytest.approx(T, rel=1e-13)
        assert e.cost == pytest.approx((1.0 + 1.0 / 3.0) * T, rel=1e-13)   # one GPU at each price
    fast = orc.eval_split_assignment(0, 0, 0, 0, 0, [0], [0])
    assert fast.iter_time == pytest.approx(2 * 1e-3 + 3e-4, rel=1e-13)
    assert fast.cost == pytest.approx(2.0 * fast.iter_time, rel=1e-13)


# ------------------------------------------------------------------ two pools and a TP degree per stage

@pytest.mark.parametrize("seed", [4, 5, 6])
def test_with_a_degree_per_stage_the_two_special_cases_come_back(seed):
    # equal halves: the evaluation with a TP degree per stage; one degree for all stages: the
    # split evaluation above -- both pinned on their own
    prob = _tiny(seed, n_types=2, n_zones=2 + seed % 2)
    orc = Oracle(prob)
    rng = np.random.default_rng(seed)
    zg = prob.n_zones * prob.n_types
    for _ in range(600):
        ip = int(rng.integers(0, len(prob.pp_values)))
        P = int(prob.pp_values[ip])
        args = (ip, int(rng.integers(0, prob.n_partitions[ip])), int(rng.integers(0, len(prob.dp_values))),
                int(rng.integers(0, len(prob.mb_values))))
        pools, other = rng.integers(0, zg, P), rng.integers(0, zg, P)
        tps = rng.integers(0, len(prob.tp_values), P)
        one = int(rng.integers(0, len(prob.tp_values)))
        for objective, bound in ((MAX_THROUGHPUT, None), (MIN_COST, 3.0)):
            a = orc.eval_assignment_tp(*args, tps, pools, objective, bound)
            b = orc.eval_split_assignment_tp(*args, tps, pools, pools, objective, bound)
            assert (a.mask, a.peak_mem) == (b.mask, b.peak_mem)
            if np.isfinite(a.iter_time):
                assert b.iter_time == pytest.approx(a.iter_time, rel=1e-13)
                assert b.cost == pytest.approx(a.cost, rel=1e-13)
            c = orc.eval_split_assignment(*args, one, pools, other, objective, bound)
            d = orc.eval_split_assignment_tp(*args, np.full(P, one), pools, other, objective, bound)
            assert (c.mask, c.peak_mem, c.iter_time, c.cost) == (d.mask, d.peak_mem, d.iter_time, d.cost) or \
                (np.isnan(c.cost) and np.isnan(d.cost))


def test_two_zones_and_two_degrees_by_hand():
    # the two-zone problem above with TP degrees 1 and 2: at degree 2 a layer takes half the
    # time and a worker holds half of the parameters.  Stage 0 (degree 2) split over the zones,
    # stage 1 (degree 1) in zone 0.
    tf = np.zeros((1, 1, 2, 1)); tf[0, 0, :, 0] = (1e-3, 0.5e-3)
    tb = 2 * tf
    tu = np.zeros((1, 2, 1)); tu[0, :, 0] = (5e-4, 2.5e-4)
    # GPUs: zone 0 gives one replica of stage 0 (2) and both of stage 1 (1 + 1), zone 1 the other
    # replica of stage 0 (2)
    orc = Oracle(_two_zone(tp_list=(1, 2), t_fwd=tf, t_bwd=tb, t_upd=tu, avail=np.array([[4], [2]])))
    e = orc.eval_split_assignment_tp(0, 0, 0, 0, [1, 0], [0, 0], [1, 0])
    assert e.mask == 0
    ms = 1e-3
    a = [1.5 * ms + 1 * ms, 3 * ms + 1 * ms]             # both stages in zone 0
    b = [1.5 * ms + 5 * ms, 3 * ms + 10 * ms]            # zone 1 -> zone 0 (5 ms forward, 10 ms back)
    t_pp = max(sum(a) + 3 * max(a), sum(b) + 3 * max(b))
    # stage 0's ring carries half of the parameters (1 MB of gradients) over the slowest link, stage 1's 2 MB in zone 0
    t_sync = max(1e6 / 1e8, 2e6 / 1e9)
    T = t_pp + t_sync + 5e-4                              # stage 1's update at degree 1 is the slower one
    assert e.iter_time == pytest.approx(T, rel=1e-13)
    # rent: stage 0 two replicas of 2 GPUs, stage 1 two of 1, at 1 $/s; traffic as before, the ring half as much
    assert e.cost == pytest.approx(6 * T + 4 * 1e6 * 4e-9 + 1e6 * 4e-9, rel=1e-13)
    # memory: stage 0 holds half of its parameters and two microbatches in flight (10 MB), stage 1
    # all of its parameters and one microbatch (17 MB)
    assert e.peak_mem == 1_000_000 * 16 + 1_000_000
    # one GPU fewer in either zone: stage 0's wider replicas no longer fit
    for avail in ([[3], [2]], [[4], [1]]):
        short = Oracle(_two_zone(tp_list=(1, 2), t_fwd=tf, t_bwd=tb, t_upd=tu, avail=np.array(avail)))
        assert short.eval_split_assignment_tp(0, 0, 0, 0, [1, 0], [0, 0], [1, 0]).mask == BIT_QUOTA
        # ... while degree 1 everywhere still does (zone 0: 1 + 2, zone 1: 1)
        assert short.eval_split_assignment_tp(0, 0, 0, 0, [0, 0], [0, 0], [1, 0]).mask == 0
    # a node of one GPU cannot host degree 2, whichever half sits on it
    small = Oracle(_two_zone(tp_list=(1, 2), t_fwd=tf, t_bwd=tb, t_upd=tu, node=1))
    assert small.eval_split_assignment_tp(0, 0, 0, 0, [1, 0], [0, 0], [1, 0]).mask & BIT_TP_NODE
    assert small.eval_split_assignment_tp(0, 0, 0, 0, [0, 0], [0, 0], [1, 0]).mask & BIT_TP_NODE == 0
