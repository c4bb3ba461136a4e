"""Pins of the oracle's discrete-event 1F1B schedule (warm-up, steady and cool-down phases of
Sec. 4.3, op by op) and of the closed form it is reported beside (Sec. 4.2.2).

The reference here is the event simulator written in Python for the simulator pins
(tests/test_oracle_simulator.py), textbook makespans and hand-computed schedules.
"""
import math

import numpy as np
import pytest

from oracle.oracle import Oracle
from paper_2504_17096_amd import workloads as W
from tests.helpers import find_index, make_problem
from tests.test_oracle_simulator import one_f_one_b_makespan


def stage_durations(p, g):
    """(forward + send, backward + send) per stage of plan g from the raw tables."""
    row0 = sum(int(p.n_partitions[i]) * int(p.pp_values[i]) for i in range(g.pp_idx))
    nl = [int(x) for x in p.partition_layers[row0 + g.partition * g.pp: row0 + (g.partition + 1) * g.pp]]
    Lc = 1 if p.uniform_layers else p.n_layers
    fd, bd, first = [], [], 0
    zone = []
    for i in range(g.pp):
        seg = 0 if i < g.cut[0] else 1 if i < g.cut[1] else 2
        zone.append(g.pool[seg] // p.n_types)
    for i in range(g.pp):
        seg = 0 if i < g.cut[0] else 1 if i < g.cut[1] else 2
        gt, ti = g.pool[seg] % p.n_types, g.seg_tp_idx[seg]
        if p.uniform_layers:
            f = nl[i] * p.t_fwd[gt, g.mb_idx, ti, 0]
            b = nl[i] * p.t_bwd[gt, g.mb_idx, ti, 0]
        else:
            f = float(np.sum(p.t_fwd[gt, g.mb_idx, ti, first:first + nl[i]]))
            b = float(np.sum(p.t_bwd[gt, g.mb_idx, ti, first:first + nl[i]]))
        x = float(p.p2p_bytes[g.mb_idx])
        sf = x / p.bandwidth[zone[i], zone[i + 1]] if i < g.pp - 1 else 0.0
        sb = x / p.bandwidth[zone[i], zone[i - 1]] if i > 0 else 0.0
        fd.append(f + sf)
        bd.append(b + sb)
        first += nl[i]
    return fd, bd


@pytest.mark.parametrize("seed", [1, 2, 5])
def test_against_the_python_event_simulator(seed):
    p = W.tiny_problem(seed)
    o = Oracle(p)
    rng = np.random.default_rng(seed)
    checked = 0
    for c in rng.integers(0, o.num_candidates, 400):
        c = int(c)
        g = o.decode(c)
        ev, closed = o.simulate_1f1b(c)
        if int(p.global_batch) % (g.dp * g.mb):
            assert math.isinf(ev) and math.isinf(closed)
            continue
        nb = int(p.global_batch) // (g.dp * g.mb)
        fd, bd = stage_durations(p, g)
        assert ev == pytest.approx(one_f_one_b_makespan(fd, bd, nb), rel=1e-12)
        t = [f + b for f, b in zip(fd, bd)]
        assert closed == pytest.approx(sum(t) + (nb - 1) * max(t), rel=1e-12)
        checked += 1
    assert checked > 150


@pytest.mark.parametrize("pp,dp,mb", [(1, 1, 1), (2, 2, 4), (4, 1, 2), (8, 4, 1), (8, 1, 1)])
def test_homogeneous_pipeline_has_the_textbook_makespan(pp, dp, mb):
    L, B, tf, tb = 8, 32, 1.3e-3, 2.9e-3
    p = make_problem(n_layers=L, global_batch=B, t_fwd=tf, t_bwd=tb, layer_params=0, tp_list=(1,))
    o = Oracle(p)
    ev, closed = o.simulate_1f1b(find_index(o, pp=pp, dp=dp, mb=mb))
    nb = B // (dp * mb)
    want = (nb + pp - 1) * (L // pp) * (tf + tb)
    assert ev == pytest.approx(want, rel=1e-12) and closed == pytest.approx(want, rel=1e-12)


def test_two_stages_two_microbatches_with_transfers_by_hand():
    # stage 0 (zone 0): f = 2, b = 4 ; stage 1 (zone 1): f = 1, b = 3 ; sends 0->1: 0.5, 1->0: 0.25
    tf = np.zeros((1, 1, 1, 2)); tb = np.zeros((1, 1, 1, 2))
    tf[0, 0, 0] = [2.0, 1.0]; tb[0, 0, 0] = [4.0, 3.0]
    bw = np.array([[1e30, 2.0], [4.0, 1e30]])
    p = make_problem(n_layers=2, n_zones=2, mb_list=(1,), tp_list=(1,), dp_list=(1,), pp_list=[2],
                     global_batch=2, max_segments=2, t_fwd=tf, t_bwd=tb, uniform_layers=False,
                     p2p=1, bw=bw, layer_params=0)
    o = Oracle(p)
    ev, closed = o.simulate_1f1b(find_index(o, n_segments=2, pool=(0, 1, -1)))
    # stage 0: F0 [0, 2.5]  F1 [2.5, 5]            B0 [6.75, 10.75]  B1 [11, 15] (waits for stage 1)
    # stage 1:      F0 [2.5, 3.5]  B0 [3.5, 6.75]  F1 [6.75, 7.75]   B1 [7.75, 11]
    assert ev == pytest.approx(15.0, rel=1e-12)
    assert closed == pytest.approx((6.5 + 4.25) + 1 * 6.5, rel=1e-12)


def test_bounds_and_limits_on_a_workload():
    p = W.config2()
    o = Oracle(p)
    rng = np.random.default_rng(0)
    seen, worst = 0, 0.0
    for c in rng.integers(0, o.num_candidates, 600):
        c = int(c)
        g = o.decode(c)
        ev, closed = o.simulate_1f1b(c)
        if math.isinf(ev):
            continue
        fd, bd = stage_durations(p, g)
        t = [f + b for f, b in zip(fd, bd)]
        nb = int(p.global_batch) // (g.dp * g.mb)
        # one microbatch passes every stage; the slowest stage runs every microbatch; nothing
        # is slower than running the microbatches one after the other
        assert max(sum(t), nb * max(t)) * (1 - 1e-12) <= ev <= nb * sum(t) * (1 + 1e-12)
        # the closed form is an estimate of the schedule (it may fall on either side when
        # forward and backward durations of neighbouring stages differ a lot)
        assert 0.5 < closed / ev < 1.5
        worst = max(worst, abs(closed / ev - 1.0))
        if g.pp == 1 or nb == 1:
            assert ev == pytest.approx(closed, rel=1e-12)  # one stage / one microbatch: no slack
        e = o.eval_one(c)                                  # the evaluator's T_pp is the closed form
        assert closed <= e.iter_time * (1 + 1e-12)
        seen += 1
    assert seen > 300 and worst > 1e-3  # and the two do differ on heterogeneous plans


def test_the_straggler_counts_n_b_times_not_n_b_plus_one():
    # Sec. 4.2.2 and 4.2.3 print sum_i t_i + N_b t_straggler; the evaluator uses
    # sum_i t_i + (N_b - 1) t_straggler.  Against the op-by-op schedule of the same stage times
    # the second is exact for uniform pipelines and closer for uneven ones, most visibly with
    # few microbatches, where one extra straggler period is a large share of the makespan.
    rng = np.random.default_rng(7)
    err_used, err_printed = [], []
    for trial in range(60):
        P = int(rng.integers(1, 7))
        nb = int(rng.integers(1, 5))
        uniform = trial % 3 == 0
        f = np.full(P, 1e-3) if uniform else rng.uniform(0.5e-3, 3e-3, P)
        b = 2 * f if uniform else rng.uniform(1e-3, 6e-3, P)
        event = one_f_one_b_makespan(list(f), list(b), nb)
        t = f + b
        used = t.sum() + (nb - 1) * t.max()
        printed = t.sum() + nb * t.max()
        if uniform:
            assert used == pytest.approx(event, rel=1e-12)
        assert printed > used
        err_used.append(abs(used - event) / event)
        err_printed.append(abs(printed - event) / event)
    assert np.mean(err_used) < 0.25 * np.mean(err_printed)
    assert np.max(err_used) < np.max(err_printed)
    # the oracle's own closed form is the first one (two stages, one microbatch: the sum)
    p = make_problem(n_layers=2, pp_list=[2], mb_list=(4,), tp_list=(1,), dp_list=(1,), global_batch=4,
                     t_fwd=1e-3, t_bwd=2e-3, layer_params=0)
    o = Oracle(p)
    ev, closed = o.simulate_1f1b(0)
    assert closed == pytest.approx(2 * 3e-3, rel=1e-12) and ev == pytest.approx(closed, rel=1e-12)
