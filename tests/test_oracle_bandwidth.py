"""Pins of the oracle's message-size dependent bandwidth (Sec. 4.1: a polynomial fitted per
link over the message size; Sec. 4.3: used for peer-to-peer transfers and collectives).

Expected values come from numpy's polynomial evaluation and hand-written formulas, never
from the oracle.
"""
import math

import numpy as np
import pytest

from oracle.oracle import MAX_THROUGHPUT, Oracle
from paper_2504_17096_amd import workloads as W
from tests.helpers import find_index, make_problem


def bw_of(poly, peak, nbytes):
    """Bandwidth of one link for one message size, from numpy's polyval."""
    v = np.polynomial.polynomial.polyval(math.log2(nbytes), poly)
    return float(min(max(v, peak * 1e-3), peak))


def test_a_constant_polynomial_is_the_constant_model():
    base = W.tiny_problem(3)
    Z = base.n_zones
    poly = np.zeros((Z, Z, 3))
    poly[:, :, 0] = base.bandwidth
    a, b = Oracle(base).eval_batch(), Oracle(base.with_bw_poly(poly)).eval_batch()
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
    # ... and so is any polynomial that stays above the peak (upper limit)
    poly[:, :, 0] *= 3.0
    poly[:, :, 1] = 1.0
    c = Oracle(base.with_bw_poly(poly)).eval_batch()
    for x, y in zip(a, c):
        assert np.array_equal(x, y)


def test_two_stage_cross_zone_transfer_with_a_size_dependent_link():
    # stage 0 in zone 0, stage 1 in zone 1, one microbatch, no all-reduce (D = 1)
    tf, tb, L = 1e-3, 2e-3, 4
    bw = np.array([[1e10, 2e9], [1e9, 1e10]])
    poly = np.zeros((2, 2, 3))
    poly[0, 1] = [-3.0e9, 2.5e8, -2.0e6]   # 0 -> 1
    poly[1, 0] = [1.0e8, 1.0e7, 1.0e6]     # 1 -> 0
    poly[0, 0] = poly[1, 1] = [1e12, 0, 0]  # intra-zone: always the peak
    for p2p in (1 << 12, 3_000_000, 1 << 26):
        p = make_problem(n_layers=L, n_zones=2, mb_list=(1,), tp_list=(1,), dp_list=(1,), pp_list=[2],
                         global_batch=1, max_segments=2, t_fwd=tf, t_bwd=tb, p2p=p2p, bw=bw,
                         layer_params=0).with_bw_poly(poly)
        o = Oracle(p)
        c = find_index(o, n_segments=2, pool=(0, 1, -1))
        fwd = p2p / bw_of(poly[0, 1], 2e9, p2p)  # activations 0 -> 1
        back = p2p / bw_of(poly[1, 0], 1e9, p2p)  # gradients 1 -> 0
        stage = (L // 2) * (tf + tb)
        assert o.eval_one(c).iter_time == pytest.approx(2 * stage + fwd + back, rel=1e-12)
        # the mirrored placement uses the other direction for each transfer
        c2 = find_index(o, n_segments=2, pool=(1, 0, -1))
        fwd2 = p2p / bw_of(poly[1, 0], 1e9, p2p)
        back2 = p2p / bw_of(poly[0, 1], 2e9, p2p)
        assert o.eval_one(c2).iter_time == pytest.approx(2 * stage + fwd2 + back2, rel=1e-12)
    assert bw_of(poly[0, 1], 2e9, 1 << 12) != bw_of(poly[0, 1], 2e9, 1 << 26)  # the sizes matter


def test_both_limits_of_the_fitted_curve():
    poly = np.zeros((1, 1, 2))
    poly[0, 0] = [-1e9, 1e8]  # negative below 1 KiB, above the 2e9 peak beyond 2^30
    tf = 1e-3

    def t_iter(p2p):
        p = make_problem(n_layers=2, mb_list=(1,), tp_list=(1,), dp_list=(1,), pp_list=[2],
                         global_batch=1, t_fwd=tf, t_bwd=0.0, p2p=p2p, bw=2e9,
                         layer_params=0).with_bw_poly(poly)
        o = Oracle(p)
        return o.eval_one(find_index(o, pp=2)).iter_time

    assert t_iter(512) == pytest.approx(2 * tf + 2 * 512 / 2e6, rel=1e-12)              # floor: peak / 1000
    assert t_iter(1 << 31) == pytest.approx(2 * tf + 2 * (1 << 31) / 2e9, rel=1e-12)    # peak
    mid = 1 << 20
    assert t_iter(mid) == pytest.approx(2 * tf + 2 * mid / (-1e9 + 1e8 * 20), rel=1e-12)
    assert t_iter(0) == pytest.approx(2 * tf, rel=1e-12)                                # nothing to send


@pytest.mark.parametrize("tp", [1, 2])
def test_all_reduce_uses_the_gradient_buffer_as_message_size(tp):
    params, gb, L = 1_000_003, 2, 4
    poly = np.zeros((1, 1, 3))
    poly[0, 0] = [2.0e8, -1.0e7, 1.5e6]
    p = make_problem(n_layers=L, mb_list=(1,), tp_list=(1, 2), dp_list=(1, 2, 4), pp_list=[1, 2],
                     global_batch=8, t_fwd=1e-3, t_bwd=1e-3, layer_params=params, grad_bytes=gb,
                     bw=5e9).with_bw_poly(poly)
    o = Oracle(p)
    for pp in (1, 2):
        for dp in (1, 2, 4):
            e = o.eval_one(find_index(o, pp=pp, dp=dp, tp=tp, mb=1))
            nb = 8 // dp
            t_pp = (nb + pp - 1) * (L // pp) * 2e-3
            buf = -(-(params * (L // pp)) // tp) * gb
            ring = 0.0 if dp == 1 else 2 * (dp - 1) / dp * buf / bw_of(poly[0, 0], 5e9, buf)
            assert e.iter_time == pytest.approx(t_pp + ring, rel=1e-12)


def test_t_sync_is_the_slowest_stage_not_the_largest_buffer():
    # a link that collapses for large messages... then recovers: the stage with the smaller
    # buffer can be the slower one
    layer = np.array([4_000_000, 1_000_000], np.uint64)
    poly = np.zeros((1, 1, 3))
    # bandwidth over x = log2(bytes): a parabola with its minimum near 2 MB messages
    x0 = math.log2(2_000_000)
    poly[0, 0] = [1e8 + 1e9 * x0 * x0, -2e9 * x0, 1e9]
    p = make_problem(n_layers=2, mb_list=(1,), tp_list=(1,), dp_list=(2,), pp_list=[2], global_batch=2,
                     t_fwd=1e-3, t_bwd=0.0, layer_params=layer, grad_bytes=2, bw=1e10,
                     uniform_layers=True).with_bw_poly(poly)
    o = Oracle(p)
    e = o.eval_one(find_index(o, pp=2))
    t = [2 * (2 - 1) / 2 * (n * 2) / bw_of(poly[0, 0], 1e10, n * 2) for n in (4_000_000, 1_000_000)]
    assert t[1] > t[0]  # the smaller buffer is slower on this link
    assert e.iter_time == pytest.approx(2 * 1e-3 + max(t), rel=1e-12)


def test_seeded_profile_slows_small_messages_and_keeps_large_ones():
    base = W.config2()
    prof = base.with_bw_poly(W.bandwidth_poly(base))
    a, b = Oracle(base).eval_batch(), Oracle(prof).eval_batch()
    fin = np.isfinite(a[0])
    assert np.array_equal(a[2], b[2]) and np.array_equal(a[3], b[3])  # memory and validity: unchanged
    assert np.all(b[0][fin] >= a[0][fin] * (1 - 1e-12))               # never faster than the peak
    assert np.max(b[0][fin] / a[0][fin]) > 1.05                        # and visibly slower somewhere
    best_a, best_b = Oracle(base).best(MAX_THROUGHPUT), Oracle(prof).best(MAX_THROUGHPUT)
    assert best_b.iter_time >= best_a.iter_time * (1 - 1e-12)
