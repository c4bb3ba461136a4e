"""Pins of the oracle's candidate space (plan tuple of Sec. 4.2 as a flat index space).

The decoder is checked against an independent loop-nest enumerator, against a count
derived here from first principles, and by brute-force uniqueness of the plans.
"""
import numpy as np
import pytest

from oracle.oracle import Oracle
from paper_2504_17096_amd import workloads as W
from tests.helpers import make_problem


def expected_count(p):
    """Count plans directly: choose pp, a number of contiguous segments, the cut
    points, an ordered pool per segment with neighbours distinct, a partition and
    (dp, tp, mb)."""
    ZG = p.n_zones * p.n_types
    inner = len(p.mb_values) * len(p.tp_values) * len(p.dp_values)
    total = 0
    for ip, P in enumerate(p.pp_values):
        for s in (1, 2, 3):
            if s > p.max_segments or s > P or (s == 3 and P > p.seg3_max_pp):
                continue
            cuts = sum(1 for _ in _cut_sets(int(P), s))
            pools = ZG * (ZG - 1) ** (s - 1)
            total += inner * cuts * pools * int(p.n_partitions[ip])
    return total


def _cut_sets(P, s):
    import itertools
    return itertools.combinations(range(1, P), s - 1)


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_enumeration_matches_decode_and_count(seed):
    p = W.tiny_problem(seed, n_layers=4, partitions_per_pp=2)
    o = Oracle(p)
    n = o.num_candidates
    assert n == expected_count(p)
    assert o.enumerate_count() == n
    listed = o.enumerate()
    assert len(listed) == n
    seen = set()
    for c, cfg in enumerate(listed):
        assert o.decode(c) == cfg
        assert o.encode(cfg) == c
        # structure of a plan
        assert 1 <= cfg.n_segments <= 3
        cuts = cfg.cut[:cfg.n_segments - 1]
        assert all(0 < k < cfg.pp for k in cuts) and list(cuts) == sorted(set(cuts))
        pools = cfg.pool[:cfg.n_segments]
        assert all(0 <= a < p.n_zones * p.n_types for a in pools)
        assert all(pools[j] != pools[j + 1] for j in range(len(pools) - 1))
        key = (cfg.pp, cfg.n_segments, cfg.partition, cuts, pools, cfg.dp, cfg.tp, cfg.mb)
        assert key not in seen  # no plan listed twice
        seen.add(key)


def test_published_sizes_of_the_workloads():
    # sizes of the five synthetic workloads (8 640; 55 104; 6 791 040; 104 256 000)
    assert Oracle(W.config1()).num_candidates == 8640
    assert Oracle(W.config2()).num_candidates == 55104
    assert Oracle(W.config3(seg3_max_pp=0)).num_candidates == 1215360
    assert Oracle(W.config3()).num_candidates == 6791040
    p4 = W.config4()
    assert Oracle(p4).num_candidates == 104256000 == expected_count(p4)


def test_roundtrip_on_large_space():
    p = W.config4()
    o = Oracle(p)
    rng = np.random.default_rng(0)
    n = o.num_candidates
    for c in [0, n - 1] + rng.integers(0, n, 20000).tolist():
        cfg = o.decode(int(c))
        assert o.encode(cfg) == c
        row_ok = cfg.partition < p.n_partitions[cfg.pp_idx]
        assert row_ok and cfg.pp == p.pp_values[cfg.pp_idx]
    with pytest.raises(IndexError):
        o.decode(n)


def test_index_order_is_lexicographic_in_the_documented_digits():
    # mb is the fastest digit, then tp, dp, pool of segment 1; pp is the slowest
    p = make_problem(n_layers=4, n_types=2, n_zones=2, max_segments=2)
    o = Oracle(p)
    c0, c1 = o.decode(0), o.decode(1)
    assert (c0.mb_idx, c1.mb_idx) == (0, 1) and c0.tp_idx == c1.tp_idx == 0
    n_mb, n_tp, n_dp = len(p.mb_values), len(p.tp_values), len(p.dp_values)
    assert o.decode(n_mb).tp_idx == 1
    assert o.decode(n_mb * n_tp).dp_idx == 1
    assert o.decode(n_mb * n_tp * n_dp).pool[0] == 1
    pps = [o.decode(c).pp for c in range(o.num_candidates)]
    assert pps == sorted(pps)
