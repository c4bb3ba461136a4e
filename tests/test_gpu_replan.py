"""Re-planning after availability changes (Sec. 4.4; the reuse noted under H2, Sec. 4.2.1): a
plan that keeps per-piece minima and evaluates only the pieces whose quota rows changed must
return exactly what a plan that evaluates everything returns, and what the oracle returns."""
import numpy as np
import pytest

from oracle.oracle import MAX_THROUGHPUT, MIN_COST, Oracle
from paper_2504_17096_amd import workloads as W

pytestmark = pytest.mark.gpu


def _plan(prob, incremental=True):
    from paper_2504_17096_amd.binding import Plan
    p = Plan(prob)
    p.set_incremental(incremental)
    return p


def _same(a, b):
    if a is None or b is None:
        assert a is None and b is None
        return
    assert (a.index, a.peak_mem_bytes, a.mask, a.pool, a.dp, a.tp, a.mb) == \
           (b.index, b.peak_mem_bytes, b.mask, b.pool, b.dp, b.tp, b.mb)
    assert a.iter_time_s == b.iter_time_s and a.cost_per_iter == b.cost_per_iter


def _oracle_best(prob, snap, objective=MAX_THROUGHPUT, bound=None):
    return Oracle(prob.with_avail(snap)).best(objective=objective, bound=bound, n_threads=8)


def test_node_events_on_the_third_workload(torch_cuda):
    # one pool changes per snapshot: few pieces are evaluated again, results stay exact
    stream = torch_cuda.cuda.current_stream().cuda_stream
    prob = W.config3()
    inc, full = _plan(prob, True), _plan(prob, False)
    try:
        _same(inc.best_plan(stream=stream), full.best_plan(stream=stream))
        total = inc.last_scan()[1]
        assert inc.last_scan() == (total, total)  # nothing kept yet: everything evaluated
        _same(inc.best_plan(stream=stream), full.best_plan(stream=stream))
        assert inc.last_scan()[0] == 0            # same query, same availability: all kept
        # (without kept minima the best-plan pass also passes over pieces that cannot come near
        # the minimum seen so far)
        assert 0 < full.last_scan()[0] <= total and full.last_scan()[1] == total
        evaluated = []
        for i, snap in enumerate(W.node_events(prob)):
            inc.set_avail(snap)
            full.set_avail(snap)
            a, b = inc.best_plan(stream=stream), full.best_plan(stream=stream)
            _same(a, b)
            evaluated.append(inc.last_scan()[0])
            if i % 8 == 0:  # the oracle, on a sample of the snapshots (0.4 s each)
                want = _oracle_best(prob, snap)
                assert (a is None) == (want is None)
                if want is not None:
                    assert a.index == want.index
        # a pool that crosses a multiple of a power of two changes the validity of plans in most
        # pieces (every piece covers all pools of its first segment); other steps touch a few
        assert max(evaluated) < total and np.mean(evaluated) < 0.75 * total, (evaluated, total)
        assert sum(e < 0.1 * total for e in evaluated) >= 8, evaluated
        # the 64 best plans go through the same kept minima
        ta, tb = inc.topk(64, stream=stream), full.topk(64, stream=stream)
        assert inc.last_scan()[0] == 0
        assert len(ta) == len(tb)
        for x, y in zip(ta, tb):
            _same(x, y)
    finally:
        inc.destroy()
        full.destroy()


def test_a_different_query_evaluates_everything_again(torch_cuda):
    stream = torch_cuda.cuda.current_stream().cuda_stream
    prob = W.config2()
    inc, full = _plan(prob, True), _plan(prob, False)
    orc = Oracle(prob)
    try:
        total = None
        cheapest = orc.best(objective=MIN_COST)
        queries = [(MAX_THROUGHPUT, None), (MAX_THROUGHPUT, None), (MIN_COST, None),
                   (MAX_THROUGHPUT, 1.2 * cheapest.cost), (MAX_THROUGHPUT, 1.2 * cheapest.cost),
                   (MAX_THROUGHPUT, 1.3 * cheapest.cost), (MIN_COST, 2.0), (MIN_COST, 2.0)]
        kept_expected = [False, True, False, False, True, False, False, True]
        for (objective, bound), kept in zip(queries, kept_expected):
            a = inc.best_plan(objective=objective, bound=bound, stream=stream)
            _same(a, full.best_plan(objective=objective, bound=bound, stream=stream))
            want = orc.best(objective=objective, bound=bound)
            assert (a is None) == (want is None) and (a is None or a.index == want.index)
            n_eval, total = inc.last_scan()
            if kept:
                assert n_eval == 0, (objective, bound, n_eval, total)
            elif bound is None:
                assert n_eval == total, (objective, bound, n_eval, total)
            else:  # pieces that cannot meet the bound whatever the availability are passed over
                assert 0 < n_eval <= total, (objective, bound, n_eval, total)
    finally:
        inc.destroy()
        full.destroy()


def test_evaluation_calls_between_two_selections_do_not_hide_a_change(torch_cuda):
    # sailor_eval_batch also brings a new availability table to the device; the selection
    # after it must still see which rows changed
    stream = torch_cuda.cuda.current_stream().cuda_stream
    prob = W.config2()
    inc = _plan(prob, True)
    try:
        inc.best_plan(stream=stream)
        snap = prob.avail.copy()
        snap[0, 0] = 3
        snap[1, 1] = 0
        inc.set_avail(snap)
        n = inc.num_candidates()
        mask = torch_cuda.empty(n, dtype=torch_cuda.int32, device="cuda:0")
        inc.eval_batch(0, n, d_mask=mask, stream=stream)
        torch_cuda.cuda.synchronize()
        got = inc.best_plan(stream=stream)
        want = _oracle_best(prob, snap)
        assert got.index == want.index
        assert 0 < inc.last_scan()[0]
        for objective in (MAX_THROUGHPUT, MIN_COST):
            top = inc.topk(32, objective=objective, stream=stream)
            wt = Oracle(prob.with_avail(snap)).topk(32, objective=objective)
            assert [r.index for r in top] == [e.index for e in wt]
    finally:
        inc.destroy()


@pytest.mark.parametrize("seed", range(200, 212))
def test_random_availability_walks_on_small_problems(torch_cuda, seed):
    # every option flag, both objectives, with and without a bound; availability tables drawn
    # at random, the same table twice now and then
    stream = torch_cuda.cuda.current_stream().cuda_stream
    rng = np.random.default_rng(seed)
    prob = W.tiny_problem(seed, n_types=2 + seed % 2, n_zones=2 + seed % 3)
    if seed % 2:
        prob = prob.with_per_segment_tp()
    if seed % 3 == 0:
        prob = prob.with_mixed_types()
    inc, full = _plan(prob, True), _plan(prob, False)
    try:
        objective = MAX_THROUGHPUT if seed % 4 < 2 else MIN_COST
        ref = Oracle(prob).best(objective=MIN_COST if objective == MAX_THROUGHPUT else MAX_THROUGHPUT)
        bound = None
        if ref is not None and seed % 5 < 3:
            bound = 1.5 * ref.cost * (1 + 1e-7) if objective == MAX_THROUGHPUT else 0.5 / ref.iter_time * (1 + 1e-7)
        avail = prob.avail.copy()
        for step in range(12):
            if step % 4 != 3:  # (every fourth step repeats the table)
                change = rng.integers(0, 2, avail.shape).astype(bool)
                avail = np.where(change, rng.integers(0, 40, avail.shape), avail).astype(np.int32)
            inc.set_avail(avail)
            full.set_avail(avail)
            orc = Oracle(prob.with_avail(avail))
            if step % 2:
                ta = inc.topk(16, objective=objective, bound=bound, stream=stream)
                tb = full.topk(16, objective=objective, bound=bound, stream=stream)
                assert [r.index for r in ta] == [r.index for r in tb]
                assert [r.index for r in ta] == [e.index for e in orc.topk(16, objective, bound)]
            else:
                a = inc.best_plan(objective=objective, bound=bound, stream=stream)
                _same(a, full.best_plan(objective=objective, bound=bound, stream=stream))
                want = orc.best(objective=objective, bound=bound)
                assert (a is None) == (want is None) and (a is None or a.index == want.index)
    finally:
        inc.destroy()
        full.destroy()
