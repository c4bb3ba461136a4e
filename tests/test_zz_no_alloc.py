"""sailor_simulate_1f1b_static (the entry point that allocates nothing) against
sailor_simulate_1f1b, through the C ABI: both run the same kernel on the same stage times, so
the bar is bit-for-bit equality -- on two calls in a row, the second with a smaller input, since
every call on a GPU shares one static array that keeps the previous call's contents."""
import numpy as np
import pytest

from paper_2504_17096_amd import binding
from paper_2504_17096_amd import workloads as W
from tests.helpers import make_problem

pytestmark = pytest.mark.gpu


def _both(torch, plan, idx):
    """(event, closed) of the allocating entry point and of the static one."""
    stream = torch.cuda.current_stream().cuda_stream
    d_idx = torch.from_numpy(np.asarray(idx, dtype=np.uint64).view(np.int64)).to("cuda:0")
    out = []
    for call in (plan.simulate_1f1b, plan.simulate_1f1b_static):
        ev = torch.full((len(idx),), -1.0, dtype=torch.float64, device="cuda:0")
        cl = torch.full((len(idx),), -1.0, dtype=torch.float64, device="cuda:0")
        call(len(idx), d_idx, ev, cl, stream=stream)
        torch.cuda.synchronize()
        out.append((ev.cpu().numpy(), cl.cpu().numpy()))
    return out


def _deep96():
    rng = np.random.default_rng(4)
    L = 96
    return make_problem(n_layers=L, n_types=2, n_zones=2, mb_list=(1, 2), tp_list=(1,), dp_list=(1, 2),
                        pp_list=[1, 32, 96], global_batch=48, max_segments=2, uniform_layers=False,
                        t_fwd=rng.uniform(0.5e-3, 2e-3, (2, 2, 1, L)),
                        t_bwd=rng.uniform(1e-3, 4e-3, (2, 2, 1, L)), p2p=3_000_000,
                        bw=np.array([[1e10, 1e9], [2e9, 1e10]]), layer_params=1000)


@pytest.mark.parametrize("make, n_first, n_second", [
    (lambda: W.tiny_problem(2, n_zones=3), 700, 90),   # shallow: the allocating call keeps its rings in LDS
    (_deep96, 150, 37),                                 # 96 stages: several batches of the static array
])
def test_static_scratch_matches_the_allocating_entry_point(torch_cuda, make, n_first, n_second):
    prob = make()
    plan = binding.Plan(prob)
    try:
        n = plan.num_candidates()
        rng = np.random.default_rng(11)
        first = rng.integers(0, n, n_first)
        first[3] = n + 5  # an index outside the space: NaN from both
        second = rng.integers(0, n, n_second)
        for idx in (first, second):  # the second call finds the first one's rings in the array
            (ev_a, cl_a), (ev_s, cl_s) = _both(torch_cuda, plan, idx)
            assert np.array_equal(ev_a, ev_s, equal_nan=True)
            assert np.array_equal(cl_a, cl_s, equal_nan=True)
            assert np.isfinite(ev_s).sum() > 0
        assert np.isnan(_both(torch_cuda, plan, first[:8])[1][0][3])
    finally:
        plan.destroy()


def test_static_entry_point_rejects_what_does_not_fit(torch_cuda):
    plan = binding.Plan(W.tiny_problem(1))
    try:
        too_many = 4096 + 1  # SAILOR_STATIC_MAX_PLANS + 1
        d_idx = torch_cuda.zeros(too_many, dtype=torch_cuda.int64, device="cuda:0")
        out = torch_cuda.empty(too_many, dtype=torch_cuda.float64, device="cuda:0")
        with pytest.raises(binding.SailorError) as err:
            plan.simulate_1f1b_static(too_many, d_idx, out, None)
        assert err.value.status == binding.SAILOR_ERANGE
        plan.simulate_1f1b_static(0, None)  # nothing to do
        with pytest.raises(binding.SailorError) as err:
            plan.simulate_1f1b_static(4, d_idx, None, None)
        assert err.value.status == binding.SAILOR_EINVAL
    finally:
        plan.destroy()
