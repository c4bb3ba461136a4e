"""Hand-built problems for the oracle pins (inputs only, no method arithmetic)."""
import numpy as np

from paper_2504_17096_amd.workloads import Problem

GIB = 1 << 30


def make_problem(*, n_layers=8, n_types=1, n_zones=1, mb_list=(1, 2, 4), tp_list=(1, 2),
                 dp_list=(1, 2, 4), pp_list=None, global_batch=32, max_segments=1, seg3_max_pp=0,
                 partitions=None, layer_params=1_000_000, embed=0, head=0, bytes_per_param=16,
                 grad_bytes=2, t_fwd=1e-3, t_bwd=2e-3, t_upd=0.0, act=1_000_000, p2p=0,
                 cap=64 * GIB, reserved=0, node=8, price=1.0, avail=1024, bw=1e10, egress=None,
                 uniform_layers=True):
    """Scalars are broadcast; arrays are taken as they are."""
    G, Z, L = n_types, n_zones, n_layers
    if pp_list is None:
        pp_list = [d for d in range(1, L + 1) if L % d == 0]
    n_mb, n_tp = len(mb_list), len(tp_list)
    Lc = 1 if uniform_layers else L
    if partitions is None:
        partitions = {}
    n_part, rows = [], []
    for pp in pp_list:
        plist = partitions.get(pp)
        if plist is None:
            base, rem = divmod(L, pp)
            plist = [[base + (1 if i < rem else 0) for i in range(pp)]]
        n_part.append(len(plist))
        for r in plist:
            assert len(r) == pp and sum(r) == L
            rows.extend(r)

    def full(x, shape, dtype):
        return np.ascontiguousarray(np.broadcast_to(np.asarray(x, dtype=dtype), shape)).copy()

    eg = None if egress is None else full(egress, (Z, Z), np.float64)
    return Problem(
        n_layers=L, n_types=G, n_zones=Z,
        mb_values=np.asarray(mb_list, np.int32), tp_values=np.asarray(tp_list, np.int32),
        dp_values=np.asarray(dp_list, np.int32), pp_values=np.asarray(pp_list, np.int32),
        max_segments=max_segments, seg3_max_pp=seg3_max_pp, global_batch=global_batch,
        n_partitions=np.asarray(n_part, np.int32), partition_layers=np.asarray(rows, np.int32),
        layer_params=full(layer_params, (L,), np.uint64), embed_params=embed, head_params=head,
        bytes_per_param=bytes_per_param, grad_bytes_per_param=grad_bytes,
        uniform_layers=uniform_layers,
        t_fwd=full(t_fwd, (G, n_mb, n_tp, Lc), np.float64),
        t_bwd=full(t_bwd, (G, n_mb, n_tp, Lc), np.float64),
        t_upd=full(t_upd, (G, n_tp, Lc), np.float64),
        act_store_bytes=full(act, (n_mb, n_tp), np.uint64),
        p2p_bytes=full(p2p, (n_mb,), np.uint64),
        mem_capacity=full(cap, (G,), np.uint64), mem_reserved=full(reserved, (G,), np.uint64),
        gpus_per_node=full(node, (G,), np.int32), price_per_hour=full(price, (G,), np.float64),
        avail=full(avail, (Z, G), np.int32), bandwidth=full(bw, (Z, Z), np.float64),
        egress_per_byte=eg, name="hand")


def find_index(orc, **want):
    """First candidate index whose decoded fields equal `want` (brute-force search)."""
    for c in range(orc.num_candidates):
        cfg = orc.decode(c)
        if all(getattr(cfg, k) == v for k, v in want.items()):
            return c
    raise LookupError(want)


def wide_problem(seed=0):
    """Every list at its limit: 64 pools (16 zones x 4 types), 8 microbatch sizes, 8 TP
    degrees, 24 DP degrees; a short model so that the space stays small."""
    rng = np.random.default_rng(seed)
    G, Z, L = 4, 16, 2
    mb, tp, dp = tuple(range(1, 9)), tuple(range(1, 9)), tuple(range(1, 25))
    bw = rng.uniform(0.5e9, 2e9, (Z, Z))
    np.fill_diagonal(bw, 1e10)
    eg = rng.uniform(1e-11, 5e-11, (Z, Z))
    return make_problem(
        n_layers=L, n_types=G, n_zones=Z, mb_list=mb, tp_list=tp, dp_list=dp, pp_list=[1, 2],
        global_batch=840, max_segments=2,
        t_fwd=rng.uniform(0.5e-3, 3e-3, (G, 8, 8, 1)), t_bwd=rng.uniform(1e-3, 5e-3, (G, 8, 8, 1)),
        t_upd=rng.uniform(1e-4, 3e-4, (G, 8, 1)), layer_params=30_000_000, embed=7_000_001,
        head=5_000_003, act=rng.integers(10_000_000, 400_000_000, (8, 8)).astype(np.uint64),
        p2p=rng.integers(1_000_000, 9_000_000, 8).astype(np.uint64),
        cap=np.array([4, 2, 1, 1], np.uint64) * np.uint64(GIB), reserved=100_000_000,
        node=np.array([8, 4, 2, 1], np.int32), price=rng.uniform(0.5, 4.0, G),
        avail=rng.integers(0, 40, (Z, G)), bw=bw, egress=eg)
