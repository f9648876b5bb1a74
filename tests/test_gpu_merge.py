"""GPU parity of the graph merge (GGM, Alg. 3) against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle as og
import workloads as W

pytestmark = pytest.mark.gpu
SEED = W.ALGO_SEED


def _dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def _exact(x, metric, k):
    ids, dist = og.bruteforce(x, metric, np.arange(len(x)), k)
    return og.Graph(ids, dist, np.zeros_like(ids, dtype=np.uint8))


@pytest.mark.parametrize("path", ["valu", "auto"])
@pytest.mark.parametrize("metric,gen,k,p,n1,iters", [
    (og.L2SQ_F32, lambda n: W.uniform_f32(n, 12, seed=201), 10, 10, 900, 4),
    (og.L2SQ_F32, lambda n: W.sift_like_f32(n, 128, seed=202, n_comp=8), 32, 32, 1100, 3),
    (og.L2SQ_U8, lambda n: W.sift_like_u8(n, 64, seed=203, n_comp=8), 15, 8, 700, 3),
    (og.ANGULAR_F32, lambda n: W.deep_like_f32(n, 48, seed=204, n_comp=8), 16, 16, 1000, 0),
])
def test_merge_matches_oracle(metric, gen, k, p, n1, iters, path):
    import paper_2103_15386_amd as amd
    n = 2000
    x = gen(n)
    g1 = _exact(x[:n1], metric, k)
    g2 = _exact(x[n1:], metric, k)
    want, wstats = og.merge(x, n1, k, p, metric, SEED, g1, g2, iters)
    dt = np.int32 if metric == og.L2SQ_U8 else np.float32
    out = amd.gnnd_merge(_dev(x[:n1]), _dev(x[n1:]), _dev(g1.ids), _dev(g1.dist.astype(dt)),
                         _dev(g2.ids), _dev(g2.dist.astype(dt)), k, p, metric, SEED, iters,
                         join_path=amd.JOIN_VALU if path == "valu" else amd.JOIN_AUTO,
                         want_stats=True)
    ids, dist, stats = out
    assert (ids.cpu().numpy() == want.ids).all()
    assert (dist.cpu().numpy().astype(np.float64) == want.dist).all()
    for a, b in zip(stats[:iters], wstats):
        for key in ("inserts", "dist_evals", "sum_new", "sum_old", "proposals"):
            assert a[key] == b[key], (key, a, b)
        assert a["dropped"] == 0


def test_merge_rejects_bad_arguments():
    import paper_2103_15386_amd as amd
    x = _dev(W.uniform_f32(40, 4, seed=1))
    ids = torch.zeros((20, 10), dtype=torch.int32, device="cuda")
    dist = torch.zeros((20, 10), dtype=torch.float32, device="cuda")
    with pytest.raises(amd.GnndError):  # 20 nodes per side cannot hold k = 32 lists
        amd.gnnd_merge(x[:20].contiguous(), x[20:].contiguous(), ids, dist, ids, dist, 32, 8)
