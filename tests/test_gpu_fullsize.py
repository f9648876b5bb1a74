"""Full-size checks on the benchmark workload (n = 1,000,000, d = 128, k = 32,
p = 32, the launch configuration bench.py times): the initial graph and the
whole first iteration are compared with the oracle element by element; later
iterations, which the oracle cannot replay within the test budget, are checked
through properties that hold at any size and through sampled rows the oracle
can recompute one by one."""
import numpy as np
import pytest
import torch

import oracle as og
import workloads as W

pytestmark = pytest.mark.gpu
SEED = W.ALGO_SEED
N, D, K, P = 1_000_000, 128, 32, 32


@pytest.fixture(scope="module")
def full():
    import paper_2103_15386_amd as amd
    x = W.sift_like_f32(N, D, seed=1002)
    xd = torch.from_numpy(x).cuda()
    ctx = amd.Gnnd(xd, K, P, amd.L2SQ_F32, SEED)  # auto path, as in bench.py
    yield amd, x, xd, ctx
    ctx.close()


def _np(ctx):
    ids, dist, flags = ctx.graph(with_flags=True)
    return ids.cpu().numpy(), dist.cpu().numpy(), flags.cpu().numpy()


def test_first_iteration_equals_oracle_everywhere(full):
    amd, x, xd, ctx = full
    og.set_threads(16)
    ctx.init_random()
    g = og.init_random(x, K, og.L2SQ_F32, SEED)
    ids, dist, flags = _np(ctx)
    assert (ids == g.ids).all() and (dist.astype(np.float64) == g.dist).all() and flags.all()
    print("init equal", flush=True)
    ctx.step_sample()
    snew, cnew, sold, cold = og.sample(g, P, SEED, 1)
    gs = [t.cpu().numpy() for t in ctx.samples()]
    assert (gs[1] == cnew).all() and (gs[0] == snew).all()
    assert (gs[3] == cold).all() and (gs[2] == sold).all()
    print("samples equal", flush=True)
    ctx.step_join()
    st = ctx.step_update()
    pu, pv, pd, pcnt, evals = og.join(x, og.L2SQ_F32, P, snew, cnew, sold, cold)
    print("oracle join done", flush=True)
    ins = og.update(g, P, pu, pv, pd, pcnt)
    ids, dist, flags = _np(ctx)
    assert (ids == g.ids).all(), f"{(ids != g.ids).any(1).sum()} rows differ"
    assert (dist.astype(np.float64) == g.dist).all() and (flags == g.isnew).all()
    assert st["inserts"] == ins and st["dist_evals"] == evals and st["dropped"] == 0
    assert st["sum_new"] == int(cnew.sum()) and st["proposals"] == int(pcnt.sum())


def test_later_iterations_keep_every_invariant(full):
    amd, x, xd, ctx = full
    ids0, dist0, _ = _np(ctx)  # state after the first iteration (previous test)
    rows = W.sample_nodes(N, 300, seed=11)
    tids, tdist = og.bruteforce(x, og.L2SQ_F32, rows, 10)
    recalls = []
    for it in range(2, 8):
        st = ctx.iterate()
        ids, dist, flags = _np(ctx)
        assert st["iter"] == it and st["dropped"] == 0
        assert (dist <= dist0).all()  # every rank of every list only improves
        assert (np.diff(dist, axis=1) >= 0).all()  # ascending
        srt = np.sort(ids, axis=1)
        assert (srt[:, 1:] != srt[:, :-1]).all()  # distinct ids
        assert (ids != np.arange(N)[:, None]).all() and ids.min() >= 0 and ids.max() < N
        assert int(flags.sum()) <= st["inserts"]  # p = k: NEW entries are this round's inserts
        # equal distances are ordered by id
        tie = dist[:, 1:] == dist[:, :-1]
        assert (ids[:, 1:][tie] > ids[:, :-1][tie]).all()
        # sampled rows: stored distances are the true distances of the stored ids
        for r in rows[:40]:
            for j in (0, 7, 31):
                assert dist[r, j] == og.distance(x, og.L2SQ_F32, int(r), int(ids[r, j]))
        rec, _ = og.recall_at(ids[rows], dist[rows].astype(np.float64), tids, tdist, 10)
        recalls.append(rec)
        ids0, dist0 = ids, dist
    assert recalls == sorted(recalls) and recalls[-1] > 0.9, recalls
