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


def x_is_bytes(gen):
    """Whether the generator's vectors are byte valued (0..255 integers, d <= 128)."""
    x = gen(64)
    return x.shape[1] <= 128 and bool(((x == np.rint(x)) & (x >= 0) & (x <= 255)).all())


@pytest.mark.parametrize("path", ["valu", "auto", "direct", "gram"])
@pytest.mark.parametrize("metric,gen,k,p,n1,iters", [
    (og.L2SQ_F32, lambda n: W.uniform_f32(n, 12, seed=201), 10, 10, 900, 4),
    (og.L2SQ_F32, lambda n: W.sift_like_f32(n, 128, seed=202, n_comp=8), 32, 32, 1100, 3),
    (og.L2SQ_U8, lambda n: W.sift_like_u8(n, 64, seed=203, n_comp=8), 15, 8, 700, 3),
    (og.ANGULAR_F32, lambda n: W.deep_like_f32(n, 48, seed=204, n_comp=8), 16, 16, 1000, 0),
    (og.L2SQ_U8, lambda n: W.sift_like_u8(n, 64, seed=205, n_comp=8), 97, 32, 1000, 3),  # long lists
    (og.L2SQ_F32, lambda n: W.uniform_f32(n, 9, seed=206), 128, 16, 800, 2),
    (og.CHI2_F32, lambda n: W.gist_like_f32(n, 40, seed=207, n_comp=8), 14, 10, 1200, 3),
    (og.COSINE_F32, lambda n: W.scaled_directions_f32(n, 24, seed=208, n_comp=8), 16, 12, 1000, 3),
    (og.COSINE_F32, lambda n: W.scaled_directions_f32(n, 10, seed=209, n_comp=4), 70, 16, 900, 2),
    (og.L2SQ_F32, lambda n: W.uniform_f32(n, 10, seed=210), 80, 40, 900, 3),  # long sample lists
])
def test_merge_matches_oracle(metric, gen, k, p, n1, iters, path):
    import paper_2103_15386_amd as amd
    if path == "direct" and not (metric in (og.L2SQ_U8, og.L2SQ_F32) and x_is_bytes(gen)):
        pytest.skip("the matrix-core join takes byte-valued data only")
    if path == "gram" and (metric in (og.L2SQ_U8, og.CHI2_F32) or p > 32):
        pytest.skip("the float32 matrix-core join takes float vectors, inner-product metrics, p <= 32")
    n = 2000
    x = gen(n)
    g1 = _exact(x[:n1], metric, k)
    g2 = _exact(x[n1:], metric, k)
    g2.ids += n1  # lists carry the ids of the union
    want, wstats = og.merge(x, n1, k, p, metric, SEED, g1, g2, iters)
    dt = np.int32 if metric == og.L2SQ_U8 else np.float32
    out = amd.gnnd_merge(_dev(x[:n1]), _dev(x[n1:]), _dev(g1.ids), _dev(g1.dist.astype(dt)),
                         _dev(g2.ids), _dev(g2.dist.astype(dt)), k, p, metric, SEED, iters,
                         join_path={"valu": amd.JOIN_VALU, "auto": amd.JOIN_AUTO,
                                    "direct": amd.JOIN_MFMA_DIRECT, "gram": amd.JOIN_GRAM}[path],
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


def test_merge_with_frozen_third_shard_entries_matches_oracle():
    # shards A, B, C of one collection: merge (A, B), then (A, C) where A's lists
    # already point into B - those entries are frozen during the second merge.
    import paper_2103_15386_amd as amd
    k, p, m, metric = 16, 16, 700, og.L2SQ_U8
    x = W.sift_like_u8(3 * m, 64, seed=301, n_comp=6)
    A, B, Cc = slice(0, m), slice(m, 2 * m), slice(2 * m, 3 * m)
    gA, gB, gC = _exact(x[A], metric, k), _exact(x[B], metric, k), _exact(x[Cc], metric, k)
    gB.ids += m
    gC.ids += 2 * m
    xAB = np.concatenate([x[A], x[B]])
    wAB, _ = og.merge(xAB, m, k, p, metric, SEED, gA, gB, 3, 0, m)
    ids, dist = amd.gnnd_merge(_dev(x[A]), _dev(x[B]), _dev(gA.ids), _dev(gA.dist.astype(np.int32)),
                               _dev(gB.ids), _dev(gB.dist.astype(np.int32)), k, p, metric, SEED, 3,
                               base1=0, base2=m, id_space=3 * m)
    assert (ids.cpu().numpy() == wAB.ids).all() and (dist.cpu().numpy() == wAB.dist).all()
    gA2 = og.Graph(wAB.ids[:m].copy(), wAB.dist[:m].copy(), None)
    assert (gA2.ids >= m).any()
    # second merge with the ranges in "wrong" order: S1 = C, S2 = A
    xCA = np.concatenate([x[Cc], x[A]])
    wCA, wst = og.merge(xCA, m, k, p, metric, SEED + 1, gC, gA2, 3, 2 * m, 0)
    ids, dist, st = amd.gnnd_merge(_dev(x[Cc]), _dev(x[A]), _dev(gC.ids),
                                   _dev(gC.dist.astype(np.int32)), _dev(gA2.ids),
                                   _dev(gA2.dist.astype(np.int32)), k, p, metric, SEED + 1, 3,
                                   want_stats=True, base1=2 * m, base2=0, id_space=3 * m)
    assert (ids.cpu().numpy() == wCA.ids).all() and (dist.cpu().numpy() == wCA.dist).all()
    for a, b in zip(st, wst):
        assert a["inserts"] == b["inserts"] and a["dist_evals"] == b["dist_evals"]
    assert (wCA.ids[m:] >= m).any() and ((wCA.ids[m:] >= m) & (wCA.ids[m:] < 2 * m)).any()


@pytest.mark.parametrize("metric,gen,shards,n", [
    (og.L2SQ_U8, lambda n: W.sift_like_u8(n, 128, seed=302, n_comp=8), 4, 4000),
    (og.L2SQ_F32, lambda n: W.uniform_f32(n, 10, seed=303), 3, 2001),
])
def test_sharded_build_matches_oracle(metric, gen, shards, n):
    import paper_2103_15386_amd as amd
    k, p = 12, 12
    x = gen(n)
    want = og.build_sharded(x, shards, k, p, metric, SEED, 5, 3)
    xh = torch.from_numpy(x).pin_memory()
    ids, dist, st = amd.gnnd_build_sharded(xh, shards, k, p, metric, SEED, 5, 3)
    assert (ids.numpy() == want.ids).all()
    assert (dist.numpy().astype(np.float64) == want.dist).all()
    assert st["builds"] == shards and st["merges"] == shards * (shards - 1) // 2
    # quality: the sharded graph is close to the exact one
    q = W.sample_nodes(n, 300, seed=5)
    ti, td = og.bruteforce(x, metric, q, 10)
    rec, _ = og.recall_at(want.ids[q], want.dist[q], ti, td, 10)
    assert rec > 0.85, rec


@pytest.mark.parametrize("metric,gen,shards,n,staging", [
    (og.L2SQ_U8, lambda n: W.sift_like_u8(n, 128, seed=302, n_comp=8), 4, 4000, 1 << 20),
    (og.L2SQ_F32, lambda n: W.uniform_f32(n, 300, seed=306), 3, 3001, (1 << 20) + 4096),
])
def test_sharded_build_from_files_matches_oracle(metric, gen, shards, n, staging, tmp_path):
    """The collection and the graph live in files; transfers go through one pinned
    staging buffer.  In the second case a shard's vectors (1.2 MB) exceed it, so
    those transfers are cut into pieces, the last one ragged."""
    import paper_2103_15386_amd as amd
    k, p = 12, 12
    x = gen(n)
    want = og.build_sharded(x, shards, k, p, metric, SEED, 5, 3)
    x.tofile(tmp_path / "vectors.bin")
    (tmp_path / "ids.bin").write_bytes(b"\xff" * 10)  # an older, shorter file is overwritten
    st = amd.gnnd_build_sharded_files(tmp_path / "vectors.bin", n, x.shape[1], shards, k, p,
                                      tmp_path / "ids.bin", tmp_path / "dist.bin", metric, SEED,
                                      5, 3, staging_bytes=staging)
    dt = np.int32 if metric == og.L2SQ_U8 else np.float32
    ids = np.fromfile(tmp_path / "ids.bin", dtype=np.int32).reshape(n, k)
    dist = np.fromfile(tmp_path / "dist.bin", dtype=dt).reshape(n, k)
    assert (ids == want.ids).all()
    assert (dist.astype(np.float64) == want.dist).all()
    assert st["builds"] == shards and st["merges"] == shards * (shards - 1) // 2


def test_sharded_build_from_files_reports_file_errors(tmp_path):
    import paper_2103_15386_amd as amd
    x = W.uniform_f32(2000, 8, seed=307)
    with pytest.raises(amd.GnndError) as e:
        amd.gnnd_build_sharded_files(tmp_path / "missing.bin", 2000, 8, 2, 8, 8,
                                     tmp_path / "i.bin", tmp_path / "d.bin")
    assert e.value.code == amd.binding.EIO
    x[:1000].tofile(tmp_path / "short.bin")
    with pytest.raises(amd.GnndError) as e:
        amd.gnnd_build_sharded_files(tmp_path / "short.bin", 2000, 8, 2, 8, 8,
                                     tmp_path / "i.bin", tmp_path / "d.bin")
    assert e.value.code == amd.binding.EIO and "shorter" in str(e.value)


@pytest.mark.parametrize("metric,gen,n1,n2", [
    (og.L2SQ_F32, lambda n: W.uniform_f32(n, 12, seed=304), 1300, 700),
    (og.L2SQ_U8, lambda n: W.sift_like_u8(n, 128, seed=305, n_comp=8), 900, 1100),
])
def test_append_matches_oracle(metric, gen, n1, n2):
    import paper_2103_15386_amd as amd
    k, p = 12, 12
    x = gen(n1 + n2)
    g1 = _exact(x[:n1], metric, k)
    want = og.append(x, n1, g1, k, p, metric, SEED, 5, 4)
    dt = np.int32 if metric == og.L2SQ_U8 else np.float32
    ids, dist = amd.gnnd_append(_dev(x[:n1]), _dev(g1.ids), _dev(g1.dist.astype(dt)),
                                _dev(x[n1:]), k, p, metric, SEED, 5, 4)
    assert (ids.cpu().numpy() == want.ids).all()
    assert (dist.cpu().numpy().astype(np.float64) == want.dist).all()


def test_append_rejects_a_batch_smaller_than_k():
    import paper_2103_15386_amd as amd
    x = _dev(W.uniform_f32(60, 4, seed=2))
    ids = torch.zeros((50, 16), dtype=torch.int32, device="cuda")
    dist = torch.zeros((50, 16), dtype=torch.float32, device="cuda")
    with pytest.raises(amd.GnndError):
        amd.gnnd_append(x[:50].contiguous(), ids, dist, x[50:].contiguous(), 16, 8)


@pytest.mark.parametrize("case_seed", list(range(3001, 3013)))
def test_random_merge_configurations_match_oracle(case_seed):
    # seeded draws of (n1, n2, d, k, p, metric, iterations); the inputs are graphs
    # the oracle built with a few iterations (not exact ones), in collection ids
    import paper_2103_15386_amd as amd
    rng = np.random.default_rng(case_seed)
    metric = int(rng.choice([og.L2SQ_F32, og.ANGULAR_F32, og.L2SQ_U8, og.CHI2_F32]))
    k = int(rng.choice([2, 5, 16, 31, 32, 40, 64, 65, 100, 128]))
    p = int(rng.integers(1, min(k, 32) + 1))
    n1 = int(rng.integers(k + 1, 800))
    n2 = int(rng.integers(k + 1, 800))
    d = int(rng.choice([2, 7, 16, 33, 64, 128]))
    iters = int(rng.integers(0, 4))
    seed = int(rng.integers(1, 1 << 30))
    n = n1 + n2
    if metric == og.L2SQ_U8:
        x = W.sift_like_u8(n, d, seed=seed, n_comp=4)
    elif metric == og.ANGULAR_F32:
        x = W.deep_like_f32(n, d, seed=seed, n_comp=4)
    elif metric == og.CHI2_F32:
        x = W.gist_like_f32(n, d, seed=seed, n_comp=4)
    else:
        x = W.small_integer_f32(n, d, seed=seed) if rng.random() < 0.5 else \
            W.uniform_f32(n, d, seed=seed)
    algo_seed = int(rng.integers(0, 1 << 40))
    g1, _ = og.build(np.ascontiguousarray(x[:n1]), k, p, metric, algo_seed + 1, 2)
    g2, _ = og.build(np.ascontiguousarray(x[n1:]), k, p, metric, algo_seed + 2, 2)
    g2.ids += n1
    want, _ = og.merge(x, n1, k, p, metric, algo_seed, g1, g2, iters)
    dt = np.int32 if metric == og.L2SQ_U8 else np.float32
    ids, dist = amd.gnnd_merge(_dev(x[:n1]), _dev(x[n1:]), _dev(g1.ids), _dev(g1.dist.astype(dt)),
                               _dev(g2.ids), _dev(g2.dist.astype(dt)), k, p, metric, algo_seed,
                               iters)
    what = f"n1={n1} n2={n2} d={d} k={k} p={p} metric={metric} iters={iters}"
    assert (ids.cpu().numpy() == want.ids).all(), what
    assert (dist.cpu().numpy().astype(np.float64) == want.dist).all(), what
