"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs, element by element.  With the per-pair in-order fused
arithmetic both sides compute the same float32 bits, so ids, distances, flags,
sample lists and counters are compared for equality."""
from collections import Counter

import numpy as np
import pytest
import torch

import oracle as og
import workloads as W

pytestmark = pytest.mark.gpu

SEED = W.ALGO_SEED


def _amd():
    import paper_2103_15386_amd as amd
    return amd


def _dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def _graph_np(ctx):
    ids, dist, flags = ctx.graph(with_flags=True)
    return ids.cpu().numpy(), dist.cpu().numpy().astype(np.float64), flags.cpu().numpy()


def _assert_graph_equal(ctx, g, what):
    ids, dist, flags = _graph_np(ctx)
    assert (ids == g.ids).all(), f"{what}: ids differ in {(ids != g.ids).any(1).sum()} rows"
    assert (dist == g.dist).all(), f"{what}: distances differ"
    assert (flags == g.isnew).all(), f"{what}: NEW flags differ"


CASES = {
    # name: (generator, metric, k, p, iters)
    "uniform_c1": (lambda: W.uniform_f32(4096, 16, seed=1001), og.L2SQ_F32, 10, 8, 8),
    "sift_cut": (lambda: W.sift_like_f32(3000, 128, seed=1002, n_comp=16), og.L2SQ_F32, 32, 32, 5),
    "deep_cut_angular": (lambda: W.deep_like_f32(2500, 96, seed=1004, n_comp=16),
                         og.ANGULAR_F32, 20, 12, 5),
    "u8_cut": (lambda: W.sift_like_u8(2500, 128, seed=1005, n_comp=16), og.L2SQ_U8, 32, 16, 5),
    "ragged_d13_k64": (lambda: W.uniform_f32(1500, 13, seed=5), og.L2SQ_F32, 64, 32, 4),
    "gist_cut_d200": (lambda: W.gist_like_f32(1200, 200, seed=1003, n_comp=8),
                      og.L2SQ_F32, 16, 16, 4),
    "tiny_n": (lambda: W.uniform_f32(70, 7, seed=6), og.L2SQ_F32, 5, 3, 4),
    "u8_d30": (lambda: W.sift_like_u8(900, 30, seed=8, n_comp=4), og.L2SQ_U8, 12, 12, 4),
    # chi-square distance on histogram-like (non-negative, L1-normalised) vectors
    "chi2_gist_cut": (lambda: W.gist_like_f32(1500, 96, seed=1031, n_comp=8),
                      og.CHI2_F32, 20, 16, 4),
    "chi2_ragged_d7": (lambda: W.gist_like_f32(600, 7, seed=1032, n_comp=4), og.CHI2_F32, 9, 6, 4),
    # long vectors: many staged chunks, ragged ends; bytes beyond the matrix-core kernel's 128
    "l2_d1031": (lambda: W.uniform_f32(400, 1031, seed=1071), og.L2SQ_F32, 8, 4, 3),
    "u8_d1000": (lambda: W.sift_like_u8(500, 1000, seed=1072, n_comp=4), og.L2SQ_U8, 10, 10, 3),
    "u8_d257": (lambda: W.sift_like_u8(500, 257, seed=1073, n_comp=4), og.L2SQ_U8, 6, 3, 3),
    "cosine_d515": (lambda: W.scaled_directions_f32(400, 515, seed=1074, n_comp=4),
                    og.COSINE_F32, 7, 7, 3),
    # cosine distance of vectors of any length (per-vector squared norms), with zero vectors
    "cosine_raw_d96": (lambda: W.scaled_directions_f32(2500, 96, seed=1061, n_comp=16),
                       og.COSINE_F32, 20, 12, 5),
    "cosine_ragged_d11_zero_rows": (lambda: W.scaled_directions_f32(700, 11, seed=1062, n_comp=4,
                                                                    zero_rows=3),
                                    og.COSINE_F32, 9, 6, 4),
    "cosine_k80": (lambda: W.scaled_directions_f32(1500, 32, seed=1063, n_comp=8),
                   og.COSINE_F32, 80, 20, 3),
    # lists longer than one wavefront (two entries per lane)
    "k128_uniform": (lambda: W.uniform_f32(1800, 10, seed=1021), og.L2SQ_F32, 128, 32, 4),
    "k100_angular": (lambda: W.deep_like_f32(1500, 48, seed=1022, n_comp=8),
                     og.ANGULAR_F32, 100, 24, 4),
    "k65_tiny": (lambda: W.uniform_f32(140, 6, seed=1023), og.L2SQ_F32, 65, 9, 3),
    # sample lists longer than one wavefront (p > 32: the paper varies p up to 42, Sec. 6.3)
    "p42_k64": (lambda: W.uniform_f32(2000, 12, seed=1081), og.L2SQ_F32, 64, 42, 4),
    "p64_k128_u8": (lambda: W.sift_like_u8(1500, 32, seed=1082, n_comp=6), og.L2SQ_U8, 128, 64, 3),
    "p33_k40_angular": (lambda: W.deep_like_f32(1200, 24, seed=1083, n_comp=8),
                        og.ANGULAR_F32, 40, 33, 4),
    "p40_k48_cosine_d70": (lambda: W.scaled_directions_f32(900, 70, seed=1084, n_comp=6),
                           og.COSINE_F32, 48, 40, 3),
    "p50_k50_small_n": (lambda: W.uniform_f32(90, 5, seed=1085), og.L2SQ_F32, 50, 50, 3),
}


@pytest.mark.parametrize("name", list(CASES))
def test_init_matches_oracle(name):
    amd = _amd()
    gen, metric, k, p, _ = CASES[name]
    x = gen()
    ctx = amd.Gnnd(_dev(x), k, p, metric, SEED)
    ctx.init_random()
    _assert_graph_equal(ctx, og.init_random(x, k, metric, SEED), "init")
    ctx.close()


MFMA_CASES = ["sift_cut", "u8_cut", "u8_d30", "sift_d100_k64", "u8_small_lists", "u8_k96",
              "sift_k128"]
CASES["u8_k96"] = (lambda: W.sift_like_u8(1600, 96, seed=1024, n_comp=8), og.L2SQ_U8, 96, 32, 4)
CASES["sift_k128"] = (lambda: W.sift_like_f32(1700, 128, seed=1025, n_comp=8),
                      og.L2SQ_F32, 128, 20, 3)
CASES["sift_d100_k64"] = (lambda: W.sift_like_f32(2000, 100, seed=1012, n_comp=8),
                          og.L2SQ_F32, 64, 32, 4)
CASES["u8_small_lists"] = (lambda: W.sift_like_u8(1500, 64, seed=1013, n_comp=4),
                           og.L2SQ_U8, 8, 5, 5)


# float32 matrix-core join: inner products by matrix instructions pick the partners, canonical
# sums decide - every float case with p <= 32 under squared L2, angular or cosine, and two
# with groups of (almost) identical vectors, where many partners stay in the race
CASES["near_copies_d24"] = (lambda: W.near_copies_f32(1600, 24, seed=1091), og.L2SQ_F32, 24, 16, 4)
CASES["near_copies_cosine_d70"] = (lambda: W.near_copies_f32(1200, 70, seed=1092, copies=12),
                                   og.COSINE_F32, 20, 20, 4)
# full sample lists (p = 32) over enough iterations that nodes of every shape occur - few to 64
# NEW samples, none to 64 OLD - under the other two metrics as well ("sift_cut" is squared L2)
CASES["deep_cut_angular_p32"] = (lambda: W.deep_like_f32(2200, 96, seed=1093, n_comp=12),
                                 og.ANGULAR_F32, 32, 32, 5)
CASES["cosine_p32_d40"] = (lambda: W.scaled_directions_f32(2000, 40, seed=1094, n_comp=10),
                           og.COSINE_F32, 32, 32, 5)
GRAM_CASES = [n for n, c in CASES.items()
              if c[1] in (og.L2SQ_F32, og.ANGULAR_F32, og.COSINE_F32) and c[3] <= 32]



def _gram_build_of(rb, co):
    """Which of its seven builds the float matrix-core join uses for a node with rb blocks of
    16 NEW and co blocks of 16 OLD samples (restated from the kernel's rule, only to check
    below that the parity cases exercise every build)."""
    if co == 0:
        return 0
    if rb <= 1 and co <= 2:
        return 1
    if rb <= 3 and co <= 1:
        return 2
    if rb <= 1:
        return 3
    if rb <= 2:
        return 4
    return 5 if co <= 2 else 6


@pytest.mark.parametrize("name", ["sift_cut", "deep_cut_angular_p32", "cosine_p32_d40"])
def test_gram_parity_cases_reach_every_build_of_the_kernel(name):
    """These cases (checked stage by stage against the oracle below, one per metric) have nodes
    for each of the seven builds of the float matrix-core join."""
    amd = _amd()
    gen, metric, k, p, iters = CASES[name]
    ctx = amd.Gnnd(_dev(gen()), k, p, metric, SEED, amd.JOIN_GRAM)
    ctx.init_random()
    seen = set()
    for _ in range(iters):
        ctx.step_sample()
        _, cnew, _, cold = [t.cpu().numpy() for t in ctx.samples()]
        work = (cnew > 1) | ((cnew > 0) & (cold > 0))
        seen |= {_gram_build_of(int(a), int(b))
                 for a, b in zip((cnew[work] + 15) >> 4, (cold[work] + 15) >> 4)}
        ctx.step_join()
        ctx.step_update(False)
    assert seen == set(range(7)), seen

# "all": the variant that proposes every evaluated pair (no selective update)
ALL_PAIRS_CASES = ["uniform_c1", "u8_cut", "deep_cut_angular", "tiny_n", "k100_angular",
                   "cosine_ragged_d11_zero_rows"]


@pytest.mark.parametrize("name,path", [(n, "valu") for n in CASES] +
                         [(n, "mfma") for n in MFMA_CASES] +
                         [(n, "mfma_direct") for n in MFMA_CASES] +
                         [(n, "gram") for n in GRAM_CASES] +
                         [(n, "all") for n in ALL_PAIRS_CASES])
def test_every_stage_of_every_iteration_matches_oracle(name, path):
    amd = _amd()
    gen, metric, k, p, iters = CASES[name]
    x = gen()
    n = len(x)
    every = path == "all"
    # "mfma": results leave the join staged per bucket of destinations; "mfma_direct": one by one
    join = {"mfma": amd.JOIN_MFMA, "mfma_direct": amd.JOIN_MFMA_DIRECT,
            "gram": amd.JOIN_GRAM}.get(path, amd.JOIN_VALU)
    ctx = amd.Gnnd(_dev(x), k, p, metric, SEED, join,
                   amd.UPDATE_ALL_PAIRS if every else amd.UPDATE_SELECTIVE)
    assert ctx.join_path() == {"mfma_direct": amd.JOIN_MFMA}.get(path, join) or path == "all"
    ctx.init_random()
    g = og.init_random(x, k, metric, SEED)
    for it in range(1, iters + 1):
        before = g.copy()
        # --- sampling -----------------------------------------------------
        ctx.step_sample()
        snew, cnew, sold, cold = og.sample(g, p, SEED, it)
        gs = [t.cpu().numpy() for t in ctx.samples()]
        assert (gs[1] == cnew).all() and (gs[3] == cold).all(), f"it {it}: sample sizes"
        assert (gs[0] == snew).all() and (gs[2] == sold).all(), f"it {it}: sample lists"
        # --- cross-matching + nearest objects ------------------------------
        ctx.step_join()
        pu, pv, pd, pcnt, evals = og.join(x, metric, p, snew, cnew, sold, cold, all_pairs=every)
        gu, gv, gd = [t.cpu().numpy().ravel() for t in ctx.proposals()]
        used = gu >= 0
        got = Counter(zip(gu[used].tolist(), gv[used].tolist(), gd[used].astype(np.float64).tolist()))
        want = Counter((int(pu[s, j]), int(pv[s, j]), float(pd[s, j]))
                       for s in range(n) for j in range(pcnt[s]))
        kth = before.dist[:, k - 1]
        assert not (got - want), f"it {it}: GPU proposed something the oracle did not"
        for (u, v, dd), c in (want - got).items():  # only hopeless results may be dropped early
            assert dd > kth[u], f"it {it}: dropped an admissible proposal for list {u}"
        # --- update ----------------------------------------------------------
        st = ctx.step_update()
        ins = og.update(g, p, pu, pv, pd, pcnt)
        _assert_graph_equal(ctx, g, f"iteration {it}")
        assert st["iter"] == it
        assert st["inserts"] == ins
        assert st["dist_evals"] == evals
        assert st["sum_new"] == int(cnew.sum()) and st["sum_old"] == int(cold.sum())
        assert st["proposals"] == int(pcnt.sum()) and st["dropped"] == 0
        if not every:  # what the join (or the pass behind it) let through = what the update saw
            assert st["passed"] == int(used.sum()), f"it {it}: passed"
    ctx.close()


def test_build_equals_stepwise_and_is_deterministic():
    amd = _amd()
    x = W.uniform_f32(4096, 16, seed=1001)
    xd = _dev(x)
    ids_a, dist_a, ctx_a = amd.gnnd_build(xd, 10, 8, amd.L2SQ_F32, SEED, iters=8)
    ids_b, dist_b, ctx_b = amd.gnnd_build(xd, 10, 8, amd.L2SQ_F32, SEED, iters=8)
    assert torch.equal(ids_a, ids_b) and torch.equal(dist_a, dist_b)
    g, _ = og.build(x, 10, 8, og.L2SQ_F32, SEED, 8)
    _assert_graph_equal(ctx_a, g, "build")
    # end-to-end quality agrees with the oracle's (identical graphs => identical recall)
    q = torch.arange(4096, dtype=torch.int32, device="cuda")
    tids, tdist = amd.exact_knn(xd, q, 10, amd.L2SQ_F32)
    r_gpu = amd.recall_at(dist_a, tdist, 10)
    oi, od = og.bruteforce(x, og.L2SQ_F32, np.arange(4096), 10)
    r_cpu, _ = og.recall_at(g.ids, g.dist, oi, od, 10)
    assert abs(r_gpu - r_cpu) <= 0.005 and r_gpu > 0.85
    # a different seed gives a different graph
    ids_c, _, ctx_c = amd.gnnd_build(xd, 10, 8, amd.L2SQ_F32, SEED + 1, iters=2)
    ids_d, _, ctx_d = amd.gnnd_build(xd, 10, 8, amd.L2SQ_F32, SEED, iters=2)
    assert not torch.equal(ids_c, ids_d)
    for c in (ctx_a, ctx_b, ctx_c, ctx_d):
        c.close()


def test_resume_from_saved_graph_gives_the_same_bytes():
    amd = _amd()
    x = W.uniform_f32(2000, 12, seed=77)
    xd = _dev(x)
    a = amd.Gnnd(xd, 12, 6, amd.L2SQ_F32, SEED)
    a.init_random()
    for _ in range(2):
        a.iterate(False)
    ids, dist, flags = a.graph(with_flags=True)
    b = amd.Gnnd(xd, 12, 6, amd.L2SQ_F32, SEED)
    b.set_graph(ids, dist, flags, 2)
    for _ in range(2):
        a.iterate(False)
        b.iterate(False)
    ga, gb = a.graph(with_flags=True), b.graph(with_flags=True)
    assert all(torch.equal(s, t) for s, t in zip(ga, gb))
    a.close()
    b.close()


@pytest.mark.parametrize("metric,gen", [
    (og.L2SQ_F32, lambda: W.uniform_f32(3000, 24, seed=91)),
    (og.ANGULAR_F32, lambda: W.deep_like_f32(3000, 32, seed=92, n_comp=8)),
    (og.L2SQ_U8, lambda: W.sift_like_u8(3000, 40, seed=93, n_comp=8)),
    (og.L2SQ_F32, lambda: W.small_integer_f32(2000, 5, seed=94, hi=4)),  # masses of ties
    (og.CHI2_F32, lambda: W.gist_like_f32(2500, 30, seed=95, n_comp=8)),
    (og.COSINE_F32, lambda: W.scaled_directions_f32(2500, 30, seed=96, n_comp=8, zero_rows=2)),
])
def test_exact_knn_matches_oracle_brute_force(metric, gen):
    amd = _amd()
    x = gen()
    q = W.sample_nodes(len(x), 200, seed=3)
    ids, dist = amd.exact_knn(_dev(x), _dev(q), 10, metric)
    oi, od = og.bruteforce(x, metric, q, 10)
    assert (ids.cpu().numpy() == oi).all()
    assert (dist.cpu().numpy().astype(np.float64) == od).all()
    # query ids that are no nodes are answered with "none", not read
    bad = torch.tensor([len(x), -1, 5], dtype=torch.int32, device="cuda")
    ids, dist = amd.exact_knn(_dev(x), bad, 10, metric)
    assert (ids[:2] == -1).all() and (ids[2] >= 0).all()


def test_errors_are_reported_not_fatal():
    amd = _amd()
    x = _dev(W.uniform_f32(100, 8, seed=1))
    with pytest.raises(amd.GnndError):
        amd.Gnnd(x, 100, 8)  # k >= n
    with pytest.raises(amd.GnndError):
        amd.Gnnd(x, 10, 11)  # p > k
    ctx = amd.Gnnd(x, 10, 8)
    with pytest.raises(amd.GnndError) as e:
        ctx.iterate()  # no graph yet
    assert e.value.code == -3
    ctx.init_random()
    with pytest.raises(amd.GnndError):
        ctx.step_join()  # out of order
    ctx.close()
    with pytest.raises(amd.GnndError):
        amd.Gnnd(torch.zeros(100, 8), 10, 8)  # CPU tensor: no CPU path
    with pytest.raises(amd.GnndError):  # matrix-core path refuses non-integer floats
        amd.Gnnd(x, 10, 8, amd.L2SQ_F32, 42, amd.JOIN_MFMA)
    # a graph with an id that is no node, or a node in its own list, is refused on loading
    # (ids become row numbers), and the context goes on working with a valid one
    ctx = amd.Gnnd(x, 10, 8)
    ctx.init_random()
    ids, dist, flags = ctx.graph(with_flags=True)
    for row, col, value in ((3, 2, 100), (7, 0, -1), (11, 4, 11), (99, 9, 1 << 30)):
        broken = ids.clone()
        broken[row, col] = value
        with pytest.raises(amd.GnndError) as e:
            ctx.set_graph(broken, dist, flags, 0)
        assert e.value.code == -1
        with pytest.raises(amd.GnndError):
            ctx.iterate()  # no graph any more
    ctx.set_graph(ids, dist, flags, 0)
    assert ctx.iterate()["inserts"] > 0
    ctx.close()


def test_build_with_the_delta_rule_stops_where_the_oracle_does():
    # optional termination (off by default): stop after the first iteration that
    # admits fewer than delta * n * k entries
    amd = _amd()
    x = W.uniform_f32(3000, 12, seed=61)
    k, p, delta = 12, 8, 0.02
    ctx = amd.Gnnd(_dev(x), k, p, amd.L2SQ_F32, SEED)
    last = ctx.build(30, delta=delta)
    g = og.init_random(x, k, og.L2SQ_F32, SEED)
    stopped_at = None
    for it in range(1, 31):
        st = og.iterate(x, og.L2SQ_F32, g, p, SEED, it)
        if st["inserts"] < delta * len(x) * k:
            stopped_at = it
            break
    assert stopped_at is not None and 2 < stopped_at < 30
    assert last["iter"] == stopped_at and last["inserts"] == st["inserts"]
    _assert_graph_equal(ctx, g, "build with delta")
    ctx.close()


def test_stage_times_are_recorded_per_iteration():
    amd = _amd()
    x = W.sift_like_u8(20000, 64, seed=62, n_comp=8)
    ctx = amd.Gnnd(_dev(x), 16, 16, amd.L2SQ_U8, SEED)
    ctx.set_profiling(1)
    torch.cuda.synchronize()
    import time
    t0 = time.perf_counter()
    ctx.build(5, want_stats=False)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    count, missed, ms_sample, ms_join, ms_handout, ms_update = ctx.stage_ms()
    assert count == 5 and missed == 0
    assert ms_sample > 0 and ms_join > 0 and ms_handout > 0 and ms_update > 0
    assert ms_sample + ms_join + ms_handout + ms_update <= wall_ms
    count, missed, *_ = ctx.stage_ms()  # reading clears the record
    assert count == 0 and missed == 0
    # a window holds what was asked for (never fewer than 64 iterations); what does not
    # fit is counted, not dropped silently: 20 builds of 7 iterations against a window of 100
    ctx.set_profiling(100)
    for _ in range(20):
        ctx.build(7, want_stats=False)
    count, missed, *_ = ctx.stage_ms()
    assert (count, missed) == (100, 40)
    ctx.set_profiling(140)
    for _ in range(20):
        ctx.build(7, want_stats=False)
    count, missed, ms_sample, ms_join, ms_handout, ms_update = ctx.stage_ms()
    assert (count, missed) == (140, 0) and min(ms_sample, ms_join, ms_handout, ms_update) > 0
    ctx.close()


def test_the_library_serves_a_plain_c_program():
    # csrc/abi_demo.c (C11, gcc, hipMalloc for memory; no Python, no torch in the
    # process) builds a graph through the C ABI and checks it against
    # gnnd_exact_knn; built in-tree by paper_2103_15386_amd/build.py
    import os
    import subprocess
    import paper_2103_15386_amd as amd
    exe = os.path.join(os.path.dirname(amd.library_path()), "abi_demo")
    if not os.path.exists(exe):
        pytest.skip("abi_demo is not built (python -m paper_2103_15386_amd.build)")
    r = subprocess.run([exe, "20000", "16", "16", "8", "8"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "malformed=0" in r.stdout and "iterations=8" in r.stdout
    recall = float(r.stdout.split("recall@10=")[1].split()[0])
    assert recall > 0.9
    # same parameters, same seed: the graph of the Python binding reaches the same recall
    r2 = subprocess.run([exe, "20000", "16", "16", "8", "8"], capture_output=True, text=True,
                        timeout=120)
    assert r2.stdout == r.stdout  # deterministic


def _random_case(rng):
    metric = int(rng.choice([og.L2SQ_F32, og.ANGULAR_F32, og.L2SQ_U8, og.CHI2_F32]))
    k = int(rng.choice([2, 3, 7, 16, 31, 32, 33, 50, 64, 65, 90, 128]))
    p = int(rng.integers(1, min(k, 32) + 1))
    n = int(rng.integers(k + 2, 1400))
    d = int(rng.choice([1, 2, 3, 5, 8, 17, 32, 33, 64, 100, 128, 131]))
    seed = int(rng.integers(1, 1 << 30))
    if metric == og.L2SQ_U8:
        x = W.sift_like_u8(n, d, seed=seed, n_comp=4)
    elif metric == og.ANGULAR_F32:
        x = W.deep_like_f32(n, d, seed=seed, n_comp=4)
    elif metric == og.CHI2_F32:
        x = W.gist_like_f32(n, d, seed=seed, n_comp=4)
    else:
        x = W.uniform_f32(n, d, seed=seed) if rng.random() < 0.5 else \
            W.small_integer_f32(n, d, seed=seed)  # the second kind takes the matrix-core path
    return x, metric, k, p


@pytest.mark.parametrize("case_seed", list(range(2001, 2025)))
def test_random_configurations_match_oracle(case_seed):
    # seeded draws of (n, d, k, p, metric, data): three iterations, whole graph compared
    amd = _amd()
    rng = np.random.default_rng(case_seed)
    x, metric, k, p = _random_case(rng)
    algo_seed = int(rng.integers(0, 1 << 40))
    ctx = amd.Gnnd(_dev(x), k, p, metric, algo_seed)
    ctx.init_random()
    g = og.init_random(x, k, metric, algo_seed)
    _assert_graph_equal(ctx, g, f"init {x.shape} k={k} p={p} metric={metric}")
    for it in range(1, 4):
        st = ctx.iterate()
        want = og.iterate(x, metric, g, p, algo_seed, it)
        _assert_graph_equal(ctx, g, f"iteration {it} {x.shape} k={k} p={p} metric={metric}")
        for key in ("inserts", "dist_evals", "sum_new", "sum_old", "proposals"):
            assert st[key] == want[key], (key, st, x.shape, k, p, metric)
    ctx.close()


@pytest.mark.parametrize("case_seed", list(range(3001, 3011)))
def test_random_cosine_configurations_match_oracle(case_seed):
    # the same for the metric with per-vector norms: random lengths, a few zero vectors,
    # both update modes
    amd = _amd()
    rng = np.random.default_rng(case_seed)
    k = int(rng.choice([2, 5, 16, 32, 33, 64, 70, 128]))
    p = int(rng.integers(1, min(k, 32) + 1))
    n = int(rng.integers(k + 2, 1200))
    d = int(rng.choice([1, 3, 8, 31, 64, 96, 130]))
    every = bool(rng.random() < 0.3) and p <= 8
    x = W.scaled_directions_f32(n, d, seed=int(rng.integers(1, 1 << 30)), n_comp=4,
                                zero_rows=int(rng.integers(0, 4)))
    algo_seed = int(rng.integers(0, 1 << 40))
    ctx = amd.Gnnd(_dev(x), k, p, og.COSINE_F32, algo_seed, amd.JOIN_AUTO,
                   amd.UPDATE_ALL_PAIRS if every else amd.UPDATE_SELECTIVE)
    ctx.init_random()
    g = og.init_random(x, k, og.COSINE_F32, algo_seed)
    _assert_graph_equal(ctx, g, f"init {x.shape} k={k} p={p}")
    for it in range(1, 4):
        st = ctx.iterate()
        want = og.iterate(x, og.COSINE_F32, g, p, algo_seed, it, all_pairs=every)
        _assert_graph_equal(ctx, g, f"iteration {it} {x.shape} k={k} p={p} all_pairs={every}")
        for key in ("inserts", "dist_evals", "sum_new", "sum_old", "proposals"):
            assert st[key] == want[key], (key, st, x.shape, k, p)
    ctx.close()


def test_work_runs_on_the_stream_it_is_given():
    # the context enqueues on the caller's stream (here a side stream of torch's,
    # default priority); the result equals the default-stream one and arrives on
    # that stream - an event recorded on it covers the whole build
    amd = _amd()
    x = W.sift_like_u8(30000, 64, seed=63, n_comp=8)
    xd = _dev(x)
    ids_a, dist_a, ctx_a = amd.gnnd_build(xd, 16, 16, amd.L2SQ_U8, SEED, iters=4)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        ctx_b = amd.Gnnd(xd, 16, 16, amd.L2SQ_U8, SEED)
        assert ctx_b.prm.stream == side.cuda_stream
        ctx_b.build(4, want_stats=False)
        ids_b, dist_b = ctx_b.graph()
        done = torch.cuda.Event()
        done.record(side)
    done.synchronize()
    assert torch.equal(ids_a, ids_b) and torch.equal(dist_a, dist_b)
    ctx_a.close()
    ctx_b.close()


def test_two_contexts_on_two_streams_do_not_disturb_each_other():
    # two builds of different shapes and metrics enqueued in alternation on two streams
    # (default priority), each in its own workspace: both end with the graph a build on
    # its own produces - the library keeps no state outside the context
    amd = _amd()
    xa = _dev(W.sift_like_u8(40000, 64, seed=64, n_comp=8))
    xb = _dev(W.deep_like_f32(30000, 48, seed=65, n_comp=8))
    ref_a = amd.gnnd_build(xa, 16, 16, amd.L2SQ_U8, SEED, iters=5)
    ref_b = amd.gnnd_build(xb, 24, 12, amd.ANGULAR_F32, SEED + 1, iters=5)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    for s in (sa, sb):
        s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(sa):
        ca = amd.Gnnd(xa, 16, 16, amd.L2SQ_U8, SEED)
        ca.init_random()
    with torch.cuda.stream(sb):
        cb = amd.Gnnd(xb, 24, 12, amd.ANGULAR_F32, SEED + 1)
        cb.init_random()
    for _ in range(5):
        with torch.cuda.stream(sa):
            ca.iterate(want_stats=False)
        with torch.cuda.stream(sb):
            cb.iterate(want_stats=False)
    with torch.cuda.stream(sa):
        ga = ca.graph()
    with torch.cuda.stream(sb):
        gb = cb.graph()
    sa.synchronize()
    sb.synchronize()
    assert torch.equal(ga[0], ref_a[0]) and torch.equal(ga[1], ref_a[1])
    assert torch.equal(gb[0], ref_b[0]) and torch.equal(gb[1], ref_b[1])
    for c in (ca, cb, ref_a[2], ref_b[2]):
        c.close()


# ---- segmented lists (Sec. 4.3, "Multiple Spinlocks") ---------------------------------------
SEGMENTED_CASES = {
    # name: (generator, metric, k, p, iters, join path)
    "seg_k64_uniform": (lambda: W.uniform_f32(2000, 12, seed=1091), og.L2SQ_F32, 64, 24, 5, "valu"),
    "seg_k128_sift_mfma": (lambda: W.sift_like_f32(1800, 128, seed=1092, n_comp=8),
                           og.L2SQ_F32, 128, 32, 4, "mfma"),
    "seg_k96_u8": (lambda: W.sift_like_u8(1500, 64, seed=1093, n_comp=6), og.L2SQ_U8, 96, 20, 4,
                   "mfma_direct"),
    "seg_k64_angular_p40": (lambda: W.deep_like_f32(1300, 24, seed=1094, n_comp=8),
                            og.ANGULAR_F32, 64, 40, 4, "valu"),
    # every residue class has 34 members only: the random init runs out of first attempts
    "seg_k128_tiny_classes": (lambda: W.uniform_f32(136, 5, seed=1095), og.L2SQ_F32, 128, 16, 3,
                              "valu"),
    "seg_k32_is_plain": (lambda: W.uniform_f32(900, 8, seed=1096), og.L2SQ_F32, 32, 16, 3, "valu"),
}


@pytest.mark.parametrize("name", list(SEGMENTED_CASES))
def test_segmented_lists_match_oracle_after_every_iteration(name):
    amd = _amd()
    gen, metric, k, p, iters, path = SEGMENTED_CASES[name]
    x = gen()
    join = {"mfma": amd.JOIN_MFMA, "mfma_direct": amd.JOIN_MFMA_DIRECT}.get(path, amd.JOIN_VALU)
    ctx = amd.Gnnd(_dev(x), k, p, metric, SEED, join, list_mode=amd.LISTS_SEGMENTED)
    ctx.init_random()
    g = og.init_random(x, k, metric, SEED, segmented=True)
    _assert_graph_equal(ctx, g, "segmented init")
    m = k // 32
    for it in range(1, iters + 1):
        st = ctx.iterate()
        ref = og.iterate(x, metric, g, p, SEED, it, segmented=True)
        _assert_graph_equal(ctx, g, f"segmented iteration {it}")
        for key in ("inserts", "dist_evals", "sum_new", "sum_old", "proposals"):
            assert st[key] == ref[key], (it, key, st[key], ref[key])
        assert st["dropped"] == 0
    ids, _, _ = _graph_np(ctx)
    assert all(np.bincount(row % m, minlength=m).tolist() == [32] * m for row in ids[::37])
    # a build in one call ends in the same graph
    ctx.build(iters, want_stats=False)
    _assert_graph_equal(ctx, g, "segmented build")
    if k == 32:  # one segment is the plain list
        plain = amd.Gnnd(_dev(x), k, p, metric, SEED, join)
        plain.build(iters, want_stats=False)
        a, b = ctx.graph(), plain.graph()
        assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
        plain.close()
    ctx.close()


def test_segmented_lists_refuse_what_the_paper_does_not_define():
    amd = _amd()
    x = _dev(W.uniform_f32(400, 6, seed=1097))
    with pytest.raises(amd.GnndError):  # k must be a multiple of 32
        amd.Gnnd(x, 48, 16, amd.L2SQ_F32, SEED, list_mode=amd.LISTS_SEGMENTED)
    with pytest.raises(amd.GnndError):  # classes of fewer than 34 members
        amd.Gnnd(x[:100].contiguous(), 96, 16, amd.L2SQ_F32, SEED, list_mode=amd.LISTS_SEGMENTED)
    ctx = amd.Gnnd(x, 64, 16, amd.L2SQ_F32, SEED, list_mode=amd.LISTS_SEGMENTED)
    ctx.build(2, want_stats=False)
    ids, dist, flags = ctx.graph(with_flags=True)
    with pytest.raises(amd.GnndError):  # a loaded graph need not be segmented
        ctx.set_graph(ids, dist, flags, 2)
    ctx.close()
