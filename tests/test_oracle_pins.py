"""Pins of the CPU oracle against things other than itself: published mixer
outputs, exactly rounded arithmetic done with rationals, numpy float64 brute
force, closed special cases, set identities and monotonicity invariants.
CPU only."""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle as og
import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- RNG -------
def test_mixer_matches_published_splitmix64_outputs():
    want = [int(l, 16) for l in open(os.path.join(GOLDEN, "splitmix64_seed0.txt"))
            if l.strip() and not l.startswith("#")]
    state = 0
    for w in want:
        state = (state + 0x9E3779B97F4A7C15) % (1 << 64)
        assert og.mix64(state) == w


def test_hash_counters_all_matter_and_bounded_is_uniform():
    base = og.hash5(42, 1, 5, 6, 7)
    assert base == og.hash5(42, 1, 5, 6, 7)
    others = {og.hash5(43, 1, 5, 6, 7), og.hash5(42, 2, 5, 6, 7), og.hash5(42, 1, 6, 5, 7),
              og.hash5(42, 1, 5, 7, 6), og.hash5(42, 1, 5, 6, 8), og.hash5(42, 1, 6, 6, 7)}
    assert base not in others and len(others) == 6
    n = 10
    counts = np.zeros(n)
    draws = 20000
    for i in range(draws):
        r = og.bounded(og.hash5(7, 1, i, 0, 0), n)
        assert 0 <= r < n
        counts[r] += 1
    chi2 = ((counts - draws / n) ** 2 / (draws / n)).sum()
    assert chi2 < 40.0  # 9 degrees of freedom; far tail
    assert og.bounded((1 << 64) - 1, 1000) == 999 and og.bounded(0, 1000) == 0
    # avalanche: flipping one counter bit flips about half of the output bits
    flips = [bin(og.hash5(1, 2, i, 9, 3) ^ og.hash5(1, 2, i ^ 1, 9, 3)).count("1")
             for i in range(0, 400, 2)]
    assert 28 < np.mean(flips) < 36


# ---------------------------------------------------------- distances -------
def _round_f32(x: Fraction) -> Fraction:
    """Exactly round a rational to the nearest float32 (ties to even), normal range."""
    if x == 0:
        return Fraction(0)
    sign = -1 if x < 0 else 1
    x = abs(x)
    e = 0
    while x >= 2:
        x /= 2
        e += 1
    while x < 1:
        x *= 2
        e -= 1
    scaled = x * (1 << 23)
    fl = scaled.numerator // scaled.denominator
    rem = scaled - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    return sign * Fraction(fl, 1 << 23) * (Fraction(2) ** e)


def _fr(v):
    return Fraction(float(v))


def test_l2_is_float32_fused_in_dimension_order():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((6, 11)).astype(np.float32)
    differs_from_unfused = 0
    for i in range(6):
        for j in range(6):
            acc = Fraction(0)
            unf = np.float32(0)
            for q in range(x.shape[1]):
                diff = _round_f32(_fr(x[i, q]) - _fr(x[j, q]))
                acc = _round_f32(diff * diff + acc)
                dq = np.float32(x[i, q] - x[j, q])
                unf = np.float32(np.float32(dq * dq) + unf)
            got = og.distance(x, og.L2SQ_F32, i, j)
            assert Fraction(got) == acc
            differs_from_unfused += float(unf) != got
            assert got == og.distance(x, og.L2SQ_F32, j, i)
    assert differs_from_unfused > 0  # the test can tell fused from unfused


def test_angular_is_one_minus_float32_fused_dot():
    rng = np.random.default_rng(4)
    x = rng.standard_normal((5, 9)).astype(np.float32)
    x /= np.linalg.norm(x, axis=1, keepdims=True)
    for i in range(5):
        for j in range(5):
            acc = Fraction(0)
            for q in range(x.shape[1]):
                acc = _round_f32(_fr(x[i, q]) * _fr(x[j, q]) + acc)
            want = _round_f32(Fraction(1) - acc)
            assert Fraction(og.distance(x, og.ANGULAR_F32, i, j)) == want


def test_chi_square_is_float32_term_by_term_with_zero_sums_skipped():
    # sum over the dimensions of (a - b)^2 / (a + b), every operation rounded to
    # float32 on its own (exact rational arithmetic with explicit rounding), a
    # dimension where both entries are zero adding nothing; symmetric; zero on
    # equal vectors; close to the float64 value of the textbook formula.
    rng = np.random.default_rng(6)
    x = np.abs(rng.standard_normal((6, 13))).astype(np.float32)
    x[:, 4] = 0.0   # a dimension that is empty everywhere
    x[2, 7] = 0.0
    for i in range(6):
        for j in range(6):
            acc = Fraction(0)
            for q in range(x.shape[1]):
                diff = _round_f32(_fr(x[i, q]) - _fr(x[j, q]))
                tot = _round_f32(_fr(x[i, q]) + _fr(x[j, q]))
                if tot > 0:
                    acc = _round_f32(acc + _round_f32(_round_f32(diff * diff) / tot))
            got = og.distance(x, og.CHI2_F32, i, j)
            assert Fraction(got) == acc
            assert got == og.distance(x, og.CHI2_F32, j, i)
            a, b = x[i].astype(np.float64), x[j].astype(np.float64)
            ok = (a + b) > 0
            ref = (((a - b) ** 2)[ok] / (a + b)[ok]).sum()
            assert abs(got - ref) <= 1e-5 * max(ref, 1e-3)
        assert og.distance(x, og.CHI2_F32, i, i) == 0.0


def _sqrt_f32(p):
    """Correctly rounded float32 square root of the exact rational p >= 0, decided
    by comparing p with the squares of the midpoints between neighbouring floats."""
    if p == 0:
        return Fraction(0)
    c = np.float32(np.sqrt(float(p)))
    for cand in (c, np.nextafter(c, np.float32(0)), np.nextafter(c, np.float32(np.inf))):
        lo = (_fr(np.nextafter(cand, np.float32(-np.inf))) + _fr(cand)) / 2
        hi = (_fr(cand) + _fr(np.nextafter(cand, np.float32(np.inf)))) / 2
        if lo * lo <= p <= hi * hi:
            return _fr(cand)
    raise AssertionError("no float32 neighbour brackets the root")


def test_cosine_distance_is_float32_step_by_step():
    # 1 - a.b / sqrt(|a|^2 |b|^2): inner product and squared norms with one fused
    # multiply-add per dimension in order, then product, root, quotient and
    # difference each rounded to float32 (exact rational arithmetic, explicit
    # rounding, the root bracketed by midpoints); a zero vector is at distance 1.
    rng = np.random.default_rng(8)
    x = (rng.standard_normal((6, 11)) * rng.uniform(0.1, 30.0, size=(6, 1))).astype(np.float32)
    x[5] = 0.0

    def fdot(a, b):
        acc = Fraction(0)
        for q in range(len(a)):
            acc = _round_f32(_fr(a[q]) * _fr(b[q]) + acc)
        return acc

    for i in range(6):
        for j in range(6):
            dot, na, nb = fdot(x[i], x[j]), fdot(x[i], x[i]), fdot(x[j], x[j])
            den = _sqrt_f32(_round_f32(na * nb))
            want = _round_f32(1 - _round_f32(dot / den)) if den > 0 else Fraction(1)
            got = og.distance(x, og.COSINE_F32, i, j)
            assert Fraction(got) == want, (i, j)
            assert got == og.distance(x, og.COSINE_F32, j, i)
            if i < 5 and j < 5:
                a, b = x[i].astype(np.float64), x[j].astype(np.float64)
                assert abs(got - (1 - a @ b / np.sqrt((a @ a) * (b @ b)))) < 3e-7


def test_cosine_distance_ignores_length_and_has_the_textbook_special_cases():
    rng = np.random.default_rng(9)
    x = rng.standard_normal((4, 9)).astype(np.float32)
    base = og.distance(x, og.COSINE_F32, 0, 1)
    for e0, e1 in ((3, 0), (-2, 5), (7, -7), (10, 11)):  # powers of two scale exactly
        y = x.copy()
        y[0] *= np.float32(2.0 ** e0)
        y[1] *= np.float32(2.0 ** e1)
        assert og.distance(y, og.COSINE_F32, 0, 1) == base
    assert abs(og.distance(x, og.COSINE_F32, 2, 2)) < 2e-7
    y = np.stack([x[3], -3 * x[3]]).astype(np.float32)
    assert abs(og.distance(y, og.COSINE_F32, 0, 1) - 2.0) < 3e-7
    z = np.zeros((3, 9), np.float32)
    z[0, 0], z[0, 1] = 3.0, 4.0          # |a| = 5
    z[1, 1] = 5.0                        # |b| = 5, a.b = 20
    z[2, 4] = 7.0                        # orthogonal to both
    assert og.distance(z, og.COSINE_F32, 0, 1) == float(np.float32(1) - np.float32(20) / np.float32(25))
    assert og.distance(z, og.COSINE_F32, 0, 2) == 1.0 and og.distance(z, og.COSINE_F32, 1, 2) == 1.0


def test_u8_distance_is_exact_integer():
    rng = np.random.default_rng(5)
    x = rng.integers(0, 256, size=(8, 37)).astype(np.uint8)
    for i in range(8):
        for j in range(8):
            want = int(((x[i].astype(np.int64) - x[j].astype(np.int64)) ** 2).sum())
            assert og.distance(x, og.L2SQ_U8, i, j) == want


# -------------------------------------------------------- brute force -------
def _numpy_knn(x, metric, K):
    xd = x.astype(np.float64)
    if metric == og.ANGULAR_F32:
        D = 1.0 - xd @ xd.T
    elif metric == og.COSINE_F32:
        nrm = np.sqrt((xd ** 2).sum(1))
        D = 1.0 - (xd @ xd.T) / (nrm[:, None] * nrm[None, :])
    elif metric == og.CHI2_F32:
        tot = xd[:, None, :] + xd[None, :, :]
        D = np.where(tot > 0, (xd[:, None, :] - xd[None, :, :]) ** 2 / np.where(tot > 0, tot, 1),
                     0.0).sum(-1)
    else:
        D = ((xd[:, None, :] - xd[None, :, :]) ** 2).sum(-1)
    n = len(x)
    ids = np.empty((n, K), np.int64)
    for i in range(n):
        order = sorted((D[i, j], j) for j in range(n) if j != i)
        ids[i] = [j for _, j in order[:K]]
    return ids, D


@pytest.mark.parametrize("metric", [og.L2SQ_F32, og.L2SQ_U8])
def test_bruteforce_equals_numpy_full_sort_on_exact_data(metric):
    x = W.small_integer_f32(300, 6, seed=11)  # exact distances, many ties
    if metric == og.L2SQ_U8:
        x = x.astype(np.uint8)
    ids, dist = og.bruteforce(x, metric, np.arange(300), 12)
    want, D = _numpy_knn(x, metric, 12)
    assert (ids == want).all()
    assert (dist == np.take_along_axis(D, want, 1)).all()


def test_bruteforce_angular_close_to_float64():
    x = W.deep_like_f32(200, 24, seed=12, n_comp=8)
    ids, dist = og.bruteforce(x, og.ANGULAR_F32, np.arange(200), 10)
    want, D = _numpy_knn(x, og.ANGULAR_F32, 10)
    ref = np.take_along_axis(D, ids.astype(np.int64), 1)
    assert np.abs(dist - ref).max() < 1e-6
    assert (ids == want).mean() > 0.99  # only float32 near-ties may differ


def test_bruteforce_chi_square_close_to_float64_and_build_converges():
    x = W.gist_like_f32(300, 20, seed=14, n_comp=6)
    ids, dist = og.bruteforce(x, og.CHI2_F32, np.arange(300), 10)
    want, D = _numpy_knn(x, og.CHI2_F32, 10)
    ref = np.take_along_axis(D, ids.astype(np.int64), 1)
    assert np.abs(dist - ref).max() < 1e-6
    assert (ids == want).mean() > 0.99  # only float32 near-ties may differ
    g, _ = og.build(x, 16, 16, og.CHI2_F32, 7, 8)
    rec, _ = og.recall_at(g.ids, g.dist, ids, dist, 10)
    assert rec > 0.97
    _check_lists(g, x, og.CHI2_F32)


def test_bruteforce_cosine_close_to_float64_and_build_converges():
    # vectors of very different lengths: the ranking is that of the angles
    x = W.deep_like_f32(300, 24, seed=15, n_comp=6)
    x = (x * np.random.default_rng(15).uniform(0.05, 40.0, size=(300, 1))).astype(np.float32)
    ids, dist = og.bruteforce(x, og.COSINE_F32, np.arange(300), 10)
    want, D = _numpy_knn(x, og.COSINE_F32, 10)
    ref = np.take_along_axis(D, ids.astype(np.int64), 1)
    assert np.abs(dist - ref).max() < 1e-6
    assert (ids == want).mean() > 0.99  # only float32 near-ties may differ
    unit = (x / np.linalg.norm(x.astype(np.float64), axis=1, keepdims=True)).astype(np.float32)
    ids_unit, _ = og.bruteforce(unit, og.ANGULAR_F32, np.arange(300), 10)
    assert (ids == ids_unit).mean() > 0.98
    g, _ = og.build(x, 16, 16, og.COSINE_F32, 7, 8)
    rec, _ = og.recall_at(g.ids, g.dist, ids, dist, 10)
    assert rec > 0.97
    _check_lists(g, x, og.COSINE_F32)


def test_bruteforce_points_on_a_line():
    # 1-d points at distinct integer positions: the K nearest are the K closest
    # positions in sorted order.
    rng = np.random.default_rng(13)
    pos = rng.permutation(500)[:64].astype(np.float32)
    x = pos[:, None].copy()
    ids, dist = og.bruteforce(x, og.L2SQ_F32, np.arange(64), 4)
    for i in range(64):
        want = sorted(((pos[j] - pos[i]) ** 2, j) for j in range(64) if j != i)[:4]
        assert [j for _, j in want] == list(ids[i])


# ------------------------------------------------------------ init ----------
def _check_lists(g, x, metric, expect_all_new=None):
    n, k = g.ids.shape
    for s in range(n):
        row = g.ids[s]
        assert len(set(row.tolist())) == k and s not in row and row.min() >= 0 and row.max() < n
        keys = list(zip(g.dist[s].tolist(), row.tolist()))
        assert keys == sorted(keys)
    if expect_all_new is not None:
        assert (g.isnew == expect_all_new).all()


def test_init_invariants_and_stored_distances():
    x = W.uniform_f32(200, 8, seed=21)
    g = og.init_random(x, 12, og.L2SQ_F32, 5)
    _check_lists(g, x, og.L2SQ_F32, expect_all_new=1)
    for s in range(0, 200, 17):
        for j in range(12):
            assert g.dist[s, j] == og.distance(x, og.L2SQ_F32, s, int(g.ids[s, j]))
    g2 = og.init_random(x, 12, og.L2SQ_F32, 6)
    assert (g2.ids != g.ids).mean() > 0.5  # the seed matters
    # ids look uniformly drawn: mean in-degree equals k, no node dominates
    indeg = np.bincount(g.ids.ravel(), minlength=200)
    assert indeg.sum() == 200 * 12 and indeg.max() < 40


@pytest.mark.parametrize("metric", [og.L2SQ_F32, og.ANGULAR_F32, og.L2SQ_U8])
def test_init_with_k_equal_n_minus_1_is_the_exact_graph(metric):
    n = 24
    if metric == og.L2SQ_U8:
        x = W.sift_like_u8(n, 10, seed=22, n_comp=3)
    elif metric == og.ANGULAR_F32:
        x = W.deep_like_f32(n, 10, seed=22, n_comp=3)
    else:
        x = W.uniform_f32(n, 10, seed=22)
    g = og.init_random(x, n - 1, metric, 9)
    ids, dist = og.bruteforce(x, metric, np.arange(n), n - 1)
    assert (g.ids == ids).all() and (g.dist == dist).all()


# ------------------------------------------------------- Eq. 1-2 map --------
def test_pair_map_enumerates_the_strict_lower_triangle_once():
    seen = {}
    for t in range(64 * 63 // 2):
        u, v = og.pair_of(t)
        assert 0 <= v < u <= 63 and u * (u - 1) // 2 + v == t
        seen[(u, v)] = t
    assert len(seen) == 2016
    assert og.pair_of(0) == (1, 0) and og.pair_of(1) == (2, 0) and og.pair_of(2) == (2, 1)


# ---------------------------------------------------------- sampling --------
def _forward(ids_row, flags_row, p):
    new = [int(v) for v, f in zip(ids_row, flags_row) if f][:p]
    old = [int(v) for v, f in zip(ids_row, flags_row) if not f][:p]
    return new, old


def _check_sampling(g_before, g_after, p, seed, it, snew, cnew, sold, cold):
    n, k = g_before.ids.shape
    fwd_new, fwd_old = [], []
    for s in range(n):
        a, b = _forward(g_before.ids[s], g_before.isnew[s], p)
        fwd_new.append(a)
        fwd_old.append(b)
        # flags: exactly the sampled NEW entries were cleared
        for j in range(k):
            was = g_before.isnew[s, j]
            now = g_after.isnew[s, j]
            sampled = was and int(g_before.ids[s, j]) in a
            assert now == (1 if (was and not sampled) else 0)
    for kind, fwd, lists, cnts, tag in (("new", fwd_new, snew, cnew, og.TAG_REV_NEW),
                                        ("old", fwd_old, sold, cold, og.TAG_REV_OLD)):
        cands = [[] for _ in range(n)]
        for s in range(n):
            for v in fwd[s]:
                cands[v].append(s)
        for v in range(n):
            got = lists[v, :cnts[v]].tolist()
            assert got == sorted(set(got)) and len(got) <= 2 * p and v not in got
            assert (lists[v, cnts[v]:] == -1).all()
            room = 2 * p - len(fwd[v])
            ranked = sorted(cands[v], key=lambda s: (og.hash5(seed, tag, v, s, it) >> 32, s))
            want = sorted(set(fwd[v]) | set(ranked[:room]))
            assert got == want, (kind, v)
            if len(cands[v]) <= room:  # everything fits: the full reverse list is present
                assert set(cands[v]) <= set(got)


def test_sampling_definition_first_and_later_iterations():
    x = W.uniform_f32(300, 6, seed=31)
    k, p, seed = 10, 4, 77
    g = og.init_random(x, k, og.L2SQ_F32, seed)
    for it in range(1, 4):
        before = g.copy()
        snew, cnew, sold, cold = og.sample(g, p, seed, it)
        if it == 1:
            assert cold.sum() == 0  # first iteration: every entry is NEW
        _check_sampling(before, g, p, seed, it, snew, cnew, sold, cold)
        pu, pv, pd, pcnt, _ = og.join(x, og.L2SQ_F32, p, snew, cnew, sold, cold)
        og.update(g, p, pu, pv, pd, pcnt)
    assert (cnew == 2 * p).any()  # the cap was active somewhere


def test_sampling_without_cap_gives_full_reverse_lists():
    # 2p - k >= n - 1: nothing can overflow, so each list is forward + all reverse.
    x = W.uniform_f32(20, 4, seed=32)
    k, p = 4, 12
    g = og.init_random(x, k, og.L2SQ_F32, 1)
    before = g.copy()
    snew, cnew, sold, cold = og.sample(g, p, 1, 1)
    for v in range(20):
        want = set(before.ids[v].tolist()) | {s for s in range(20) if v in before.ids[s]}
        assert set(snew[v, :cnew[v]].tolist()) == want
    assert (g.isnew == 0).all()


# -------------------------------------------------------------- join --------
def _python_join(x64, dist_fn, N, O, split):
    """Proposals of one node from the definition, distances via dist_fn."""
    props = []
    for u in N:
        if split < 0:
            c = sorted((dist_fn(u, v), v) for v in N if v != u)
            if c:
                props.append((u, c[0][1], c[0][0]))
        c = sorted((dist_fn(u, v), v) for v in O
                   if v != u and (split < 0 or (u < split) != (v < split)))
        if c:
            props.append((u, c[0][1], c[0][0]))
    for u in O:
        c = sorted((dist_fn(u, v), v) for v in N
                   if v != u and (split < 0 or (u < split) != (v < split)))
        if c:
            props.append((u, c[0][1], c[0][0]))
    return props


@pytest.mark.parametrize("split", [-1, 60])
def test_join_against_python_brute_force(split):
    x = W.small_integer_f32(120, 5, seed=41, hi=8)  # exact arithmetic, many ties
    x64 = x.astype(np.float64)
    k, p, seed = 8, 4, 3
    g = og.init_random(x, k, og.L2SQ_F32, seed)
    dist_fn = lambda a, b: float(((x64[a] - x64[b]) ** 2).sum())
    for it in range(1, 4):
        snew, cnew, sold, cold = og.sample(g, p, seed, it)
        pu, pv, pd, pcnt, evals = og.join(x, og.L2SQ_F32, p, snew, cnew, sold, cold, split)
        want_evals = 0
        for s in range(120):
            N = snew[s, :cnew[s]].tolist()
            O = sold[s, :cold[s]].tolist()
            want = _python_join(x64, dist_fn, N, O, split)
            got = list(zip(pu[s, :pcnt[s]].tolist(), pv[s, :pcnt[s]].tolist(),
                           pd[s, :pcnt[s]].tolist()))
            assert sorted(got) == sorted(want), (it, s)
            assert len(got) <= 6 * p
            if split < 0:
                want_evals += len(N) * (len(N) - 1) // 2
                want_evals += sum(1 for a in N for b in O if a != b)
            else:
                want_evals += sum(1 for a in N for b in O
                                  if a != b and (a < split) != (b < split))
        assert evals == want_evals
        og.update(g, p, pu, pv, pd, pcnt)


def test_join_skips_an_object_sampled_as_both_new_and_old():
    x = W.small_integer_f32(6, 3, seed=42)
    p = 2
    snew = np.full((6, 4), -1, np.int32)
    sold = np.full((6, 4), -1, np.int32)
    cnew = np.zeros(6, np.int32)
    cold = np.zeros(6, np.int32)
    snew[0, :2] = [1, 2]
    sold[0, :2] = [2, 3]
    cnew[0], cold[0] = 2, 2
    pu, pv, pd, pcnt, evals = og.join(x, og.L2SQ_F32, p, snew, cnew, sold, cold)
    assert evals == 1 + 3  # (1,2) and (1,2),(1,3),(2,3); the pair (2,2) is skipped
    props = set(zip(pu[0, :pcnt[0]].tolist(), pv[0, :pcnt[0]].tolist()))
    assert all(u != v for u, v in props)


# ------------------------------------------------------------ update --------
def test_update_is_order_independent_and_equals_sorted_union():
    x = W.small_integer_f32(150, 4, seed=51, hi=6)
    k, p, seed = 6, 3, 8
    g = og.init_random(x, k, og.L2SQ_F32, seed)
    rng = np.random.default_rng(0)
    for it in range(1, 4):
        snew, cnew, sold, cold = og.sample(g, p, seed, it)
        pu, pv, pd, pcnt, _ = og.join(x, og.L2SQ_F32, p, snew, cnew, sold, cold)
        before = g.copy()
        props = [(int(pu[s, j]), int(pv[s, j]), float(pd[s, j]))
                 for s in range(150) for j in range(pcnt[s])]
        inserts = og.update(g, p, pu, pv, pd, pcnt)
        # (a) definition: sort the union, one entry per id, truncate
        total_new = 0
        for u in range(150):
            pool = {int(i): (float(d), int(f)) for i, d, f in
                    zip(before.ids[u], before.dist[u], before.isnew[u])}
            for (uu, v, d) in props:
                if uu == u and v not in pool:
                    pool[v] = (d, 1)
            top = sorted((d, v, f) for v, (d, f) in pool.items())[:k]
            assert [v for _, v, _ in top] == g.ids[u].tolist()
            assert [d for d, _, _ in top] == g.dist[u].tolist()
            assert [f for _, _, f in top] == g.isnew[u].tolist()
            total_new += len(set(g.ids[u].tolist()) - set(before.ids[u].tolist()))
        assert inserts == total_new
        # (b) one-at-a-time insertion in random orders gives the same lists
        for _ in range(3):
            h = before.copy()
            for idx in rng.permutation(len(props)):
                u, v, d = props[idx]
                og.insert_one(h.ids[u], h.dist[u], h.isnew[u], v, d)
            assert (h.ids == g.ids).all() and (h.dist == g.dist).all()
            assert (h.isnew == g.isnew).all()


# ---------------------------------------------------- whole iterations ------
@pytest.mark.parametrize("metric", [og.L2SQ_F32, og.ANGULAR_F32, og.L2SQ_U8])
def test_iterations_improve_monotonically_and_keep_invariants(metric):
    n, k, p, seed = 500, 10, 6, 42
    if metric == og.L2SQ_U8:
        x = W.sift_like_u8(n, 16, seed=61, n_comp=8)
    elif metric == og.ANGULAR_F32:
        x = W.deep_like_f32(n, 16, seed=61, n_comp=8)
    else:
        x = W.uniform_f32(n, 16, seed=61)
    g = og.init_random(x, k, metric, seed)
    phi = og.phi(g.dist)
    for it in range(1, 7):
        before = g.copy()
        st = og.iterate(x, metric, g, p, seed, it)
        _check_lists(g, x, metric)
        assert (g.dist <= before.dist).all()  # every rank of every list
        new_phi = og.phi(g.dist)
        assert new_phi <= phi
        phi = new_phi
        # flag bookkeeping: NEW entries = unsampled NEW left over + admitted entries
        left = 0
        for s in range(n):
            left += max(0, int(before.isnew[s].sum()) - p)
        assert int(g.isnew.sum()) <= left + st["inserts"]
        if p >= k:
            assert int(g.isnew.sum()) <= st["inserts"]
        for s in range(0, n, 37):
            for j in range(k):
                assert g.dist[s, j] == og.distance(x, metric, s, int(g.ids[s, j]))
    assert st["inserts"] < n  # it converges


def test_tiny_build_reaches_the_exact_graph():
    x = W.uniform_f32(256, 8, seed=62)
    g, stats = og.build(x, 32, 32, og.L2SQ_F32, 42, 12)
    ids, dist = og.bruteforce(x, og.L2SQ_F32, np.arange(256), 10)
    tol, strict = og.recall_at(g.ids, g.dist, ids, dist, 10)
    assert tol == 1.0 and strict == 1.0


def test_recall_formula_on_a_hand_made_case():
    # two nodes, K = 2: node 0 lists both true neighbours, node 1 lists one.
    truth_ids = np.array([[1, 2], [0, 2]])
    truth_dist = np.array([[1.0, 2.0], [1.0, 3.0]])
    g_ids = np.array([[2, 1], [0, 3]])
    g_dist = np.array([[2.0, 1.0], [1.0, 4.0]])
    tol, strict = og.recall_at(g_ids, g_dist, truth_ids, truth_dist, 2)
    assert tol == 0.75 and strict == 0.75
    # a different id at the same distance as the K-th counts for the tolerant form only
    g_ids2 = np.array([[1, 5], [0, 2]])
    g_dist2 = np.array([[1.0, 2.0], [1.0, 3.0]])
    tol, strict = og.recall_at(g_ids2, g_dist2, truth_ids, truth_dist, 2)
    assert tol == 1.0 and strict == 0.75
    assert og.phi(g_dist) == 8.0


# ------------------------------------------------------------- merge --------
def _exact_graph(x, metric, k, base=0):
    """Exact k-NN graph of x; ids shifted to the collection range [base, base + n)."""
    ids, dist = og.bruteforce(x, metric, np.arange(len(x)), k)
    return og.Graph(ids + base, dist, np.zeros_like(ids, dtype=np.uint8))


def test_merge_final_is_top_k_of_union_with_the_set_aside_half():
    k, n1, n2 = 9, 40, 30
    x = W.uniform_f32(n1 + n2, 6, seed=72)
    g1 = _exact_graph(x[:n1], og.L2SQ_F32, k)
    g2 = _exact_graph(x[n1:], og.L2SQ_F32, k, base=n1)
    g, aside_ids, aside_dist = og.merge_init(x, n1, k, og.L2SQ_F32, 4, g1, g2)
    og.iterate(x, og.L2SQ_F32, g, k, 4, 1, split=n1)
    before = g.copy()
    og.merge_final(g, aside_ids, aside_dist)
    for s in range(n1 + n2):
        pool = dict(zip(before.ids[s].tolist(), before.dist[s].tolist()))
        for v, d in zip(aside_ids[s].tolist(), aside_dist[s].tolist()):
            pool.setdefault(v, d)
        top = sorted((d, v) for v, d in pool.items())[:k]
        assert [v for _, v in top] == g.ids[s].tolist()
        assert [d for d, _ in top] == g.dist[s].tolist()


def test_merge_with_no_iterations_keeps_each_input_list():
    # Zero refinement rounds: top-k of (kept half + random fill + set-aside
    # half) can only be as good as or better than the input list, rank by rank,
    # and it contains the whole input list unless a fill object displaced a tail.
    k, n1, n2 = 8, 30, 25
    x = W.uniform_f32(n1 + n2, 5, seed=76)
    g1 = _exact_graph(x[:n1], og.L2SQ_F32, k)
    g2 = _exact_graph(x[n1:], og.L2SQ_F32, k, base=n1)
    g, _ = og.merge(x, n1, k, k, og.L2SQ_F32, 5, g1, g2, 0)
    assert (g.dist[:n1] <= g1.dist).all() and (g.dist[n1:] <= g2.dist).all()
    for s in range(n1):
        own = [v for v in g.ids[s].tolist() if v < n1]
        assert own == g1.ids[s, :len(own)].tolist()


def test_merge_init_structure():
    k, n1, n2, seed = 9, 40, 30, 4
    x = W.uniform_f32(n1 + n2, 6, seed=73)
    g1 = _exact_graph(x[:n1], og.L2SQ_F32, k)
    g2 = _exact_graph(x[n1:], og.L2SQ_F32, k, base=n1)
    g, aside_ids, aside_dist = og.merge_init(x, n1, k, og.L2SQ_F32, seed, g1, g2)
    keep, fill = 5, 4
    for s in range(n1 + n2):
        first = s < n1
        src = g1 if first else g2
        loc = s if first else s - n1
        shift = 0  # the input lists already carry the ids of the union
        kept = (src.ids[loc, :keep] + shift).tolist()
        aside = (src.ids[loc, keep:] + shift).tolist()
        assert aside_ids[s].tolist() == aside and (aside_dist[s] == src.dist[loc, keep:]).all()
        row = g.ids[s].tolist()
        assert len(set(row)) == k
        old = [v for v, f in zip(row, g.isnew[s]) if not f]
        new = [v for v, f in zip(row, g.isnew[s]) if f]
        assert sorted(old) == sorted(kept) and len(new) == fill
        for v in new:  # random objects of the other subset
            assert (v >= n1) if first else (v < n1)
        keys = list(zip(g.dist[s].tolist(), row))
        assert keys == sorted(keys)
        for j in range(k):
            assert g.dist[s, j] == og.distance(x, og.L2SQ_F32, s, row[j])
    # fills differ between nodes (they are random) and with the seed
    g_b, _, _ = og.merge_init(x, n1, k, og.L2SQ_F32, seed + 1, g1, g2)
    assert (g_b.ids != g.ids).any()


def test_merge_of_exact_subgraphs_recovers_the_exact_graph_and_never_worsens():
    k, p, n1, n2 = 10, 10, 150, 130
    x = W.uniform_f32(n1 + n2, 6, seed=74)
    g1 = _exact_graph(x[:n1], og.L2SQ_F32, k)
    g2 = _exact_graph(x[n1:], og.L2SQ_F32, k, base=n1)
    g, stats = og.merge(x, n1, k, p, og.L2SQ_F32, 11, g1, g2, 6)
    n = n1 + n2
    _check_lists(g, x, og.L2SQ_F32)
    # per rank never worse than the input list of the node
    assert (g.dist[:n1] <= g1.dist).all() and (g.dist[n1:] <= g2.dist).all()
    ids, dist = og.bruteforce(x, og.L2SQ_F32, np.arange(n), k)
    tol, strict = og.recall_at(g.ids, g.dist, ids, dist, k)
    g0, _ = og.merge(x, n1, k, p, og.L2SQ_F32, 11, g1, g2, 0)
    tol0, _ = og.recall_at(g0.ids, g0.dist, ids, dist, k)
    assert tol > 0.95 and tol > tol0 + 0.2  # the refinement rounds do the work
    # only cross-subset pairs were evaluated: far fewer than a raw build needs
    _, raw_stats = og.build(x, k, p, og.L2SQ_F32, 11, 6)
    assert sum(s["dist_evals"] for s in stats) < sum(s["dist_evals"] for s in raw_stats)


def test_merge_join_only_proposes_cross_subset_pairs():
    k, p, n1, n2 = 8, 8, 50, 40
    x = W.uniform_f32(n1 + n2, 5, seed=75)
    g1 = _exact_graph(x[:n1], og.L2SQ_F32, k)
    g2 = _exact_graph(x[n1:], og.L2SQ_F32, k, base=n1)
    g, aside_ids, aside_dist = og.merge_init(x, n1, k, og.L2SQ_F32, 3, g1, g2)
    for it in range(1, 4):
        snew, cnew, sold, cold = og.sample(g, p, 3, it)
        # NEW entries of a node always lie in the other subset
        for s in range(n1 + n2):
            for v in snew[s, :cnew[s]]:
                assert (v < n1) != (s < n1)
        pu, pv, pd, pcnt, _ = og.join(x, og.L2SQ_F32, p, snew, cnew, sold, cold, split=n1)
        for s in range(n1 + n2):
            for j in range(pcnt[s]):
                assert (pu[s, j] < n1) != (pv[s, j] < n1)
        og.update(g, p, pu, pv, pd, pcnt)


# ------------------------------------------------- shards and frozen entries -
def test_merge_keeps_third_shard_entries_frozen():
    # Three shards A, B, C of one collection.  After merging (A, B), A's lists
    # hold ids of B; in the merge (A, C) those entries are frozen: they stay in
    # place by their stored distance unless something closer displaces them, and
    # no join ever involves them.
    k, p, m = 8, 8, 60
    x = W.uniform_f32(3 * m, 5, seed=81)
    A, B, Cc = (slice(0, m), slice(m, 2 * m), slice(2 * m, 3 * m))
    gA = _exact_graph(x[A], og.L2SQ_F32, k, base=0)
    gB = _exact_graph(x[B], og.L2SQ_F32, k, base=m)
    gC = _exact_graph(x[Cc], og.L2SQ_F32, k, base=2 * m)
    gAB, _ = og.merge(np.concatenate([x[A], x[B]]), m, k, p, og.L2SQ_F32, 7, gA, gB, 4, 0, m)
    gA2 = og.Graph(gAB.ids[:m].copy(), gAB.dist[:m].copy(), None)
    assert (gA2.ids >= m).any()  # A's lists now point into B
    xAC = np.concatenate([x[A], x[Cc]])
    g, aside_ids, aside_dist = og.merge_init(xAC, m, k, og.L2SQ_F32, 9, gA2, gC, 0, 2 * m)
    n = 2 * m
    frozen_before = {s: {int(v) for v in np.concatenate([g.ids[s], aside_ids[s]]) if v >= n}
                     for s in range(n)}
    assert any(frozen_before.values())
    for it in range(1, 4):
        st = og.iterate(xAC, og.L2SQ_F32, g, p, 9, it, split=m)
        for arr in (st["snew"], st["sold"]):
            assert arr.max() < n  # frozen entries are never sampled
    og.merge_final(g, aside_ids, aside_dist)
    for s in range(n):  # a frozen entry only leaves when k closer entries exist
        now = {int(v) for v in g.ids[s] if v >= n}
        assert now <= frozen_before[s]
        kth = g.dist[s, -1]
        pool = dict(zip(np.concatenate([aside_ids[s]]).tolist(), aside_dist[s].tolist()))
        for v in frozen_before[s] - now:
            if v in pool:
                assert pool[v] >= kth
    # full merge in collection ids: sorted by (distance, id), true distances, better than before
    out, _ = og.merge(xAC, m, k, p, og.L2SQ_F32, 9, gA2, gC, 3, 0, 2 * m)
    for s in range(n):
        keys = list(zip(out.dist[s].tolist(), out.ids[s].tolist()))
        assert keys == sorted(keys) and len(set(out.ids[s].tolist())) == k
        g_s = s if s < m else s + m  # collection id of row s
        for v, dd in zip(out.ids[s], out.dist[s]):
            assert dd == og.distance(x, og.L2SQ_F32, g_s, int(v))
    assert (out.dist[:m] <= gA2.dist).all() and (out.dist[m:] <= gC.dist).all()


def test_renumbering_round_trip():
    lib = og.gnnd_oracle._load()
    n1, b1, n2, b2 = 5, 40, 7, 10
    seen = set()
    for gid in range(0, 60):
        i = lib.og_to_internal(gid, n1, b1, n2, b2)
        assert lib.og_to_global(i, n1, b1, n2, b2) == gid
        assert (i < n1) == (b1 <= gid < b1 + n1)
        assert (n1 <= i < n1 + n2) == (b2 <= gid < b2 + n2)
        seen.add(i)
    assert len(seen) == 60


def test_merge_closed_case_small_second_set_gives_the_exact_lists():
    # Closed case of Alg. 3: with n2 = floor(k/2) objects in S2 the random fill of
    # every S1 list holds ALL of S2 (floor(k/2) distinct draws out of floor(k/2)
    # objects), and the kept + set-aside halves hold all of the exact list G1.  So
    # whatever the iterations do, "Merge and Sort" must return, for every S1 node,
    # its exact k nearest neighbours in S1 u S2 - ids and distances, ties by id.
    # S2's own lists cannot hold k objects of S2; they carry entries of a third
    # shard instead (ids outside both ranges), which are frozen and far away.
    for k, n1, seed in ((10, 60, 5), (7, 33, 6), (4, 19, 7)):
        n2 = k // 2
        x = W.small_integer_f32(n1 + n2, 5, seed=seed, hi=6)  # many equal distances
        ids1, dist1 = og.bruteforce(np.ascontiguousarray(x[:n1]), og.L2SQ_F32, np.arange(n1), k)
        g1 = og.Graph(ids1, dist1, None)
        third = (n1 + n2 + 100 + np.arange(k, dtype=np.int32))[None, :].repeat(n2, 0)
        g2 = og.Graph(np.ascontiguousarray(third), np.full((n2, k), 1e6) + np.arange(k), None)
        want_ids, want_dist = og.bruteforce(x, og.L2SQ_F32, np.arange(n1), k)
        for iters in (0, 1, 3):
            out, _ = og.merge(x, n1, k, max(1, k // 2), og.L2SQ_F32, 40 + seed, g1, g2, iters)
            assert (out.ids[:n1] == want_ids).all(), (k, iters)
            assert (out.dist[:n1] == want_dist).all(), (k, iters)
        # with iterations the S2 rows shed the far third-shard entries for true ones
        assert (out.ids[n1:] < n1 + n2).any()
        for s in range(n1, n1 + n2):
            for v, dd in zip(out.ids[s], out.dist[s]):
                if v < n1 + n2:
                    assert dd == og.distance(x, og.L2SQ_F32, s, int(v))


def test_sharded_build_covers_the_whole_collection():
    # Sec. 5.1: "any two sub-graphs has been merged once".  What holds for any order
    # of the merges is pinned exactly: every pair once; a stored-back sub-graph is
    # never worse than it was, rank by rank (Alg. 3 ends with the best k of the
    # refined list and the set-aside half, and the refined list only improves);
    # rows sorted by (distance, id) with true distances; the lists reach into the
    # other shards.  The recall the scheme reaches is an empirical figure of the
    # method, not a law: on this input (1200 uniform 6-d points, 4 shards, k = p =
    # 10, 6 build + 6 merge iterations, seeds 42..44) the round-robin order the
    # driver uses gives 0.896..0.900, the lexicographic order 0.922..0.927, an
    # unsharded build of 12 iterations 0.955; more merge iterations do not close
    # the gap (0.90 / 0.93 at 20).  The floor below only guards against a broken
    # driver (a skipped pair costs > 0.1); the two orders must stay close.
    n, shards, k, p = 1200, 4, 10, 10
    x = W.uniform_f32(n, 6, seed=82)
    size = n // shards
    seen = []

    def never_worse(m, i, j, before_i, before_j, after_i, after_j):
        seen.append((i, j))
        assert (after_i.dist <= before_i.dist).all() and (after_j.dist <= before_j.dist).all()
        # a pair meets once: before its merge neither sub-graph points into the other shard
        assert not ((before_i.ids // size) == j).any() and not ((before_j.ids // size) == i).any()

    g = og.build_sharded(x, shards, k, p, og.L2SQ_F32, 42, 6, 6, after_merge=never_worse)
    assert sorted(seen) == [(i, j) for i in range(shards) for j in range(i + 1, shards)]
    assert seen == og.pair_schedule(shards)
    ids, dist = og.bruteforce(x, og.L2SQ_F32, np.arange(n), k)
    tol, _ = og.recall_at(g.ids, g.dist, ids, dist, k)
    lex = [(i, j) for i in range(shards) for j in range(i + 1, shards)]
    g_lex = og.build_sharded(x, shards, k, p, og.L2SQ_F32, 42, 6, 6, schedule=lex)
    tol_lex, _ = og.recall_at(g_lex.ids, g_lex.dist, ids, dist, k)
    assert tol > 0.85 and tol_lex > 0.85 and abs(tol - tol_lex) < 0.05, (tol, tol_lex)
    assert sorted(og.pair_schedule(5)) == [(i, j) for i in range(5) for j in range(i + 1, 5)]
    assert sorted(og.pair_schedule(4)) == [(i, j) for i in range(4) for j in range(i + 1, 4)]
    for s in range(0, n, 13):
        keys = list(zip(g.dist[s].tolist(), g.ids[s].tolist()))
        assert keys == sorted(keys) and s not in g.ids[s]
        for v, dd in zip(g.ids[s], g.dist[s]):
            assert dd == og.distance(x, og.L2SQ_F32, s, int(v))
    # every shard's lists reach into the other shards
    own = (g.ids // (n // shards)) == (np.arange(n)[:, None] // (n // shards))
    assert 0.1 < own.mean() < 0.6


def test_append_is_a_sub_build_followed_by_a_merge_and_lifts_recall():
    # Incremental construction (Sec. 5.1): the batch's sub-graph is built on the
    # batch alone, with ids of its own, and only then joined to the resident
    # graph.  Pins: (a) the result equals the two documented steps done by hand;
    # (b) rows of the resident collection can only improve, rank by rank;
    # (c) the appended graph is close to the exact graph of the union and far
    # better than the two separate graphs are for the union.
    k, p, n1, n2, seed = 10, 10, 160, 120, 21
    x = W.uniform_f32(n1 + n2, 6, seed=75)
    g1 = _exact_graph(x[:n1], og.L2SQ_F32, k)
    g = og.append(x, n1, g1, k, p, og.L2SQ_F32, seed, 6, 6)
    sub, _ = og.build(np.ascontiguousarray(x[n1:]), k, p, og.L2SQ_F32, seed + 1, 6)
    assert sub.ids.min() >= 0 and sub.ids.max() < n2  # built on the batch alone
    by_hand, _ = og.merge(x, n1, k, p, og.L2SQ_F32, seed,
                          g1, og.Graph(sub.ids + np.int32(n1), sub.dist, sub.isnew), 6)
    assert (g.ids == by_hand.ids).all() and (g.dist == by_hand.dist).all()
    assert (g.dist[:n1] <= g1.dist).all()
    q = np.arange(n1 + n2, dtype=np.int32)
    ti, td = og.bruteforce(x, og.L2SQ_F32, q, k)
    rec, _ = og.recall_at(g.ids, g.dist, ti, td, 10)
    apart = np.concatenate([g1.ids, sub.ids + np.int32(n1)])
    apart_d = np.concatenate([g1.dist, sub.dist])
    rec0, _ = og.recall_at(apart, apart_d, ti, td, 10)
    assert rec > 0.95 and rec0 < 0.8, (rec, rec0)
    for s in range(n1 + n2):  # well formed lists in the ids of the union
        row = g.ids[s].tolist()
        assert len(set(row)) == k and s not in row and 0 <= min(row) and max(row) < n1 + n2


def test_all_pairs_join_proposes_every_evaluated_pair_both_ways():
    # The variant without the selective update (ablation of Sec. 6.2): same pairs
    # evaluated, each proposed to both of its objects.  Pins: the count identity
    # proposals = 2 x evaluations; every proposal carries the true distance and
    # has its mirror image; the selective join's results are exactly the
    # per-(node, destination, partner kind) minima of this set.
    k, p, seed = 8, 5, 9
    x = W.uniform_f32(300, 6, seed=81)
    g = og.init_random(x, k, og.L2SQ_F32, seed)
    og.iterate(x, og.L2SQ_F32, g, p, seed, 1)
    snew, cnew, sold, cold = og.sample(g, p, seed, 2)
    pu, pv, pd, pcnt, ev = og.join(x, og.L2SQ_F32, p, snew, cnew, sold, cold)
    au, av, ad, acnt, aev = og.join(x, og.L2SQ_F32, p, snew, cnew, sold, cold, all_pairs=True)
    assert aev == ev and int(acnt.sum()) == 2 * ev
    for s in range(300):
        every = [(int(au[s, j]), int(av[s, j]), float(ad[s, j])) for j in range(acnt[s])]
        # (an object sampled both as NEW and as OLD meets a NEW partner twice, so
        # the same proposal can occur twice: compare as sets)
        for u, v, dd in every:
            assert dd == og.distance(x, og.L2SQ_F32, u, v) and (v, u, dd) in set(every)
        news = set(snew[s, :cnew[s]].tolist())
        olds = set(sold[s, :cold[s]].tolist())
        # nearest partner of u among the NEW (resp. OLD) samples, by (distance, id)
        want = set()
        for u in news | olds:
            mine = [(dd, v) for uu, v, dd in every if uu == u]
            if u in news:
                for pool in (news, olds):
                    cand = [(dd, v) for dd, v in mine if v in pool and v != u]
                    # NEW x NEW and NEW x OLD only: a pair of two OLD samples is never evaluated
                    if cand:
                        dd, v = min(cand)
                        want.add((u, v, dd))
            if u in olds:
                cand = [(dd, v) for dd, v in mine if v in news and v != u]
                if cand:
                    dd, v = min(cand)
                    want.add((u, v, dd))
        got = set((int(pu[s, j]), int(pv[s, j]), float(pd[s, j])) for j in range(pcnt[s]))
        assert got == want, s


def test_all_pairs_build_is_at_least_as_good_per_iteration_and_costs_more_proposals():
    k, p, seed = 10, 8, 42
    x = W.uniform_f32(600, 8, seed=3)
    g_sel, st_sel = og.build(x, k, p, og.L2SQ_F32, seed, 5)
    g_all, st_all = og.build(x, k, p, og.L2SQ_F32, seed, 5, all_pairs=True)
    ti, td = og.bruteforce(x, og.L2SQ_F32, np.arange(600, dtype=np.int32), k)
    r_sel, _ = og.recall_at(g_sel.ids, g_sel.dist, ti, td, 10)
    r_all, _ = og.recall_at(g_all.ids, g_all.dist, ti, td, 10)
    assert r_all >= r_sel and r_all > 0.97
    assert st_all[0]["proposals"] > 5 * st_sel[0]["proposals"]
    # the first iteration sees the same samples, hence the same evaluations
    assert st_all[0]["dist_evals"] == st_sel[0]["dist_evals"]
    _check_lists(g_all, x, og.L2SQ_F32)


def test_phi_trend_of_gnnd_overlaps_classic_nn_descent():
    # The paper's own check of the selective update (Sec. 4.3, the phi(G) figure):
    # the sum of all list distances falls along the same curve as under classic
    # NN-Descent, which inserts every evaluated pair at once.  Classic NN-Descent
    # here is a separate sequential routine that shares only the sampling.
    k, p, seed, iters = 10, 8, 42, 8
    x = W.uniform_f32(4096, 16, seed=1001)
    g_classic, trend_classic = og.build_classic(x, k, p, og.L2SQ_F32, seed, iters)
    g = og.init_random(x, k, og.L2SQ_F32, seed)
    trend = []
    for it in range(1, iters + 1):
        og.iterate(x, og.L2SQ_F32, g, p, seed, it)
        trend.append(og.phi(g.dist))
    assert all(b <= a for a, b in zip(trend, trend[1:]))
    assert all(b <= a for a, b in zip(trend_classic, trend_classic[1:]))
    for a, b in zip(trend, trend_classic):
        assert abs(a - b) / b < 0.05, (trend, trend_classic)
    _, td = og.bruteforce(x, og.L2SQ_F32, np.arange(4096, dtype=np.int32), k)
    exact = og.phi(td)
    assert exact <= trend_classic[-1] <= 1.02 * exact and exact <= trend[-1] <= 1.02 * exact
    _check_lists(g_classic, x, og.L2SQ_F32)


# ---- segmented lists (Sec. 4.3, "Multiple Spinlocks") ------------------------------------
def _class_rows(g, s, m):
    """Per residue class the (distance, id) pairs of row s, in list order."""
    return [[(float(dd), int(v)) for v, dd in zip(g.ids[s], g.dist[s]) if v % m == r]
            for r in range(m)]


def test_segmented_init_draws_32_of_every_class_and_reduces_to_the_plain_init():
    # "k-NN list is divided into k/32 segments. Each segment keeps 32 neighbors.  The object
    # v will be inserted into the v % (k/32)-th segment": a list that starts segmented holds
    # 32 objects of every residue class.  With one segment (k = 32) nothing distinguishes the
    # segmented form from the plain one: same draws, same list.
    x = W.uniform_f32(500, 7, seed=91)
    plain = og.init_random(x, 32, og.L2SQ_F32, 5)
    seg = og.init_random(x, 32, og.L2SQ_F32, 5, segmented=True)
    assert (plain.ids == seg.ids).all() and (plain.dist == seg.dist).all()
    for k in (64, 96, 128):
        m = k // 32
        g = og.init_random(x, k, og.L2SQ_F32, 5, segmented=True)
        assert g.isnew.all()
        for s in range(0, 500, 7):
            assert s not in g.ids[s] and len(set(g.ids[s].tolist())) == k
            keys = list(zip(g.dist[s].tolist(), g.ids[s].tolist()))
            assert keys == sorted(keys)
            assert np.bincount(g.ids[s] % m, minlength=m).tolist() == [32] * m
            for v, dd in zip(g.ids[s], g.dist[s]):
                assert dd == og.distance(x, og.L2SQ_F32, s, int(v))
        # the draws are the documented ones: slot 32 r + j takes the first member number of
        # hash(seed, INIT, s, 32 r + j, attempt), attempt = 0, 1, ..., that is neither s nor
        # taken by an earlier slot of the segment (the rule written out here in Python)
        for s in (0, 11, 250, 499):
            for r in range(m):
                members = (500 - r + m - 1) // m
                own = s // m if s % m == r else -1
                taken = []
                for j in range(32):
                    for attempt in range(256):
                        c = og.bounded(og.hash5(5, og.TAG_INIT, s, 32 * r + j, attempt), members)
                        if c != own and c not in taken:
                            break
                    else:
                        raise AssertionError("256 attempts exhausted on a class of 125+ members")
                    taken.append(c)
                want = sorted(c * m + r for c in taken)
                assert want == sorted(v for v in g.ids[s].tolist() if v % m == r), (k, s, r)
    # tiny classes: with n = 34 m every class has 34 members, one of them possibly s itself
    tiny = og.init_random(W.uniform_f32(68, 3, seed=92), 64, og.L2SQ_F32, 6, segmented=True)
    assert all(np.bincount(tiny.ids[s] % 2, minlength=2).tolist() == [32, 32] for s in range(68))
    with pytest.raises(ValueError):
        og.init_random(x, 48, og.L2SQ_F32, 5, segmented=True)


def test_segmented_update_is_the_per_class_best_32_and_order_independent():
    # The update as a set function, recomputed from its definition in Python: per class the
    # 32 best of (class entries before) u (proposals of that class), one entry per id; and
    # the same lists come out of one-by-one insertions into the 32-entry segments in any
    # order (each segment behind its own lock, Sec. 4.3).
    rng = np.random.default_rng(17)
    x = W.small_integer_f32(400, 4, seed=93, hi=5)  # many equal distances
    for k in (64, 128):
        m = k // 32
        g = og.init_random(x, k, og.L2SQ_F32, 9, segmented=True)
        p = 16
        snew, cnew, sold, cold = og.sample(g, p, 9, 1)
        pu, pv, pd, pcnt, _ = og.join(x, og.L2SQ_F32, p, snew, cnew, sold, cold)
        before = g.copy()
        ins = og.update(g, p, pu, pv, pd, pcnt, segmented=True)
        props = {}
        for s in range(400):
            for j in range(pcnt[s]):
                props.setdefault(int(pu[s, j]), []).append((float(pd[s, j]), int(pv[s, j])))
        admitted = 0
        for u in range(400):
            old = _class_rows(before, u, m)
            want = []
            for r in range(m):
                pool = {v: dd for dd, v in old[r]}
                for dd, v in props.get(u, []):
                    if v % m == r:
                        pool.setdefault(v, dd)
                best = sorted((dd, v) for v, dd in pool.items())[:32]
                admitted += len({v for _, v in best} - {v for _, v in old[r]})
                want += best
            got = list(zip(g.dist[u].tolist(), g.ids[u].tolist()))
            assert got == sorted(want), u
        assert ins == admitted
        # admitted entries are NEW, the others keep the flag sampling left them with
        for u in range(0, 400, 9):
            was = dict(zip(before.ids[u].tolist(), before.isnew[u].tolist()))
            for v, f in zip(g.ids[u].tolist(), g.isnew[u].tolist()):
                assert f == (1 if v not in was else was[v])
        # one by one, random order, into per-class arrays of 32
        for u in rng.choice(400, 25, replace=False):
            segs = [[np.array([v for _, v in c], np.int32), np.array([dd for dd, _ in c]),
                     np.zeros(32, np.uint8)] for c in _class_rows(before, int(u), m)]
            mine = props.get(int(u), [])
            for i in rng.permutation(len(mine)):
                dd, v = mine[i]
                og.insert_one(segs[v % m][0], segs[v % m][1], segs[v % m][2], v, dd)
            merged = sorted((float(dd), int(v)) for sg in segs for v, dd in zip(sg[0], sg[1]))
            assert merged == list(zip(g.dist[u].tolist(), g.ids[u].tolist()))


def test_segmented_build_converges_to_the_exact_lists_of_every_class():
    # On a tiny input the iteration finds, for every node, its exact nearest neighbours
    # (Recall@10 = 1 against exhaustive search) and the exact 8 nearest members of every
    # residue class (exhaustive search per class); phi never grows on the way and every
    # class keeps its 32 entries.  (The far end of a 32-entry segment is not reached by the
    # nearest-partner proposals of Alg. 2 on so small a set, hence the first 8.)
    n, k, m = 600, 64, 2
    x = W.uniform_f32(n, 3, seed=94)
    g = og.init_random(x, k, og.L2SQ_F32, 3, segmented=True)
    phi = [og.phi(g.dist)]
    for it in range(1, 11):
        prev = g.dist.copy()
        og.iterate(x, og.L2SQ_F32, g, 32, 3, it, segmented=True)
        assert ((g.ids % m) == 0).sum(1).tolist() == [32] * n
        assert (np.sort(g.dist, axis=1) == g.dist).all()
        phi.append(og.phi(g.dist))
        assert phi[-1] <= phi[-2] and (g.dist.sum(1) <= prev.sum(1)).all()
    tids, tdist = og.bruteforce(x, og.L2SQ_F32, np.arange(n), 10)
    assert og.recall_at(g.ids, g.dist, tids, tdist, 10) == (1.0, 1.0)
    hit = total = 0
    for s in range(0, n, 5):
        for r in range(m):
            members = np.array([v for v in range(r, n, m) if v != s], np.int32)
            dd = np.array([og.distance(x, og.L2SQ_F32, s, int(v)) for v in members])
            exact = sorted(zip(dd.tolist(), members.tolist()))[:8]
            got = [(float(a), int(v)) for v, a in zip(g.ids[s], g.dist[s]) if v % m == r][:8]
            hit += len(set(exact) & set(got))
            total += 8
    assert hit / total > 0.995, hit / total
