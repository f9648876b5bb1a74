"""ctypes front-end of the C oracle (oracle/gnnd_oracle.c) plus the evaluation
formulas of the paper (Recall@k, Sec. 6.1; phi(G), Sec. 4.3) in numpy.

TEST INFRASTRUCTURE: see the header of gnnd_oracle.c.  Argument marshalling
only; the algorithm is in the C file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

L2SQ_F32, ANGULAR_F32, L2SQ_U8, CHI2_F32, COSINE_F32 = 0, 1, 2, 3, 4
TAG_INIT, TAG_REV_NEW, TAG_REV_OLD, TAG_MERGE = 1, 2, 3, 4

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gnnd_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_gnnd.so")
_lib = None


def build_oracle(force=False):
    """Compile the oracle with gcc (plain C, -O2, contraction off so that only
    the explicit fmaf calls fuse)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=gnu11", "-O2", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
               "-Wall", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build_oracle()
    lib = C.CDLL(_LIB)
    i32p, f64p, u8p = (np.ctypeslib.ndpointer(dtype=t, flags="C_CONTIGUOUS")
                       for t in (np.int32, np.float64, np.uint8))
    vp = C.c_void_p
    lib.og_mix64.restype = C.c_uint64
    lib.og_mix64.argtypes = [C.c_uint64]
    lib.og_hash.restype = C.c_uint64
    lib.og_hash.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32]
    lib.og_bounded.restype = C.c_uint32
    lib.og_bounded.argtypes = [C.c_uint64, C.c_uint32]
    lib.og_distance.restype = C.c_double
    lib.og_distance.argtypes = [C.c_int, C.c_int, vp, C.c_int64, C.c_int64]
    lib.og_bruteforce.restype = None
    lib.og_bruteforce.argtypes = [vp, C.c_int64, C.c_int, C.c_int, i32p, C.c_int64, C.c_int,
                                  i32p, f64p]
    lib.og_init_random.restype = None
    lib.og_init_random.argtypes = [vp, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_uint64, i32p,
                                   f64p, u8p]
    lib.og_sample.restype = None
    lib.og_sample.argtypes = [C.c_int64, C.c_int, C.c_int, C.c_uint64, C.c_uint32, i32p, u8p,
                              i32p, i32p, i32p, i32p]
    lib.og_pair_of.restype = None
    lib.og_pair_of.argtypes = [C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    lib.og_join.restype = C.c_uint64
    lib.og_join.argtypes = [vp, C.c_int64, C.c_int, C.c_int, C.c_int, i32p, i32p, i32p, i32p,
                            C.c_int64, i32p, i32p, f64p, i32p]
    lib.og_insert_one.restype = C.c_int
    lib.og_insert_one.argtypes = [C.c_int, i32p, f64p, u8p, C.c_int32, C.c_double]
    lib.og_join_all.restype = C.c_uint64
    lib.og_join_all.argtypes = lib.og_join.argtypes
    lib.og_update_rows.restype = C.c_uint64
    lib.og_update_rows.argtypes = [C.c_int64, C.c_int, C.c_int, i32p, f64p, u8p, i32p, i32p, f64p,
                                   i32p]
    lib.og_classic_join_update.restype = C.c_uint64
    lib.og_classic_join_update.argtypes = [vp, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int,
                                           i32p, i32p, i32p, i32p, i32p, f64p, u8p,
                                           np.ctypeslib.ndpointer(np.uint64, flags="C")]
    lib.og_update_segmented.restype = C.c_uint64
    lib.og_update_segmented.argtypes = [C.c_int64, C.c_int, C.c_int, i32p, f64p, u8p, i32p, i32p,
                                        f64p, i32p]
    lib.og_init_random_segmented.restype = None
    lib.og_init_random_segmented.argtypes = [vp, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_uint64,
                                             i32p, f64p, u8p]
    lib.og_update.restype = C.c_uint64
    lib.og_update.argtypes = [C.c_int64, C.c_int, C.c_int, i32p, f64p, u8p, i32p, i32p, f64p,
                              i32p]
    lib.og_merge_init.restype = None
    lib.og_merge_init.argtypes = [vp, C.c_int64, C.c_int64, C.c_int64, C.c_int64, C.c_int,
                                  C.c_int, C.c_int, C.c_uint64, i32p, f64p, i32p, f64p, i32p,
                                  f64p, u8p, i32p, f64p]
    lib.og_merge_to_global.restype = None
    lib.og_merge_to_global.argtypes = [C.c_int64, C.c_int64, C.c_int64, C.c_int64, C.c_int,
                                       i32p, f64p]
    lib.og_merge_final.restype = None
    lib.og_merge_final.argtypes = [C.c_int64, C.c_int, i32p, f64p, i32p, f64p]
    _lib = lib
    return lib


def _vec(vectors, metric):
    want = np.uint8 if metric == L2SQ_U8 else np.float32
    v = np.ascontiguousarray(vectors)
    if v.dtype != want:
        raise TypeError(f"metric {metric} needs {want} vectors, got {v.dtype}")
    return v


def set_threads(t):
    """Number of OpenMP threads of the join / brute-force loops (results do not
    depend on it: every node writes its own output rows)."""
    C.CDLL("libgomp.so.1").omp_set_num_threads(int(t))


def mix64(z):
    return int(_load().og_mix64(C.c_uint64(z)))


def hash5(seed, tag, a, b, c):
    return int(_load().og_hash(seed, tag, a, b, c))


def bounded(h, n):
    return int(_load().og_bounded(h, n))


def distance(vectors, metric, i, j):
    v = _vec(vectors, metric)
    return float(_load().og_distance(metric, v.shape[1], v.ctypes.data, i, j))


def pair_of(t):
    u, v = C.c_int32(), C.c_int32()
    _load().og_pair_of(t, C.byref(u), C.byref(v))
    return u.value, v.value


def bruteforce(vectors, metric, queries, K):
    v = _vec(vectors, metric)
    q = np.ascontiguousarray(queries, dtype=np.int32)
    ids = np.empty((len(q), K), np.int32)
    dist = np.empty((len(q), K), np.float64)
    _load().og_bruteforce(v.ctypes.data, v.shape[0], v.shape[1], metric, q, len(q), K, ids, dist)
    return ids, dist


class Graph:
    """k-NN graph state: ids, dist (float64 holding the metric's own float32 or
    int32 values exactly) and the NEW flags, n rows of k."""

    def __init__(self, ids, dist, isnew):
        self.ids, self.dist, self.isnew = ids, dist, isnew

    def copy(self):
        return Graph(self.ids.copy(), self.dist.copy(), self.isnew.copy())


def init_random(vectors, k, metric, seed, segmented=False):
    """Alg. 1, first loop.  segmented: the list of k = 32 m entries starts as m segments of
    32 random objects of one residue class each (Sec. 4.3, "Multiple Spinlocks")."""
    v = _vec(vectors, metric)
    n, d = v.shape
    g = Graph(np.empty((n, k), np.int32), np.empty((n, k), np.float64), np.empty((n, k), np.uint8))
    if segmented:
        if k % 32 or not 32 <= k <= 128 or n < 34 * (k // 32):
            raise ValueError("segmented lists need k in {32, 64, 96, 128} and n >= 34 k / 32")
        _load().og_init_random_segmented(v.ctypes.data, n, d, k, metric, seed, g.ids, g.dist,
                                         g.isnew)
    else:
        _load().og_init_random(v.ctypes.data, n, d, k, metric, seed, g.ids, g.dist, g.isnew)
    return g


def sample(g, p, seed, it):
    """Returns (snew, cnew, sold, cold); clears the flags of the sampled NEW
    entries of g in place."""
    n, k = g.ids.shape
    snew = np.empty((n, 2 * p), np.int32)
    sold = np.empty((n, 2 * p), np.int32)
    cnew = np.empty(n, np.int32)
    cold = np.empty(n, np.int32)
    _load().og_sample(n, k, p, seed, it, g.ids, g.isnew, snew, cnew, sold, cold)
    return snew, cnew, sold, cold


def join(vectors, metric, p, snew, cnew, sold, cold, split=-1, all_pairs=False):
    """Returns (pu, pv, pd, pcnt, dist_evals): proposals 'insert pv with distance
    pd into the list of pu', up to 6p per joined node (Alg. 2: nearest partners
    only), or with all_pairs every evaluated pair both ways, up to 2p(6p - 1)
    per node (the ablation variant without the selective update, Sec. 6.2)."""
    v = _vec(vectors, metric)
    n, d = v.shape
    width = 2 * p * (6 * p - 1) if all_pairs else 6 * p
    pu = np.full((n, width), -1, np.int32)
    pv = np.full((n, width), -1, np.int32)
    pd = np.full((n, width), np.inf, np.float64)
    pcnt = np.zeros(n, np.int32)
    fn = _load().og_join_all if all_pairs else _load().og_join
    ev = fn(v.ctypes.data, n, d, p, metric, snew, cnew, sold, cold, split, pu, pv, pd, pcnt)
    return pu, pv, pd, pcnt, int(ev)


def insert_one(ids_row, dist_row, isnew_row, v, d):
    return int(_load().og_insert_one(len(ids_row), ids_row, dist_row, isnew_row, v, d))


def update(g, p, pu, pv, pd, pcnt, segmented=False):
    n, k = g.ids.shape
    if segmented:  # object v competes inside segment v % (k / 32) only
        return int(_load().og_update_segmented(n, k, pu.shape[1], g.ids, g.dist, g.isnew, pu, pv,
                                               pd, pcnt))
    if pu.shape[1] != 6 * p:  # rows of the all-pairs join
        return int(_load().og_update_rows(n, k, pu.shape[1], g.ids, g.dist, g.isnew, pu, pv, pd,
                                          pcnt))
    return int(_load().og_update(n, k, p, g.ids, g.dist, g.isnew, pu, pv, pd, pcnt))


def iterate(vectors, metric, g, p, seed, it, split=-1, all_pairs=False, segmented=False):
    """One GNND iteration (Alg. 1 loop body) in place; `it` counts from 1.
    Returns a dict of statistics and the intermediate sample lists/proposals."""
    snew, cnew, sold, cold = sample(g, p, seed, it)
    pu, pv, pd, pcnt, ev = join(vectors, metric, p, snew, cnew, sold, cold, split, all_pairs)
    ins = update(g, p, pu, pv, pd, pcnt, segmented)
    return dict(iter=it, inserts=ins, dist_evals=ev, sum_new=int(cnew.sum()),
                sum_old=int(cold.sum()), proposals=int(pcnt.sum()),
                snew=snew, cnew=cnew, sold=sold, cold=cold)


def build(vectors, k, p, metric, seed, iters, all_pairs=False, segmented=False):
    """Alg. 1 as a whole: random initial graph, then `iters` iterations."""
    g = init_random(vectors, k, metric, seed, segmented)
    stats = []
    for it in range(1, iters + 1):
        st = iterate(vectors, metric, g, p, seed, it, all_pairs=all_pairs, segmented=segmented)
        stats.append({key: st[key] for key in ("iter", "inserts", "dist_evals", "sum_new",
                                               "sum_old", "proposals")})
    return g, stats


def build_classic(vectors, k, p, metric, seed, iters):
    """Classic NN-Descent (Sec. 3) for comparison: the same initial graph and the
    same sampling as build(), but every evaluated pair is inserted into both lists
    at once, node after node.  Returns the graph and phi after every iteration."""
    v = _vec(vectors, metric)
    n, d = v.shape
    g = init_random(vectors, k, metric, seed)
    trend = []
    for it in range(1, iters + 1):
        snew, cnew, sold, cold = sample(g, p, seed, it)
        ins = np.zeros(1, np.uint64)
        _load().og_classic_join_update(v.ctypes.data, n, d, k, p, metric, snew, cnew, sold, cold,
                                       g.ids, g.dist, g.isnew, ins)
        trend.append(phi(g.dist))
    return g, trend


def merge_init(vectors, n1, k, metric, seed, g1, g2, base1=0, base2=None):
    """g1, g2 carry collection ids: S1 = [base1, base1+n1), S2 = [base2, base2+n2).
    The returned graph uses the merge's own numbering (S1 rows, S2 rows, then
    n + collection id for entries that belong to neither set)."""
    v = _vec(vectors, metric)
    n, d = v.shape
    n2 = n - n1
    base2 = n1 if base2 is None else base2
    fill = k // 2
    g = Graph(np.empty((n, k), np.int32), np.empty((n, k), np.float64), np.empty((n, k), np.uint8))
    aside_ids = np.empty((n, fill), np.int32)
    aside_dist = np.empty((n, fill), np.float64)
    _load().og_merge_init(v.ctypes.data, n1, base1, n2, base2, d, k, metric, seed,
                          np.ascontiguousarray(g1.ids), np.ascontiguousarray(g1.dist),
                          np.ascontiguousarray(g2.ids), np.ascontiguousarray(g2.dist),
                          g.ids, g.dist, g.isnew, aside_ids, aside_dist)
    return g, aside_ids, aside_dist


def merge_final(g, aside_ids, aside_dist):
    n, k = g.ids.shape
    _load().og_merge_final(n, k, g.ids, g.dist, aside_ids, aside_dist)


def merge(vectors, n1, k, p, metric, seed, g1, g2, iters, base1=0, base2=None):
    """Alg. 3 as a whole.  vectors = S1 rows then S2 rows; g1 and g2 carry
    collection ids (S1 = [base1, base1+n1), S2 = [base2, base2+n2), default
    0 and n1: the union itself).  Returns the merged graph in collection ids,
    lists ascending by (distance, id), and per-iteration statistics."""
    n = len(vectors)
    base2 = n1 if base2 is None else base2
    g, aside_ids, aside_dist = merge_init(vectors, n1, k, metric, seed, g1, g2, base1, base2)
    stats = []
    for it in range(1, iters + 1):
        st = iterate(vectors, metric, g, p, seed, it, split=n1)
        stats.append({key: st[key] for key in ("iter", "inserts", "dist_evals", "sum_new",
                                               "sum_old", "proposals")})
    merge_final(g, aside_ids, aside_dist)
    _load().og_merge_to_global(n1, base1, n - n1, base2, k, g.ids, g.dist)
    return g, stats


def append(vectors, n1, g1, k, p, metric, seed, build_iters, merge_iters):
    """Incremental construction (Sec. 5.1): rows n1.. of `vectors` are a batch
    that joins the collection of rows 0..n1-1 with graph g1.  The batch's own
    graph is built first (Alg. 1, seed + 1), then merged into g1 (Alg. 3, seed).
    Returns the graph of the union in ids 0..n-1."""
    sub, _ = build(np.ascontiguousarray(vectors[n1:]), k, p, metric, seed + 1, build_iters)
    g2 = Graph(sub.ids + np.int32(n1), sub.dist, sub.isnew)
    g, _ = merge(vectors, n1, k, p, metric, seed, g1, g2, merge_iters)
    return g


def pair_schedule(shards):
    """Every pair of shards once ("any two sub-graphs has been merged once",
    Sec. 5.1), as a round-robin tournament: rounds of disjoint pairs, the last
    shard fixed and the others rotating around it (an odd count gets a bye)."""
    m = shards + (shards % 2)
    ring = m - 1
    order = []
    for r in range(ring):
        for i in range(m // 2):
            a, b = (m - 1, r) if i == 0 else ((r + i) % ring, (r - i) % ring)
            if a < shards and b < shards:
                order.append((min(a, b), max(a, b)))
    return order


def build_sharded(vectors, shards, k, p, metric, seed, build_iters, merge_iters, schedule=None,
                  after_merge=None):
    """Sec. 5.1 out-of-core scheme on equal shards of consecutive rows: a graph
    per shard (seed + shard number), then every pair of shards merged once in
    the order of pair_schedule() (or of `schedule`, a list of pairs, for
    comparisons of orders); each merged graph is stored back as the two shards'
    sub-graphs.  Merge number m uses seed + 1000 + m.  `after_merge(m, i, j,
    before_i, before_j, after_i, after_j)` is called with the two sub-graphs as
    they were and as they are stored back (a hook for invariant checks)."""
    n = len(vectors)
    size = n // shards
    bases = [i * size for i in range(shards)]
    sizes = [size] * (shards - 1) + [n - size * (shards - 1)]
    graphs = []
    for i in range(shards):
        g, _ = build(vectors[bases[i]:bases[i] + sizes[i]], k, p, metric, seed + i, build_iters)
        graphs.append(Graph(g.ids + bases[i], g.dist, g.isnew))
    for m, (i, j) in enumerate(pair_schedule(shards) if schedule is None else schedule):
        x = np.concatenate([vectors[bases[i]:bases[i] + sizes[i]],
                            vectors[bases[j]:bases[j] + sizes[j]]])
        g, _ = merge(x, sizes[i], k, p, metric, seed + 1000 + m, graphs[i], graphs[j],
                     merge_iters, bases[i], bases[j])
        before = graphs[i], graphs[j]
        graphs[i] = Graph(g.ids[:sizes[i]].copy(), g.dist[:sizes[i]].copy(), None)
        graphs[j] = Graph(g.ids[sizes[i]:].copy(), g.dist[sizes[i]:].copy(), None)
        if after_merge is not None:
            after_merge(m, i, j, before[0], before[1], graphs[i], graphs[j])
    ids = np.concatenate([g.ids for g in graphs])
    dist = np.concatenate([g.dist for g in graphs])
    return Graph(ids, dist, np.zeros_like(ids, dtype=np.uint8))


# --- evaluation formulas ----------------------------------------------------
def recall_at(graph_ids, graph_dist, truth_ids, truth_dist, K=10):
    """Recall@K (Sec. 6.1 equation) over the evaluated rows.  Returns
    (tie_tolerant, strict): the first counts a listed neighbour among the first
    K as a true positive when its distance does not exceed the exact K-th
    distance of that node (equal distances are interchangeable neighbours); the
    second counts id matches with the exact (distance, id)-ordered list."""
    gi = np.asarray(graph_ids)[:, :K]
    gd = np.asarray(graph_dist)[:, :K]
    kth = np.asarray(truth_dist)[:, K - 1:K]
    tol = float(((gd <= kth) & (gi >= 0)).sum()) / gi.size
    strict = sum(len(np.intersect1d(gi[r], truth_ids[r, :K])) for r in range(len(gi))) / gi.size
    return tol, float(strict)


def phi(graph_dist):
    """phi(G): sum of all listed distances (Sec. 4.3 equation)."""
    return float(np.asarray(graph_dist, dtype=np.float64).sum())
