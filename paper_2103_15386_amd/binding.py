"""ctypes binding of the C ABI in include/gnnd.h.  Marshalling only."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

L2SQ_F32, ANGULAR_F32, L2SQ_U8, CHI2_F32, COSINE_F32 = 0, 1, 2, 3, 4
JOIN_AUTO, JOIN_VALU, JOIN_MFMA, JOIN_MFMA_DIRECT, JOIN_GRAM = 0, 1, 2, 3, 4
UPDATE_SELECTIVE, UPDATE_ALL_PAIRS = 0, 1
LISTS_PLAIN, LISTS_SEGMENTED = 0, 1
OK, EINVAL, ENOSPC, ESTATE, EHIP, EIO = 0, -1, -2, -3, -4, -5
STATIC_SCRATCH_BYTES = 64 << 20  # GNND_STATIC_SCRATCH_BYTES of include/gnnd.h

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libgnnd_hip.so")
_lib = None

EXPORTS = [
    "gnnd_workspace_bytes", "gnnd_create", "gnnd_destroy", "gnnd_last_error", "gnnd_init_random",
    "gnnd_iterate", "gnnd_step_sample", "gnnd_step_join", "gnnd_step_update", "gnnd_build",
    "gnnd_get_graph", "gnnd_set_graph", "gnnd_get_samples", "gnnd_get_proposals", "gnnd_merge",
    "gnnd_exact_knn", "gnnd_join_path", "gnnd_set_profiling", "gnnd_get_stage_ms",
    "gnnd_sharded_arena_bytes", "gnnd_build_sharded", "gnnd_build_sharded_files", "gnnd_append",
    "gnnd_build_static",
]


class GnndError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"gnnd error {code}: {msg}")
        self.code = code


class Params(C.Structure):
    _fields_ = [("n", C.c_int64), ("d", C.c_int32), ("k", C.c_int32), ("p", C.c_int32),
                ("metric", C.c_int32), ("seed", C.c_uint64), ("stream", C.c_void_p),
                ("workspace_dev", C.c_void_p), ("workspace_bytes", C.c_size_t),
                ("join_path", C.c_int32), ("update_mode", C.c_int32),
                ("list_mode", C.c_int32), ("reserved", C.c_int32)]


class IterStats(C.Structure):
    _fields_ = [("iter", C.c_int32), ("reserved", C.c_int32), ("inserts", C.c_uint64),
                ("dist_evals", C.c_uint64), ("sum_new", C.c_uint64), ("sum_old", C.c_uint64),
                ("proposals", C.c_uint64), ("dropped", C.c_uint64), ("passed", C.c_uint64),
                ("ms_sample", C.c_float), ("ms_join", C.c_float),
                ("ms_update", C.c_float), ("ms_handout", C.c_float)]

    def as_dict(self):
        return {f: getattr(self, f) for f, _ in self._fields_ if not f.startswith("reserved")}


class ShardStats(C.Structure):
    _fields_ = [("builds", C.c_int32), ("merges", C.c_int32), ("ms_build", C.c_float),
                ("ms_merge", C.c_float), ("ms_total", C.c_float), ("reserved", C.c_float)]


def library_path():
    return _LIB_PATH


def load_library():
    """Load libgnnd_hip.so (built in-tree by paper_2103_15386_amd.build).  Raises
    if it has not been built: there is no other implementation to fall back to."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise GnndError(EHIP, f"{_LIB_PATH} is missing: run `python -m paper_2103_15386_amd.build`")
    lib = C.CDLL(_LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    PP = C.POINTER(Params)
    SP = C.POINTER(IterStats)
    lib.gnnd_workspace_bytes.restype = C.c_size_t
    lib.gnnd_workspace_bytes.argtypes = [PP]
    lib.gnnd_create.restype = C.c_int
    lib.gnnd_create.argtypes = [C.POINTER(vp), PP, vp]
    lib.gnnd_destroy.restype = None
    lib.gnnd_destroy.argtypes = [vp]
    lib.gnnd_last_error.restype = C.c_char_p
    lib.gnnd_last_error.argtypes = [vp]
    for name in ("gnnd_init_random", "gnnd_step_sample", "gnnd_step_join"):
        getattr(lib, name).restype = C.c_int
        getattr(lib, name).argtypes = [vp]
    lib.gnnd_iterate.restype = C.c_int
    lib.gnnd_iterate.argtypes = [vp, SP]
    lib.gnnd_step_update.restype = C.c_int
    lib.gnnd_step_update.argtypes = [vp, SP]
    lib.gnnd_build.restype = C.c_int
    lib.gnnd_build.argtypes = [vp, i32, C.c_float, SP]
    lib.gnnd_get_graph.restype = C.c_int
    lib.gnnd_get_graph.argtypes = [vp, vp, vp, vp]
    lib.gnnd_set_graph.restype = C.c_int
    lib.gnnd_set_graph.argtypes = [vp, vp, vp, vp, i32]
    lib.gnnd_get_samples.restype = C.c_int
    lib.gnnd_get_samples.argtypes = [vp, vp, vp, vp, vp]
    lib.gnnd_get_proposals.restype = C.c_int
    lib.gnnd_get_proposals.argtypes = [vp, vp, vp, vp]
    lib.gnnd_merge.restype = C.c_int
    lib.gnnd_merge.argtypes = [PP, vp, i64, i64, vp, i64, i64, i64, vp, vp, vp, vp, i32, vp, vp, SP]
    lib.gnnd_append.restype = C.c_int
    lib.gnnd_append.argtypes = [PP, vp, i64, vp, vp, vp, i64, i32, i32, vp, vp]
    lib.gnnd_sharded_arena_bytes.restype = C.c_size_t
    lib.gnnd_sharded_arena_bytes.argtypes = [PP, i32]
    lib.gnnd_build_sharded.restype = C.c_int
    lib.gnnd_build_sharded.argtypes = [PP, vp, i32, i32, i32, vp, vp, vp, C.POINTER(ShardStats)]
    lib.gnnd_build_sharded_files.restype = C.c_int
    lib.gnnd_build_sharded_files.argtypes = [PP, C.c_char_p, i32, i32, i32, C.c_char_p, C.c_char_p,
                                             vp, C.c_size_t, vp, C.POINTER(ShardStats)]
    lib.gnnd_join_path.restype = C.c_int
    lib.gnnd_join_path.argtypes = [vp]
    lib.gnnd_set_profiling.restype = C.c_int
    lib.gnnd_set_profiling.argtypes = [vp, C.c_int]
    lib.gnnd_get_stage_ms.restype = C.c_int
    lib.gnnd_get_stage_ms.argtypes = [vp, C.POINTER(i32), C.POINTER(i32), C.POINTER(C.c_float),
                                      C.POINTER(C.c_float), C.POINTER(C.c_float),
                                      C.POINTER(C.c_float)]
    lib.gnnd_build_static.restype = C.c_int
    lib.gnnd_build_static.argtypes = [PP, vp, i32, vp, vp]
    lib.gnnd_exact_knn.restype = C.c_int
    lib.gnnd_exact_knn.argtypes = [vp, i64, i32, i32, vp, i64, i32, vp, vp, vp]
    _lib = lib
    return lib


def _err(ctx=None):
    return load_library().gnnd_last_error(ctx).decode()


def _check(rc, ctx=None):
    if rc != OK:
        raise GnndError(rc, _err(ctx))


def _elem_dtype(metric):
    return torch.uint8 if metric == L2SQ_U8 else torch.float32


def _dist_dtype(metric):
    return torch.int32 if metric == L2SQ_U8 else torch.float32


def _require_device(t, dtype, what):
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise GnndError(EINVAL, f"{what} must be a GPU tensor (no CPU path exists)")
    if t.dtype != dtype or not t.is_contiguous():
        raise GnndError(EINVAL, f"{what} must be contiguous {dtype}")
    return t


def _stream_ptr(device):
    return torch.cuda.current_stream(device).cuda_stream


def make_params(n, d, k, p, metric, seed=42, join_path=JOIN_AUTO, stream=0, workspace=None,
                update_mode=UPDATE_SELECTIVE, list_mode=LISTS_PLAIN):
    prm = Params()
    prm.n, prm.d, prm.k, prm.p, prm.metric = n, d, k, p, metric
    prm.seed = seed
    prm.stream = stream
    prm.join_path = join_path
    prm.update_mode = update_mode
    prm.list_mode = list_mode
    if workspace is not None:
        prm.workspace_dev = workspace.data_ptr()
        prm.workspace_bytes = workspace.numel() * workspace.element_size()
    return prm


def workspace_bytes(n, d, k, p, metric, update_mode=UPDATE_SELECTIVE, list_mode=LISTS_PLAIN,
                    join_path=JOIN_AUTO):
    """Bytes of device scratch a context with these parameters needs (0 = invalid)."""
    prm = make_params(n, d, k, p, metric, join_path=join_path, update_mode=update_mode,
                      list_mode=list_mode)
    return int(load_library().gnnd_workspace_bytes(C.byref(prm)))


class Gnnd:
    """One GNND context over a resident vector tensor (n x d, float32 or uint8)."""

    def __init__(self, vectors, k, p, metric=L2SQ_F32, seed=42, join_path=JOIN_AUTO,
                 update_mode=UPDATE_SELECTIVE, list_mode=LISTS_PLAIN):
        lib = load_library()
        self.vectors = _require_device(vectors, _elem_dtype(metric), "vectors")
        self.n, self.d = vectors.shape
        self.k, self.p, self.metric, self.seed = k, p, metric, seed
        self.update_mode = update_mode
        need = workspace_bytes(self.n, self.d, k, p, metric, update_mode, list_mode, join_path)
        if need == 0:
            prm = make_params(self.n, self.d, k, p, metric, seed, join_path,
                              update_mode=update_mode, list_mode=list_mode)
            ctx = C.c_void_p()
            rc = lib.gnnd_create(C.byref(ctx), C.byref(prm), vectors.data_ptr())
            raise GnndError(rc, _err())
        self.workspace = torch.empty(need, dtype=torch.uint8, device=vectors.device)
        self.prm = make_params(self.n, self.d, k, p, metric, seed, join_path,
                               _stream_ptr(vectors.device), self.workspace, update_mode, list_mode)
        self._ctx = C.c_void_p()
        _check(lib.gnnd_create(C.byref(self._ctx), C.byref(self.prm), vectors.data_ptr()))
        self._lib = lib

    def close(self):
        if getattr(self, "_ctx", None):
            self._lib.gnnd_destroy(self._ctx)
            self._ctx = None

    __del__ = close

    def join_path(self):
        """JOIN_VALU or JOIN_MFMA: the distance evaluation this context resolved to."""
        return int(self._lib.gnnd_join_path(self._ctx))

    def set_profiling(self, iterations=64):
        """Open a recording window of `iterations` iterations (0 / False: off)."""
        _check(self._lib.gnnd_set_profiling(self._ctx, int(iterations)), self._ctx)

    def stage_ms(self):
        """(iterations recorded, iterations missed because the window was full, ms sampling,
        ms cross-matching, ms hand-out pass, ms update) since the last call."""
        cnt, miss = C.c_int32(), C.c_int32()
        a, b, h, c = C.c_float(), C.c_float(), C.c_float(), C.c_float()
        _check(self._lib.gnnd_get_stage_ms(self._ctx, C.byref(cnt), C.byref(miss), C.byref(a),
                                           C.byref(b), C.byref(h), C.byref(c)), self._ctx)
        return cnt.value, miss.value, a.value, b.value, h.value, c.value

    def init_random(self):
        _check(self._lib.gnnd_init_random(self._ctx), self._ctx)

    def iterate(self, want_stats=True):
        st = IterStats()
        _check(self._lib.gnnd_iterate(self._ctx, C.byref(st) if want_stats else None), self._ctx)
        return st.as_dict() if want_stats else None

    def step_sample(self):
        _check(self._lib.gnnd_step_sample(self._ctx), self._ctx)

    def step_join(self):
        _check(self._lib.gnnd_step_join(self._ctx), self._ctx)

    def step_update(self, want_stats=True):
        st = IterStats()
        _check(self._lib.gnnd_step_update(self._ctx, C.byref(st) if want_stats else None),
               self._ctx)
        return st.as_dict() if want_stats else None

    def build(self, max_iters, delta=0.0, want_stats=True):
        st = IterStats()
        _check(self._lib.gnnd_build(self._ctx, max_iters, delta,
                                    C.byref(st) if want_stats else None), self._ctx)
        return st.as_dict() if want_stats else None

    def graph(self, with_flags=False):
        dev = self.vectors.device
        ids = torch.empty((self.n, self.k), dtype=torch.int32, device=dev)
        dist = torch.empty((self.n, self.k), dtype=_dist_dtype(self.metric), device=dev)
        flags = torch.empty((self.n, self.k), dtype=torch.uint8, device=dev) if with_flags else None
        _check(self._lib.gnnd_get_graph(self._ctx, ids.data_ptr(), dist.data_ptr(),
                                        flags.data_ptr() if with_flags else None), self._ctx)
        return (ids, dist, flags) if with_flags else (ids, dist)

    def set_graph(self, ids, dist, flags, it):
        _require_device(ids, torch.int32, "ids")
        _require_device(dist, _dist_dtype(self.metric), "dist")
        _require_device(flags, torch.uint8, "flags")
        _check(self._lib.gnnd_set_graph(self._ctx, ids.data_ptr(), dist.data_ptr(),
                                        flags.data_ptr(), it), self._ctx)

    def samples(self):
        dev = self.vectors.device
        L = 2 * self.p
        snew = torch.empty((self.n, L), dtype=torch.int32, device=dev)
        sold = torch.empty((self.n, L), dtype=torch.int32, device=dev)
        cnew = torch.empty(self.n, dtype=torch.int32, device=dev)
        cold = torch.empty(self.n, dtype=torch.int32, device=dev)
        _check(self._lib.gnnd_get_samples(self._ctx, snew.data_ptr(), cnew.data_ptr(),
                                          sold.data_ptr(), cold.data_ptr()), self._ctx)
        return snew, cnew, sold, cold

    def proposals(self):
        dev = self.vectors.device
        per_node = 6 * self.p if self.update_mode == UPDATE_SELECTIVE \
            else 2 * self.p * (6 * self.p - 1)
        shape = (self.n, per_node)
        u = torch.empty(shape, dtype=torch.int32, device=dev)
        v = torch.empty(shape, dtype=torch.int32, device=dev)
        dist = torch.empty(shape, dtype=_dist_dtype(self.metric), device=dev)
        _check(self._lib.gnnd_get_proposals(self._ctx, u.data_ptr(), v.data_ptr(),
                                            dist.data_ptr()), self._ctx)
        return u, v, dist


# ---- free functions with the names of the C entry points --------------------
def gnnd_init_random(ctx: Gnnd):
    ctx.init_random()


def gnnd_iterate(ctx: Gnnd, want_stats=True):
    return ctx.iterate(want_stats)


def gnnd_build(vectors, k, p, metric=L2SQ_F32, seed=42, iters=12, join_path=JOIN_AUTO,
               update_mode=UPDATE_SELECTIVE):
    """Build a graph from scratch; returns (ids, dist, context)."""
    ctx = Gnnd(vectors, k, p, metric, seed, join_path, update_mode)
    ctx.build(iters, want_stats=False)
    ids, dist = ctx.graph()
    return ids, dist, ctx


def gnnd_build_static(vectors, k, p, metric=L2SQ_F32, seed=42, iters=12, join_path=JOIN_AUTO,
                      ids_out=None, dist_out=None):
    """gnnd_build through the library's static scratch array (no workspace is
    allocated or passed); returns (ids, dist).  The outputs may be handed in."""
    lib = load_library()
    _require_device(vectors, _elem_dtype(metric), "vectors")
    n, d = vectors.shape
    dev = vectors.device
    ids = torch.empty((n, k), dtype=torch.int32, device=dev) if ids_out is None else ids_out
    dist = (torch.empty((n, k), dtype=_dist_dtype(metric), device=dev) if dist_out is None
            else dist_out)
    _require_device(ids, torch.int32, "ids_out")
    _require_device(dist, _dist_dtype(metric), "dist_out")
    prm = make_params(n, d, k, p, metric, seed, join_path, _stream_ptr(dev))
    with torch.cuda.device(dev):
        _check(lib.gnnd_build_static(C.byref(prm), vectors.data_ptr(), iters, ids.data_ptr(),
                                     dist.data_ptr()))
    return ids, dist


def gnnd_merge(vec1, vec2, ids1, dist1, ids2, dist2, k, p, metric=L2SQ_F32, seed=42, iters=6,
               join_path=JOIN_AUTO, want_stats=False, base1=0, base2=None, id_space=None):
    """GGM of two graphs given in collection ids (S1 = [base1, base1+n1), S2 =
    [base2, base2+n2); default: the two halves of one array); returns (ids,
    dist[, stats]) for the rows of S1 then S2, in collection ids."""
    lib = load_library()
    et, dt = _elem_dtype(metric), _dist_dtype(metric)
    _require_device(vec1, et, "vec1")
    _require_device(vec2, et, "vec2")
    for t, ty, nm in ((ids1, torch.int32, "ids1"), (ids2, torch.int32, "ids2"),
                      (dist1, dt, "dist1"), (dist2, dt, "dist2")):
        _require_device(t, ty, nm)
    n1, d = vec1.shape
    n2 = vec2.shape[0]
    n = n1 + n2
    base2 = n1 if base2 is None else base2
    id_space = max(base1 + n1, base2 + n2) if id_space is None else id_space
    need = workspace_bytes(n, d, k, p, metric, join_path=join_path)
    dev = vec1.device
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    prm = make_params(n, d, k, p, metric, seed, join_path, _stream_ptr(dev), ws)
    ids = torch.empty((n, k), dtype=torch.int32, device=dev)
    dist = torch.empty((n, k), dtype=dt, device=dev)
    stats = (IterStats * max(iters, 1))()
    rc = lib.gnnd_merge(C.byref(prm), vec1.data_ptr(), n1, base1, vec2.data_ptr(), n2, base2,
                        id_space, ids1.data_ptr(), dist1.data_ptr(), ids2.data_ptr(),
                        dist2.data_ptr(), iters, ids.data_ptr(), dist.data_ptr(),
                        stats if want_stats else None)
    _check(rc)
    torch.cuda.current_stream(dev).synchronize()  # the workspace dies with this frame
    if want_stats:
        return ids, dist, [stats[i].as_dict() for i in range(iters)]
    return ids, dist


def gnnd_append(vec1, ids1, dist1, vec2, k, p, metric=L2SQ_F32, seed=42, build_iters=8,
                merge_iters=6, join_path=JOIN_AUTO):
    """Incremental construction: the batch vec2 joins the collection vec1 whose
    graph is (ids1, dist1); returns (ids, dist) of the union, rows of vec1 first,
    the new objects numbered n1.."""
    lib = load_library()
    et, dt = _elem_dtype(metric), _dist_dtype(metric)
    _require_device(vec1, et, "vec1")
    _require_device(vec2, et, "vec2")
    _require_device(ids1, torch.int32, "ids1")
    _require_device(dist1, dt, "dist1")
    n1, d = vec1.shape
    n2 = vec2.shape[0]
    n = n1 + n2
    dev = vec1.device
    ws = torch.empty(max(workspace_bytes(n, d, k, p, metric, join_path=join_path), 256),
                     dtype=torch.uint8, device=dev)
    prm = make_params(n, d, k, p, metric, seed, join_path, _stream_ptr(dev), ws)
    ids = torch.empty((n, k), dtype=torch.int32, device=dev)
    dist = torch.empty((n, k), dtype=dt, device=dev)
    _check(lib.gnnd_append(C.byref(prm), vec1.data_ptr(), n1, ids1.data_ptr(), dist1.data_ptr(),
                           vec2.data_ptr(), n2, build_iters, merge_iters, ids.data_ptr(),
                           dist.data_ptr()))
    torch.cuda.current_stream(dev).synchronize()  # the workspace dies with this frame
    return ids, dist


def gnnd_build_sharded(vectors_host, shards, k, p, metric=L2SQ_F32, seed=42, build_iters=8,
                       merge_iters=4, join_path=JOIN_AUTO, device="cuda:0"):
    """Out-of-core build (Sec. 5.1): `vectors_host` is a pinned host tensor that
    never becomes resident as a whole.  Returns (ids, dist, stats): pinned host
    tensors n x k in collection ids, and the timing record."""
    lib = load_library()
    et, dt = _elem_dtype(metric), _dist_dtype(metric)
    if (not isinstance(vectors_host, torch.Tensor) or vectors_host.is_cuda
            or not vectors_host.is_pinned() or vectors_host.dtype != et
            or not vectors_host.is_contiguous()):
        raise GnndError(EINVAL, f"vectors_host must be a contiguous pinned host tensor of {et}")
    n, d = vectors_host.shape
    dev = torch.device(device)
    prm = make_params(n, d, k, p, metric, seed, join_path)
    need = int(lib.gnnd_sharded_arena_bytes(C.byref(prm), shards))
    if need == 0:
        rc = lib.gnnd_build_sharded(C.byref(prm), vectors_host.data_ptr(), shards, build_iters,
                                    merge_iters, None, None, None, None)
        raise GnndError(rc, _err())
    arena = torch.empty(need, dtype=torch.uint8, device=dev)
    copy_stream = torch.cuda.Stream(device=dev)
    prm = make_params(n, d, k, p, metric, seed, join_path, _stream_ptr(dev), arena)
    ids = torch.empty((n, k), dtype=torch.int32).pin_memory()
    dist = torch.empty((n, k), dtype=dt).pin_memory()
    st = ShardStats()
    _check(lib.gnnd_build_sharded(C.byref(prm), vectors_host.data_ptr(), shards, build_iters,
                                  merge_iters, ids.data_ptr(), dist.data_ptr(),
                                  copy_stream.cuda_stream, C.byref(st)))
    return ids, dist, {f: getattr(st, f) for f, _ in st._fields_ if f != "reserved"}


def gnnd_build_sharded_files(vectors_path, n, d, shards, k, p, ids_path, dist_path,
                             metric=L2SQ_F32, seed=42, build_iters=8, merge_iters=4,
                             join_path=JOIN_AUTO, staging_bytes=256 << 20, device="cuda:0"):
    """Out-of-core build with the collection and the graph in files (Sec. 5.1):
    `vectors_path` holds n x d elements row-major; `ids_path` / `dist_path` are
    created and receive the n x k graph in collection ids.  One pinned staging
    buffer of `staging_bytes` is the only host memory used.  Returns the timing
    record."""
    lib = load_library()
    dev = torch.device(device)
    prm = make_params(n, d, k, p, metric, seed, join_path)
    need = int(lib.gnnd_sharded_arena_bytes(C.byref(prm), shards))
    paths = [str(x).encode() for x in (vectors_path, ids_path, dist_path)]
    if need == 0:
        rc = lib.gnnd_build_sharded_files(C.byref(prm), paths[0], shards, build_iters, merge_iters,
                                          paths[1], paths[2], None, 0, None, None)
        raise GnndError(rc, _err())
    arena = torch.empty(need, dtype=torch.uint8, device=dev)
    staging = torch.empty(int(staging_bytes), dtype=torch.uint8).pin_memory()
    copy_stream = torch.cuda.Stream(device=dev)
    prm = make_params(n, d, k, p, metric, seed, join_path, _stream_ptr(dev), arena)
    st = ShardStats()
    _check(lib.gnnd_build_sharded_files(C.byref(prm), paths[0], shards, build_iters, merge_iters,
                                        paths[1], paths[2], staging.data_ptr(), staging.numel(),
                                        copy_stream.cuda_stream, C.byref(st)))
    return {f: getattr(st, f) for f, _ in st._fields_ if f != "reserved"}


def exact_knn(vectors, queries, K, metric=L2SQ_F32):
    """Exhaustive exact K-NN of the query nodes (evaluation ground truth)."""
    lib = load_library()
    _require_device(vectors, _elem_dtype(metric), "vectors")
    _require_device(queries, torch.int32, "queries")
    n, d = vectors.shape
    nq = queries.numel()
    ids = torch.empty((nq, K), dtype=torch.int32, device=vectors.device)
    dist = torch.empty((nq, K), dtype=_dist_dtype(metric), device=vectors.device)
    _check(lib.gnnd_exact_knn(vectors.data_ptr(), n, d, metric, queries.data_ptr(), nq, K,
                              ids.data_ptr(), dist.data_ptr(), _stream_ptr(vectors.device)))
    return ids, dist


def recall_at(graph_dist, truth_dist, K=10):
    """Recall@K (Sec. 6.1) of graph rows against exact rows of the same nodes: a
    listed neighbour among the first K is a true positive when its distance does
    not exceed the exact K-th distance (equal distances are interchangeable)."""
    gd = graph_dist[:, :K]
    kth = truth_dist[:, K - 1:K]
    return float((gd <= kth).sum().item()) / gd.numel()
