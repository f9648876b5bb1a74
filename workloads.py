"""Seeded synthetic inputs for the k-NN graph construction workloads.

This module only draws input vectors.  It holds none of the graph
construction arithmetic (no distances, no hashing of node ids, no sampling)
and is the one piece of code the CPU oracle's tests and the GPU path's tests
both use, so that both sides always see the very same bytes.

The paper evaluates on public descriptor collections (Table 1: SIFT, GIST,
DEEP); those files are not available, so each generator below produces vectors
with the same n x d shape, value range and clustered structure as a stand-in.
"""
from __future__ import annotations

import numpy as np

# Algorithm seed used by every benchmark / parity configuration.
ALGO_SEED = 42


def _mixture(rng, n, d, n_comp, centre_fn, sigma, chunk=1 << 16):
    centres = centre_fn((n_comp, d)).astype(np.float32)
    comp = rng.integers(0, n_comp, size=n)
    out = np.empty((n, d), dtype=np.float32)
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        noise = rng.standard_normal((hi - lo, d), dtype=np.float32)
        out[lo:hi] = centres[comp[lo:hi]] + np.float32(sigma) * noise
    return out


def uniform_f32(n=4096, d=16, seed=1001):
    """Config 'uniform': i.i.d. U[0,1) float32 (the small parity workload)."""
    rng = np.random.default_rng(seed)
    return rng.random((n, d), dtype=np.float32)


def sift_like_f32(n=1_000_000, d=128, seed=1002, n_comp=256):
    """SIFT-shaped: Gaussian mixture, centres U[0,128]^d, sigma 20 per
    dimension, clipped to [0,255] and rounded to integer values (float32)."""
    rng = np.random.default_rng(seed)
    x = _mixture(rng, n, d, n_comp, lambda s: rng.uniform(0.0, 128.0, size=s), 20.0)
    np.clip(x, 0.0, 255.0, out=x)
    np.rint(x, out=x)
    return x


def sift_like_u8(n=1_000_000, d=128, seed=1005, n_comp=64):
    """Byte-valued SIFT-shaped vectors (the merge workload's element type)."""
    return sift_like_f32(n, d, seed, n_comp).astype(np.uint8)


def gist_like_f32(n=1_000_000, d=960, seed=1003, n_comp=128):
    """GIST-shaped: mixture with N(0,1) centres, sigma 0.3, abs(), then each
    vector L1-normalised: small non-negative entries."""
    rng = np.random.default_rng(seed)
    x = _mixture(rng, n, d, n_comp, lambda s: rng.standard_normal(s), 0.3)
    np.abs(x, out=x)
    x /= x.sum(axis=1, keepdims=True, dtype=np.float32)
    return x


def deep_like_f32(n=10_000_000, d=96, seed=1004, n_comp=1024):
    """DEEP-shaped: mixture with N(0,1) centres, sigma 0.5, each vector
    L2-normalised to unit length (used with the angular metric)."""
    rng = np.random.default_rng(seed)
    x = _mixture(rng, n, d, n_comp, lambda s: rng.standard_normal(s), 0.5)
    nrm = np.sqrt((x * x).sum(axis=1, keepdims=True, dtype=np.float32))
    x /= nrm
    return x


def scaled_directions_f32(n, d, seed, n_comp=16, zero_rows=0):
    """Vectors of very different lengths (for the cosine distance): DEEP-shaped
    directions times log-uniform lengths in [0.05, 40); the first `zero_rows`
    rows are zero vectors."""
    x = deep_like_f32(n, d, seed=seed, n_comp=n_comp)
    rng = np.random.default_rng(seed + 7)
    x *= np.exp(rng.uniform(np.log(0.05), np.log(40.0), size=(n, 1))).astype(np.float32)
    x[:zero_rows] = 0.0
    return np.ascontiguousarray(x, dtype=np.float32)


def near_copies_f32(n, d, seed, copies=8, jitter=1e-6):
    """Groups of `copies` almost identical vectors: n / copies uniform vectors, each
    repeated `copies` times, half of the repeats exactly, the others moved by a relative
    `jitter` per coordinate.  Many partners of a sample are then equally near, or nearer
    than float32 inner products can tell apart: ties by id and near-ties everywhere."""
    rng = np.random.default_rng(seed)
    base = rng.random((-(-n // copies), d), dtype=np.float32)
    x = np.repeat(base, copies, axis=0)[:n].copy()
    moved = (np.arange(n) % copies) >= copies // 2
    x[moved] *= (1.0 + jitter * rng.standard_normal((int(moved.sum()), d))).astype(np.float32)
    return np.ascontiguousarray(x[rng.permutation(n)], dtype=np.float32)


def small_integer_f32(n, d, seed, hi=16):
    """Tiny integer-valued float vectors: every distance is an exact small
    integer in any summation order (handy for exact pins)."""
    rng = np.random.default_rng(seed)
    return rng.integers(0, hi, size=(n, d)).astype(np.float32)


def sample_nodes(n, m, seed=7):
    """m distinct node ids out of n (sorted), for sampled recall evaluation."""
    rng = np.random.default_rng(seed)
    m = min(m, n)
    return np.sort(rng.choice(n, size=m, replace=False)).astype(np.int32)
