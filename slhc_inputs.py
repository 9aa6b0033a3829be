"""Seeded synthetic point sets shaped like the workloads single-linkage clustering is run on.

This module only draws random inputs.  It holds none of the method's arithmetic (no distances,
no neighbour search, no trees) so that the CPU oracle and the HIP path can both take their
inputs from it without sharing anything else.

Every generator returns ``(X, labels)``: ``X`` is a C-contiguous float32 array [N, d]
(drawn in float64, then rounded once), ``labels`` an int32 array [N] with the id of the blob /
class template each row was drawn from (for duplicates: the label of the copied row).  Rows
are shuffled by a seeded permutation so that the row order carries no information about the
blob structure.

Named workloads (``make("c1") .. make("c5")``); ``n`` overrides the row count and the number
of blobs is scaled with it so that the per-blob population, and therefore the neighbourhood
structure, stays what it is at full size:

  c1  N=4,096     d=16   10 equal isotropic Gaussian blobs, centres U[-10,10]^d, std 1      k=16
  c2  N=100,000   d=64   50 equal blobs, centres U[-20,20]^d, per-blob std U[0.5,2.0]       k=32
  c3  N=1,000,000 d=128  1000 blobs, centres U[-50,50]^d, std 1, Zipf(1.1) blob sizes       k=32
  c4  N=250,000   d=784  image-like rows: 10 class templates (Bernoulli(0.2) masks), 80 %
                         of entries exactly 0, nonzeros U(0,1]                              k=16
  c5  N=2,000,000 d=32   20,000 tight blobs (std 0.1, centres U[-1000,1000]^d) plus 1 %
                         bit-exact duplicate rows                                           k=8
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 20230616

WORKLOADS = {
    "c1": dict(N=4096, d=16, k=16, blobs=10),
    "c2": dict(N=100_000, d=64, k=32, blobs=50),
    "c3": dict(N=1_000_000, d=128, k=32, blobs=1000),
    "c4": dict(N=250_000, d=784, k=16, blobs=10),
    "c5": dict(N=2_000_000, d=32, k=8, blobs=20_000),
}


def _rng(seed):
    return np.random.default_rng(np.random.PCG64(seed))


def _gauss_rows(rng, centres, stds, sizes, d):
    """Rows of blob b are centres[b] + stds[b] * N(0, I); drawn blob by blob in float64."""
    N = int(np.sum(sizes))
    X = np.empty((N, d), dtype=np.float32)
    labels = np.empty(N, dtype=np.int32)
    pos = 0
    for b, m in enumerate(sizes):
        m = int(m)
        if m == 0:
            continue
        block = rng.standard_normal((m, d)) * stds[b] + centres[b]
        X[pos:pos + m] = block.astype(np.float32)
        labels[pos:pos + m] = b
        pos += m
    return X, labels


def _shuffle(rng, X, labels):
    perm = rng.permutation(X.shape[0])
    return np.ascontiguousarray(X[perm]), np.ascontiguousarray(labels[perm])


def equal_sizes(N, blobs):
    base, rem = divmod(N, blobs)
    sizes = np.full(blobs, base, dtype=np.int64)
    sizes[:rem] += 1
    return sizes


def zipf_sizes(N, blobs, exponent=1.1):
    """Blob b (1-based) gets a share proportional to b**-exponent; floors, remainder to blob 1."""
    w = np.arange(1, blobs + 1, dtype=np.float64) ** (-exponent)
    sizes = np.floor(N * w / w.sum()).astype(np.int64)
    sizes[0] += N - sizes.sum()
    return sizes


def blobs_equal(N, d, blobs, box, std, seed, shuffle=True):
    rng = _rng(seed)
    centres = rng.uniform(-box, box, size=(blobs, d))
    stds = np.full(blobs, float(std))
    X, labels = _gauss_rows(rng, centres, stds, equal_sizes(N, blobs), d)
    return _shuffle(rng, X, labels) if shuffle else (X, labels)


def blobs_varstd(N, d, blobs, box, std_lo, std_hi, seed, shuffle=True):
    rng = _rng(seed)
    centres = rng.uniform(-box, box, size=(blobs, d))
    stds = rng.uniform(std_lo, std_hi, size=blobs)
    X, labels = _gauss_rows(rng, centres, stds, equal_sizes(N, blobs), d)
    return _shuffle(rng, X, labels) if shuffle else (X, labels)


def blobs_zipf(N, d, blobs, box, std, seed, exponent=1.1, shuffle=True):
    rng = _rng(seed)
    centres = rng.uniform(-box, box, size=(blobs, d))
    stds = np.full(blobs, float(std))
    X, labels = _gauss_rows(rng, centres, stds, zipf_sizes(N, blobs, exponent), d)
    return _shuffle(rng, X, labels) if shuffle else (X, labels)


def image_like(N, d, classes, seed, template_density=0.2, keep=0.9, flip_on=0.025, shuffle=True):
    """Sparse non-negative rows: a row of class c has a pixel on with probability ``keep`` where
    the class template is on and ``flip_on`` where it is off; on-pixels are fresh U(0,1] values,
    everything else is exactly 0 (overall density 0.2*0.9 + 0.8*0.025 = 0.20)."""
    rng = _rng(seed)
    templates = rng.random((classes, d)) < template_density
    labels = rng.integers(0, classes, size=N).astype(np.int32)
    X = np.empty((N, d), dtype=np.float32)
    chunk = 16384
    for s in range(0, N, chunk):
        e = min(N, s + chunk)
        t = templates[labels[s:e]]
        p_on = np.where(t, keep, flip_on)
        on = rng.random((e - s, d)) < p_on
        vals = 1.0 - rng.random((e - s, d))          # (0, 1]
        X[s:e] = np.where(on, vals, 0.0).astype(np.float32)
    return _shuffle(rng, X, labels) if shuffle else (X, labels)


def tight_blobs_with_duplicates(N, d, blobs, box, std, dup_fraction, seed, shuffle=True):
    """(1 - dup_fraction) N rows in equal tight blobs, then dup_fraction N rows that are bit-exact
    copies of uniformly chosen earlier rows."""
    rng = _rng(seed)
    n_dup = int(round(N * dup_fraction))
    n_base = N - n_dup
    centres = rng.uniform(-box, box, size=(blobs, d))
    stds = np.full(blobs, float(std))
    Xb, lb = _gauss_rows(rng, centres, stds, equal_sizes(n_base, blobs), d)
    src = rng.integers(0, n_base, size=n_dup)
    X = np.concatenate([Xb, Xb[src]], axis=0)
    labels = np.concatenate([lb, lb[src]], axis=0)
    return _shuffle(rng, X, labels) if shuffle else (X, labels)


def make(name, n=None, shuffle=True, seed_offset=0):
    """Workload ``name`` ("c1".."c5"), optionally scaled to ``n`` rows.  Returns (X, labels, k)."""
    cfg = WORKLOADS[name]
    N = cfg["N"] if n is None else int(n)
    d, k = cfg["d"], cfg["k"]
    seed = BASE_SEED + int(name[1:]) + 1000 * seed_offset
    scale = N / cfg["N"]
    if name == "c4":
        blobs = cfg["blobs"]
    else:
        blobs = max(2, int(round(cfg["blobs"] * scale)))
        blobs = min(blobs, max(2, N // (k + 2)))
    if name == "c1":
        X, y = blobs_equal(N, d, blobs, 10.0, 1.0, seed, shuffle)
    elif name == "c2":
        X, y = blobs_varstd(N, d, blobs, 20.0, 0.5, 2.0, seed, shuffle)
    elif name == "c3":
        X, y = blobs_zipf(N, d, blobs, 50.0, 1.0, seed, 1.1, shuffle)
    elif name == "c4":
        X, y = image_like(N, d, blobs, seed, shuffle=shuffle)
    elif name == "c5":
        X, y = tight_blobs_with_duplicates(N, d, blobs, 1000.0, 0.1, 0.01, seed, shuffle)
    else:
        raise KeyError(name)
    return X, y, k


def uniform_cube(N, d, seed):
    """N rows uniform in [0,1)^d (the 'randomly generated data' of the paper's kNN tables)."""
    return _rng(seed).random((N, d)).astype(np.float32)


def integer_lattice(side, d, seed=None):
    """All points of {0..side-1}^d as float32 (side**d rows); optionally row-shuffled.  Every
    squared distance is a small exact integer in float32 and float64 alike."""
    grids = np.meshgrid(*[np.arange(side)] * d, indexing="ij")
    X = np.stack([g.ravel() for g in grids], axis=1).astype(np.float32)
    if seed is not None:
        X = X[_rng(seed).permutation(X.shape[0])]
    return np.ascontiguousarray(X)


def increasing_gaps_line(N, d, seed=None):
    """Collinear points at positions 0, 1, 3, 6, 10, ... (gap i+1 before point i+1) along the
    first axis, zero elsewhere; optionally row-shuffled.  Returns (X, position)."""
    pos = np.cumsum(np.arange(N, dtype=np.float64))
    X = np.zeros((N, d), dtype=np.float32)
    X[:, 0] = pos
    if seed is not None:
        perm = _rng(seed).permutation(N)
        X, pos = X[perm], pos[perm]
    return np.ascontiguousarray(X), pos


def road_graph(side, seed, keep=0.625, integer_weights=False):
    """Planar road-like graph: the vertices of a side x side grid, each of the 4-neighbour links kept
    with probability `keep` (average degree 4 * keep = 2.5, as in road networks; the graph is usually
    not connected), vertex ids shuffled.  Weights are uniform in [1, 100) (float32), or integers
    1..10 when integer_weights is set (many ties).  Returns symmetric CSR arrays
    (offsets int32 [V+1], indices int32 [E], weights float32 [E]); every undirected edge is stored
    in both rows with the same weight."""
    rng = _rng(seed)
    V = side * side
    ids = np.arange(V, dtype=np.int64).reshape(side, side)
    a = np.concatenate([ids[:, :-1].ravel(), ids[:-1, :].ravel()])
    b = np.concatenate([ids[:, 1:].ravel(), ids[1:, :].ravel()])
    kept = rng.random(a.shape[0]) < keep
    a, b = a[kept], b[kept]
    if integer_weights:
        w = rng.integers(1, 11, size=a.shape[0]).astype(np.float32)
    else:
        w = (1.0 + 99.0 * rng.random(a.shape[0])).astype(np.float32)
    relabel = rng.permutation(V)
    a, b = relabel[a], relabel[b]
    src = np.concatenate([a, b])
    dst = np.concatenate([b, a])
    ww = np.concatenate([w, w])
    order = np.lexsort((dst, src))
    src, dst, ww = src[order], dst[order], ww[order]
    offsets = np.zeros(V + 1, dtype=np.int64)
    np.add.at(offsets, src + 1, 1)
    offsets = np.cumsum(offsets)
    return offsets.astype(np.int32), dst.astype(np.int32), np.ascontiguousarray(ww, dtype=np.float32)

