"""ctypes front end of the CPU oracle (``slhc_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()`` and by the
``cpu_baseline`` leg of ``bench.py``.  The product package never imports this module, and this
module imports nothing from the product package.

All distances are float64 values of sum_t (x_it - x_jt)^2 on the float32 inputs.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "slhc_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force=False):
    """Compile slhc_oracle.c with gcc + OpenMP into oracle/liboracle.so."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    cmd = ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared", "-std=c11",
           "-Wall", "-Wextra", "-o", _LIB + ".tmp", _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    os.replace(_LIB + ".tmp", _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        p = ctypes.c_void_p
        i64, i32 = ctypes.c_int64, ctypes.c_int32
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_knn_rows.argtypes = [p, i64, i32, i32, p, i64, p, p]
        lib.oracle_cross_1nn.argtypes = [p, i64, i32, p, p, i64, p, p]
        lib.oracle_mst_prim.argtypes = [p, i64, i32, p, p, p]
        lib.oracle_dendrogram.argtypes = [p, p, p, i64, p, p, p, p, p, p]
        lib.oracle_csr_msf.argtypes = [p, p, p, i64, p, p, p, p, p]
        for f in (lib.oracle_knn_rows, lib.oracle_cross_1nn, lib.oracle_mst_prim,
                  lib.oracle_dendrogram, lib.oracle_csr_msf):
            f.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads():
    return int(_load().oracle_num_threads())


def _f32(X):
    X = np.ascontiguousarray(X, dtype=np.float32)
    if X.ndim != 2:
        raise ValueError("X must be [N, d]")
    return X


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def knn_rows(X, rows, k):
    """k nearest neighbours (self excluded by index) of the given query rows against all of X.
    Returns (idx int32 [m,k], dist float64 [m,k]), ascending by (dist, idx)."""
    X = _f32(X)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    N, d = X.shape
    if rows.size and (rows.min() < 0 or rows.max() >= N):
        raise ValueError("row out of range")
    idx = np.empty((rows.size, k), dtype=np.int32)
    dist = np.empty((rows.size, k), dtype=np.float64)
    rc = _load().oracle_knn_rows(_ptr(X), N, d, k, _ptr(rows), rows.size, _ptr(idx), _ptr(dist))
    if rc != 0:
        raise ValueError(f"oracle_knn_rows: bad arguments (rc={rc})")
    return idx, dist


def knn_graph(X, k):
    """kNN graph of all rows of X."""
    X = _f32(X)
    return knn_rows(X, np.arange(X.shape[0], dtype=np.int64), k)


def cross_1nn(X, colour, rows):
    """Nearest differently-coloured point of each query row: (idx int32 [m], dist float64 [m]);
    idx -1 / dist inf where no such point exists."""
    X = _f32(X)
    colour = np.ascontiguousarray(colour, dtype=np.int32)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    N, d = X.shape
    if colour.shape != (N,):
        raise ValueError("colour must be [N]")
    idx = np.empty(rows.size, dtype=np.int32)
    dist = np.empty(rows.size, dtype=np.float64)
    rc = _load().oracle_cross_1nn(_ptr(X), N, d, _ptr(colour), _ptr(rows), rows.size,
                                  _ptr(idx), _ptr(dist))
    if rc != 0:
        raise ValueError(f"oracle_cross_1nn: bad arguments (rc={rc})")
    return idx, dist


def mst_prim(X):
    """Exact MST of the complete squared-L2 graph: (src, dst int32 [N-1], w float64 [N-1]) in
    Prim attachment order from vertex 0."""
    X = _f32(X)
    N, d = X.shape
    src = np.empty(N - 1, dtype=np.int32)
    dst = np.empty(N - 1, dtype=np.int32)
    w = np.empty(N - 1, dtype=np.float64)
    rc = _load().oracle_mst_prim(_ptr(X), N, d, _ptr(src), _ptr(dst), _ptr(w))
    if rc != 0:
        raise ValueError(f"oracle_mst_prim failed (rc={rc})")
    return src, dst, w


def dendrogram(src, dst, w, N):
    """Linkage arrays from N-1 tree edges.  Returns a dict with children int32 [N-1,2],
    heights float64 [N-1], sizes int32 [N-1] and the sorted edges (src < dst)."""
    src = np.ascontiguousarray(src, dtype=np.int32)
    dst = np.ascontiguousarray(dst, dtype=np.int32)
    w = np.ascontiguousarray(w, dtype=np.float64)
    if not (src.shape == dst.shape == w.shape == (N - 1,)):
        raise ValueError("need exactly N-1 edges")
    children = np.empty((N - 1, 2), dtype=np.int32)
    heights = np.empty(N - 1, dtype=np.float64)
    sizes = np.empty(N - 1, dtype=np.int32)
    ssrc = np.empty(N - 1, dtype=np.int32)
    sdst = np.empty(N - 1, dtype=np.int32)
    sw = np.empty(N - 1, dtype=np.float64)
    rc = _load().oracle_dendrogram(_ptr(src), _ptr(dst), _ptr(w), N, _ptr(children),
                                   _ptr(heights), _ptr(sizes), _ptr(ssrc), _ptr(sdst), _ptr(sw))
    if rc == -3:
        raise ValueError("edges contain a cycle")
    if rc != 0:
        raise ValueError(f"oracle_dendrogram failed (rc={rc})")
    return dict(children=children, heights=heights, sizes=sizes, src=ssrc, dst=sdst, w=sw)


def slhc(X):
    """MST + dendrogram of X (the whole oracle pipeline)."""
    X = _f32(X)
    src, dst, w = mst_prim(X)
    out = dendrogram(src, dst, w, X.shape[0])
    out["total_weight"] = float(np.sum(np.sort(w)))
    return out


def flat_clusters(children, n_clusters):
    """Flat clustering of a dendrogram into n_clusters clusters (cuSLINK paper Sec. 3.3.2,
    Alg. "extract_flattened_clusters" and Alg. "inherit_labels").

    The dendrogram is cut after its first N - n_clusters merges.  The nodes that exist at that
    level and have not been merged further are the cluster roots; they are numbered 0 .. n_clusters-1
    in ascending order of their node id (a leaf keeps its row id, merge i has id N+i), which is the
    paper's "sort the label roots", and every row gets the number of the root above it.

    children: int [N-1, 2] in linkage layout.  Returns labels int32 [N].  Plain union of the kept
    merges, written out; nothing here is shared with the GPU path."""
    children = np.asarray(children, dtype=np.int64)
    N = children.shape[0] + 1
    if not (1 <= n_clusters <= N):
        raise ValueError("need 1 <= n_clusters <= N")
    kept = N - n_clusters
    above = np.arange(2 * N - 1, dtype=np.int64)          # node directly above, or itself
    for i in range(kept):
        a, b = int(children[i, 0]), int(children[i, 1])
        if not (0 <= a < N + i and 0 <= b < N + i and a != b):
            raise ValueError("children do not form a dendrogram")
        above[a] = N + i
        above[b] = N + i
    labels = np.empty(N, dtype=np.int32)
    tops = np.empty(N, dtype=np.int64)
    for v in range(N):
        x = v
        while above[x] != x:
            x = int(above[x])
        tops[v] = x
    roots = np.unique(tops)
    if roots.size != n_clusters:
        raise ValueError("children do not form a dendrogram")
    labels[:] = np.searchsorted(roots, tops)
    return labels


def csr_msf(offsets, indices, weights):
    """Minimum spanning forest of an undirected CSR graph (paper Sec. 3.2), Kruskal under the strict
    edge order (w, lo, hi).  Returns (lo, hi, w) of the forest edges ascending in that order, and
    comp int32 [V] = smallest vertex id of each vertex's connected component."""
    offsets = np.ascontiguousarray(offsets, dtype=np.int32)
    indices = np.ascontiguousarray(indices, dtype=np.int32)
    weights = np.ascontiguousarray(weights, dtype=np.float32)
    V = offsets.shape[0] - 1
    if V < 1 or indices.shape != weights.shape or offsets[-1] != indices.shape[0]:
        raise ValueError("bad CSR arrays")
    lo = np.empty(max(V - 1, 1), dtype=np.int32)
    hi = np.empty(max(V - 1, 1), dtype=np.int32)
    w = np.empty(max(V - 1, 1), dtype=np.float32)
    comp = np.empty(V, dtype=np.int32)
    n = ctypes.c_int64(0)
    rc = _load().oracle_csr_msf(_ptr(offsets), _ptr(indices), _ptr(weights), V, _ptr(lo), _ptr(hi),
                                _ptr(w), ctypes.byref(n), _ptr(comp))
    if rc != 0:
        raise ValueError(f"oracle_csr_msf failed (rc={rc})")
    return lo[:n.value].copy(), hi[:n.value].copy(), w[:n.value].copy(), comp

