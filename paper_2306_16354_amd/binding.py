"""ctypes binding of libslhc.so.  Function names follow include/slhc.h without the prefix."""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libslhc.so")
_lib = None


class SlhcError(RuntimeError):
    def __init__(self, status, text, detail):
        super().__init__(f"slhc status {status} ({text}): {detail}")
        self.status = status


class _Stats(ctypes.Structure):
    _fields_ = [
        ("boruvka_rounds", ctypes.c_int32), ("connect_rounds", ctypes.c_int32),
        ("components_after_knn", ctypes.c_int32), ("order_pivots", ctypes.c_int32),
        ("knn_filter_survivors", ctypes.c_int64), ("connect_query_rows", ctypes.c_int64),
        ("connect_filter_survivors", ctypes.c_int64),
        ("ms_knn", ctypes.c_float), ("ms_boruvka", ctypes.c_float), ("ms_connect", ctypes.c_float),
        ("ms_sort", ctypes.c_float), ("ms_dendrogram", ctypes.c_float), ("ms_total", ctypes.c_float),
        ("ms_norm_kernel", ctypes.c_float), ("ms_knn_kernel", ctypes.c_float),
        ("ms_connect_kernels", ctypes.c_float), ("ms_order", ctypes.c_float),
        ("knn_tile_steps", ctypes.c_int64), ("connect_tile_steps", ctypes.c_int64),
        ("pruned", ctypes.c_int32), ("order_padded_rows", ctypes.c_int32),
        ("split_products", ctypes.c_int32), ("reserved0", ctypes.c_int32),
    ]

SLHC_PRUNE = 1
SLHC_SPLIT_ROUNDS = 2
SLHC_SPLIT_SCANS = 4
SLHC_NO_TILE_TABLE = 8
SLHC_FP32_FILTER = 16
SLHC_PANEL_ORDER = 32
SLHC_ONE_SHIFT = 64
SLHC_STATIC_MAX_ROWS = 1048576


def library_path():
    return _LIB_PATH


def load_library():
    """Load libslhc.so; raises if it has not been built.  Nothing here falls back to the CPU."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2306_16354_amd.build`")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_size_t
    lib.slhc_abi_version.restype = ctypes.c_int
    lib.slhc_strerror.restype = ctypes.c_char_p
    lib.slhc_strerror.argtypes = [ctypes.c_int]
    lib.slhc_last_error.restype = ctypes.c_char_p
    lib.slhc_knn_workspace_bytes.argtypes = [i64, i32, i32, ctypes.POINTER(sz)]
    lib.slhc_knn_graph.argtypes = [vp, i64, i32, i32, vp, vp, vp, sz, vp]
    lib.slhc_knn_graph_opt.argtypes = [vp, i64, i32, i32, vp, vp, vp, sz, vp, ctypes.c_uint32]
    lib.slhc_knn_graph_static.argtypes = [vp, i64, i32, i32, vp, vp, vp]
    lib.slhc_knn_graph_static.restype = ctypes.c_int
    lib.slhc_probe_fp32_mfma.argtypes = [ctypes.POINTER(ctypes.c_double), vp, sz, vp]
    lib.slhc_probe_fp32_mfma.restype = ctypes.c_int
    lib.slhc_probe_bf16_mfma.argtypes = [ctypes.POINTER(ctypes.c_double), vp, sz, vp]
    lib.slhc_probe_bf16_mfma.restype = ctypes.c_int
    lib.slhc_probe_bf16_mfma_values.argtypes = [vp, vp, vp, vp, ctypes.c_int32, vp]
    lib.slhc_probe_bf16_mfma_values.restype = ctypes.c_int
    lib.slhc_probe_panel_loop.argtypes = [i32, ctypes.POINTER(ctypes.c_double), vp, sz, vp]
    lib.slhc_probe_panel_loop.restype = ctypes.c_int
    lib.slhc_cross_1nn_workspace_bytes.argtypes = [i64, i32, i64, ctypes.POINTER(sz)]
    lib.slhc_cross_1nn.argtypes = [vp, i64, i32, vp, vp, i64, vp, vp, vp, sz, vp]
    lib.slhc_workspace_bytes.argtypes = [i64, i32, i32, ctypes.POINTER(sz)]
    lib.slhc_slhc.argtypes = [vp, i64, i32, i32, vp, vp, vp, vp, vp, vp, ctypes.POINTER(_Stats), vp, sz, vp]
    lib.slhc_slhc_opt.argtypes = lib.slhc_slhc.argtypes + [ctypes.c_uint32]
    lib.slhc_fused_1nn_workspace_bytes.argtypes = [i64, i64, i32, ctypes.POINTER(sz)]
    lib.slhc_fused_1nn.argtypes = [vp, i64, vp, i64, i32, vp, vp, vp, sz, vp]
    lib.slhc_fused_1nn_workspace_bytes.restype = ctypes.c_int
    lib.slhc_fused_1nn.restype = ctypes.c_int
    lib.slhc_csr_msf_workspace_bytes.argtypes = [i64, i64, ctypes.POINTER(sz)]
    lib.slhc_csr_msf.argtypes = [vp, vp, vp, i64, i64, vp, vp, vp, ctypes.POINTER(ctypes.c_int64), vp,
                                 ctypes.POINTER(ctypes.c_int32), vp, sz, vp]
    lib.slhc_csr_msf_workspace_bytes.restype = ctypes.c_int
    lib.slhc_csr_msf.restype = ctypes.c_int
    lib.slhc_flat_clusters_workspace_bytes.argtypes = [i64, ctypes.POINTER(sz)]
    lib.slhc_flat_clusters.argtypes = [vp, i64, i64, vp, vp, sz, vp]
    lib.slhc_flat_clusters_workspace_bytes.restype = ctypes.c_int
    lib.slhc_flat_clusters.restype = ctypes.c_int
    for name in ("slhc_knn_workspace_bytes", "slhc_knn_graph", "slhc_knn_graph_opt",
                 "slhc_cross_1nn_workspace_bytes", "slhc_cross_1nn", "slhc_workspace_bytes", "slhc_slhc",
                 "slhc_slhc_opt"):
        getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def _check(status):
    if status != 0:
        lib = load_library()
        raise SlhcError(status, lib.slhc_strerror(status).decode(), lib.slhc_last_error().decode())


def abi_version():
    return int(load_library().slhc_abi_version())


def _device_matrix(X):
    if not (isinstance(X, torch.Tensor) and X.is_cuda and X.dtype == torch.float32 and X.dim() == 2
            and X.is_contiguous()):
        raise TypeError("X must be a contiguous float32 CUDA tensor [N, d]")
    return X


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _workspace(nbytes, device):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def knn_workspace_bytes(N, d, k):
    out = ctypes.c_size_t(0)
    _check(load_library().slhc_knn_workspace_bytes(N, d, k, ctypes.byref(out)))
    return out.value


def slhc_workspace_bytes(N, d, k):
    out = ctypes.c_size_t(0)
    _check(load_library().slhc_workspace_bytes(N, d, k, ctypes.byref(out)))
    return out.value


def knn_graph(X, k, out=None, workspace=None, prune=False, tile_table=True, fp32_filter=False, panel_order=False,
              one_shift=False):
    """slhc_knn_graph (prune=False) / slhc_knn_graph_opt with SLHC_PRUNE: returns (idx int32 [N,k],
    dist float32 [N,k]) device tensors.  Asynchronous on the current stream."""
    X = _device_matrix(X)
    N, d = X.shape
    lib = load_library()
    if workspace is None:
        workspace = _workspace(knn_workspace_bytes(N, d, k), X.device)
    if out is None:
        idx = torch.empty((N, k), dtype=torch.int32, device=X.device)
        dist = torch.empty((N, k), dtype=torch.float32, device=X.device)
    else:
        idx, dist = out
    _check(lib.slhc_knn_graph_opt(X.data_ptr(), N, d, k, idx.data_ptr(), dist.data_ptr(),
                                  workspace.data_ptr(), workspace.numel(), _stream(),
                                  (SLHC_PRUNE if prune else 0) | (0 if tile_table else SLHC_NO_TILE_TABLE) |
                                  (SLHC_FP32_FILTER if fp32_filter else 0) | (SLHC_PANEL_ORDER if panel_order else 0) |
                                  (SLHC_ONE_SHIFT if one_shift else 0)))
    return idx, dist


def knn_graph_static(X, k, out):
    """slhc_knn_graph_static: slhc_knn_graph on the library's fixed scratch array; the caller passes the
    output tensors (idx int32 [N,k], dist float32 [N,k]) and nothing is allocated."""
    X = _device_matrix(X)
    N, d = X.shape
    idx, dist = out
    _check(load_library().slhc_knn_graph_static(X.data_ptr(), N, d, k, idx.data_ptr(), dist.data_ptr(), _stream()))
    return idx, dist


def probe_bf16_mfma_values(A, B, C):
    """slhc_probe_bf16_mfma_values: D[t] = C[t] + sum_k A[t, k] B[t, k] by one bf16 MFMA per row (A, B [T, 16], C [T])."""
    A, B, C = A.contiguous(), B.contiguous(), C.contiguous()
    assert A.dtype == B.dtype == C.dtype == torch.float32 and A.shape == B.shape and A.shape[1] == 16 and C.numel() == A.shape[0]
    D = torch.empty_like(C)
    _check(load_library().slhc_probe_bf16_mfma_values(A.data_ptr(), B.data_ptr(), C.data_ptr(), D.data_ptr(), A.shape[0], _stream()))
    return D


def probe_bf16_mfma(device="cuda"):
    """slhc_probe_bf16_mfma: TFLOP/s a register-only v_mfma_f32_32x32x16_bf16 loop sustains on the current device."""
    ws = _workspace(256, device)
    out = ctypes.c_double(0.0)
    _check(load_library().slhc_probe_bf16_mfma(ctypes.byref(out), ws.data_ptr(), ws.numel(), _stream()))
    return out.value


def probe_fp32_mfma(device="cuda"):
    """slhc_probe_fp32_mfma: TFLOP/s a register-only fp32 MFMA loop sustains on the current device."""
    ws = _workspace(256, device)
    out = ctypes.c_double(0.0)
    _check(load_library().slhc_probe_fp32_mfma(ctypes.byref(out), ws.data_ptr(), ws.numel(), _stream()))
    return out.value


def probe_panel_loop(steps, workspace):
    """slhc_probe_panel_loop: TFLOP/s of the multiplies with the panel loop's ingredients 0..steps.
    `workspace`: a CUDA tensor of finite float32 values to stream tiles from."""
    out = ctypes.c_double(0.0)
    _check(load_library().slhc_probe_panel_loop(int(steps), ctypes.byref(out), workspace.data_ptr(),
                                                workspace.numel() * workspace.element_size(), _stream()))
    return out.value


def cross_1nn(X, colour, rows=None, m=None):
    """slhc_cross_1nn: nearest row of another colour for each query row."""
    X = _device_matrix(X)
    N, d = X.shape
    if not (colour.is_cuda and colour.dtype == torch.int32 and colour.shape == (N,) and colour.is_contiguous()):
        raise TypeError("colour must be a contiguous int32 CUDA tensor [N]")
    if rows is not None:
        if not (rows.is_cuda and rows.dtype == torch.int32 and rows.dim() == 1 and rows.is_contiguous()):
            raise TypeError("rows must be a contiguous int32 CUDA tensor [m]")
        m = rows.numel()
    elif m is None:
        m = N
    lib = load_library()
    need = ctypes.c_size_t(0)
    _check(lib.slhc_cross_1nn_workspace_bytes(N, d, m, ctypes.byref(need)))
    ws = _workspace(need.value, X.device)
    idx = torch.empty(m, dtype=torch.int32, device=X.device)
    dist = torch.empty(m, dtype=torch.float32, device=X.device)
    _check(lib.slhc_cross_1nn(X.data_ptr(), N, d, colour.data_ptr(),
                              rows.data_ptr() if rows is not None else None, m,
                              idx.data_ptr(), dist.data_ptr(), ws.data_ptr(), ws.numel(), _stream()))
    return idx, dist


def slhc(X, k, workspace=None, out=None, prune=True, split_rounds=False, split_scans=False, tile_table=True,
         fp32_filter=False, panel_order=False, one_shift=False):
    """slhc_slhc: exact single-linkage MST and dendrogram.  Returns a dict of device tensors
    (mst_src, mst_dst, mst_w, children [N-1,2], heights, sizes) plus ``stats`` (a dict).
    ``workspace`` and ``out`` (a dict from an earlier call) may be passed in to reuse memory.
    prune=True asks for tile pruning (slhc_slhc_opt with SLHC_PRUNE), prune=False multiplies every tile
    (flags 0), prune=None is slhc_slhc, which prunes from 24 576 rows on;
    split_rounds adds SLHC_SPLIT_ROUNDS, split_scans SLHC_SPLIT_SCANS, tile_table=False SLHC_NO_TILE_TABLE."""
    X = _device_matrix(X)
    N, d = X.shape
    lib = load_library()
    if workspace is None:
        workspace = _workspace(slhc_workspace_bytes(N, d, k), X.device)
    dev = X.device
    out = out if out is not None else dict(
        mst_src=torch.empty(N - 1, dtype=torch.int32, device=dev),
        mst_dst=torch.empty(N - 1, dtype=torch.int32, device=dev),
        mst_w=torch.empty(N - 1, dtype=torch.float32, device=dev),
        children=torch.empty((N - 1, 2), dtype=torch.int32, device=dev),
        heights=torch.empty(N - 1, dtype=torch.float32, device=dev),
        sizes=torch.empty(N - 1, dtype=torch.int32, device=dev),
    )
    st = _Stats()
    if prune is None:
        _check(lib.slhc_slhc(X.data_ptr(), N, d, k, out["mst_src"].data_ptr(), out["mst_dst"].data_ptr(),
                             out["mst_w"].data_ptr(), out["children"].data_ptr(), out["heights"].data_ptr(),
                             out["sizes"].data_ptr(), ctypes.byref(st), workspace.data_ptr(),
                             workspace.numel(), _stream()))
    else:
        _check(lib.slhc_slhc_opt(X.data_ptr(), N, d, k, out["mst_src"].data_ptr(), out["mst_dst"].data_ptr(),
                                 out["mst_w"].data_ptr(), out["children"].data_ptr(), out["heights"].data_ptr(),
                                 out["sizes"].data_ptr(), ctypes.byref(st), workspace.data_ptr(),
                                 workspace.numel(), _stream(),
                                 (SLHC_PRUNE if prune else 0) | (SLHC_SPLIT_ROUNDS if split_rounds else 0) |
                                 (SLHC_SPLIT_SCANS if split_scans else 0) | (0 if tile_table else SLHC_NO_TILE_TABLE) |
                                 (SLHC_FP32_FILTER if fp32_filter else 0) | (SLHC_PANEL_ORDER if panel_order else 0) |
                                  (SLHC_ONE_SHIFT if one_shift else 0)))
    out["stats"] = {name: getattr(st, name) for name, _ in _Stats._fields_ if not name.startswith("reserved")}
    return out


def flat_clusters_workspace_bytes(N):
    out = ctypes.c_size_t(0)
    _check(load_library().slhc_flat_clusters_workspace_bytes(N, ctypes.byref(out)))
    return out.value


def flat_clusters(children, n_clusters, workspace=None, out=None):
    """slhc_flat_clusters: labels int32 [N] of the cut into n_clusters clusters.  `children` is the
    int32 CUDA tensor [N-1, 2] slhc() returns.  Asynchronous on the current stream."""
    if not (children.is_cuda and children.dtype == torch.int32 and children.dim() == 2
            and children.shape[1] == 2 and children.is_contiguous()):
        raise TypeError("children must be a contiguous int32 CUDA tensor [N-1, 2]")
    N = children.shape[0] + 1
    if workspace is None:
        workspace = _workspace(flat_clusters_workspace_bytes(N), children.device)
    if out is None:
        out = torch.empty(N, dtype=torch.int32, device=children.device)
    _check(load_library().slhc_flat_clusters(children.data_ptr(), N, int(n_clusters), out.data_ptr(),
                                             workspace.data_ptr(), workspace.numel(), _stream()))
    return out


def fused_1nn(Q, Y, workspace=None, out=None):
    """slhc_fused_1nn: for every row of Q the nearest row of Y: (idx int32 [m], dist float32 [m])."""
    Q = _device_matrix(Q)
    Y = _device_matrix(Y)
    m, d = Q.shape
    n, d2 = Y.shape
    if d != d2:
        raise ValueError("Q and Y must have the same number of columns")
    lib = load_library()
    if workspace is None:
        sz = ctypes.c_size_t(0)
        _check(lib.slhc_fused_1nn_workspace_bytes(m, n, d, ctypes.byref(sz)))
        workspace = _workspace(sz.value, Q.device)
    if out is None:
        out = (torch.empty(m, dtype=torch.int32, device=Q.device), torch.empty(m, dtype=torch.float32, device=Q.device))
    _check(lib.slhc_fused_1nn(Q.data_ptr(), m, Y.data_ptr(), n, d, out[0].data_ptr(), out[1].data_ptr(),
                              workspace.data_ptr(), workspace.numel(), _stream()))
    return out


def csr_msf(offsets, indices, weights, workspace=None):
    """slhc_csr_msf: minimum spanning forest of a symmetric CSR graph (int32 offsets [V+1], int32
    indices [E], float32 weights [E], CUDA tensors).  Returns a dict with mst_src, mst_dst, mst_w
    (the forest edges, ascending by (w, src, dst)), colours [V] and rounds.  Synchronous."""
    for t, dt in ((offsets, torch.int32), (indices, torch.int32), (weights, torch.float32)):
        if not (t.is_cuda and t.dtype == dt and t.dim() == 1 and t.is_contiguous()):
            raise TypeError("offsets/indices must be int32 and weights float32 contiguous CUDA vectors")
    V = offsets.numel() - 1
    E = indices.numel()
    if weights.numel() != E:
        raise ValueError("indices and weights differ in length")
    lib = load_library()
    if workspace is None:
        sz = ctypes.c_size_t(0)
        _check(lib.slhc_csr_msf_workspace_bytes(V, E, ctypes.byref(sz)))
        workspace = _workspace(sz.value, offsets.device)
    cap = max(V - 1, 1)
    src = torch.empty(cap, dtype=torch.int32, device=offsets.device)
    dst = torch.empty(cap, dtype=torch.int32, device=offsets.device)
    w = torch.empty(cap, dtype=torch.float32, device=offsets.device)
    colours = torch.empty(max(V, 1), dtype=torch.int32, device=offsets.device)
    n = ctypes.c_int64(0)
    rounds = ctypes.c_int32(0)
    _check(lib.slhc_csr_msf(offsets.data_ptr(), indices.data_ptr() if E else None, weights.data_ptr() if E else None,
                            V, E, src.data_ptr(), dst.data_ptr(), w.data_ptr(), ctypes.byref(n),
                            colours.data_ptr(), ctypes.byref(rounds), workspace.data_ptr(), workspace.numel(),
                            _stream()))
    return dict(mst_src=src[:n.value], mst_dst=dst[:n.value], mst_w=w[:n.value], colours=colours,
                rounds=rounds.value)

