"""Host-side checks of the C ABI that need no GPU: the shared library loads, exports every
symbol include/slhc.h declares, sizes workspaces and rejects bad shapes."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def cdll():
    from paper_2306_16354_amd import binding, build
    if not os.path.exists(binding.library_path()):
        build.build_library(verbose=False)
    return binding.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "slhc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(slhc_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_expected_entry_points():
    names = declared_functions()
    for must in ("slhc_knn_graph", "slhc_slhc", "slhc_cross_1nn", "slhc_workspace_bytes",
                 "slhc_knn_workspace_bytes", "slhc_last_error", "slhc_strerror", "slhc_abi_version",
                 "slhc_knn_graph_opt", "slhc_slhc_opt", "slhc_flat_clusters", "slhc_fused_1nn", "slhc_csr_msf",
                 "slhc_flat_clusters_workspace_bytes", "slhc_fused_1nn_workspace_bytes",
                 "slhc_csr_msf_workspace_bytes", "slhc_knn_graph_static"):
        assert must in names


def test_every_declared_symbol_is_exported(cdll):
    for name in declared_functions():
        assert hasattr(cdll, name), f"{name} declared in slhc.h but not exported"


def test_version_and_strings(cdll):
    assert cdll.slhc_abi_version() == 4
    assert cdll.slhc_strerror(0) == b"ok"
    assert cdll.slhc_strerror(3) == b"workspace too small"
    assert cdll.slhc_strerror(5) == b"input not finite"
    assert cdll.slhc_strerror(6) == b"internal error"
    assert cdll.slhc_strerror(7) == b"host allocation failed"
    assert cdll.slhc_strerror(99) == b"unknown status"


def test_status_numbering_matches_the_header():
    text = open(os.path.join(ROOT, "include", "slhc.h")).read()
    values = dict(re.findall(r"\b(SLHC_[A-Z_]+)\s*=\s*(\d+)", text))
    assert values == {"SLHC_OK": "0", "SLHC_INVALID_ARG": "1", "SLHC_UNSUPPORTED": "2",
                      "SLHC_WORKSPACE_TOO_SMALL": "3", "SLHC_HIP_ERROR": "4", "SLHC_NONFINITE": "5",
                      "SLHC_INTERNAL": "6", "SLHC_HOST_MEMORY": "7"}
    assert re.search(r"#define SLHC_ABI_VERSION 4\b", text)
    assert re.search(r"#define SLHC_PRUNE 1u", text) and re.search(r"#define SLHC_SPLIT_ROUNDS 2u", text) and re.search(r"#define SLHC_SPLIT_SCANS 4u", text) and re.search(r"#define SLHC_NO_TILE_TABLE 8u", text) and re.search(r"#define SLHC_AUTO_PRUNE_MIN_ROWS 24576", text) and re.search(r"#define SLHC_FP32_FILTER 16u", text)


def test_no_exception_crosses_the_boundary():
    # every exported function that runs code of its own does so inside the library's exception guard
    src = open(os.path.join(ROOT, "paper_2306_16354_amd", "csrc", "slhc_api.hip")).read()
    block = src[src.index('extern "C" {'):src.index('}  // extern "C"')]
    bodies = re.findall(r"\nint (slhc_[a-z0-9_]+)\([^)]*\)\n\{\n(.*?)\n\}\n", block, flags=re.S)
    assert len(bodies) >= 14
    for name, body in bodies:
        assert body.lstrip().startswith("return guarded("), name


def test_workspace_sizes_and_shape_errors(cdll):
    out = ctypes.c_size_t(0)
    assert cdll.slhc_knn_workspace_bytes(1_000_000, 128, 32, ctypes.byref(out)) == 0
    assert out.value >= 4 * 1_000_000 and out.value % 256 == 0
    knn_bytes = out.value
    assert cdll.slhc_workspace_bytes(1_000_000, 128, 32, ctypes.byref(out)) == 0
    assert out.value >= knn_bytes + 8 * 32 * 1_000_000
    assert cdll.slhc_knn_workspace_bytes(1, 4, 1, ctypes.byref(out)) == 1          # N < 2
    assert cdll.slhc_knn_workspace_bytes(10, 0, 1, ctypes.byref(out)) == 1         # d < 1
    assert cdll.slhc_knn_workspace_bytes(10, 4, 10, ctypes.byref(out)) == 1        # k > N-1
    assert cdll.slhc_knn_workspace_bytes(1000, 4, 65, ctypes.byref(out)) == 2      # k > 64
    assert cdll.slhc_knn_workspace_bytes(1 << 30, 4, 8, ctypes.byref(out)) == 2    # N*k too large
    assert cdll.slhc_knn_workspace_bytes(10, 4, 2, None) == 1
    assert b"k" in cdll.slhc_last_error() or cdll.slhc_last_error() != b""


def test_workspace_holds_the_copy_with_zero_columns(cdll):
    """The k-NN and clustering entry points work on whole chunks of 32 columns up to 128 features and on a
    multiple of 4 beyond; the padded copy of X sits at the head of the workspace, so the size for d is the size
    for the padded d plus N x d' floats (rounded up to the 256-byte slices), and nothing where d already fits.
    Where the padded matrix would pass 2^31 - 1 elements the columns stay as they are."""
    out = ctypes.c_size_t(0)

    def size(fn, N, d, k):
        assert fn(N, d, k, ctypes.byref(out)) == 0, cdll.slhc_last_error()
        return out.value

    up = lambda b: (b + 255) // 256 * 256
    for fn in (cdll.slhc_knn_workspace_bytes, cdll.slhc_workspace_bytes):
        for N, d, dw, k in ((50_000, 100, 128, 16), (50_000, 7, 32, 5), (3001, 33, 64, 8), (20_000, 130, 132, 8),
                            (20_000, 785, 788, 16)):
            assert size(fn, N, d, k) == size(fn, N, dw, k) + up(N * dw * 4), (N, d, dw)
        # 8 columns padded to 32: 67 108 863 rows stay within the element limit and get the copy; one row more
        # is still accepted and laid out for 8 columns (no copy, and every array of d columns is a quarter the size)
        last = (2 ** 31 - 1) // 32
        assert size(fn, last, 8, 3) == size(fn, last, 32, 3) + up(last * 32 * 4)
        assert size(fn, last, 8, 3) - size(fn, last + 1, 8, 3) > last * 32 * 4


def test_null_pointers_are_rejected_before_any_device_work(cdll):
    assert cdll.slhc_knn_graph(None, 10, 4, 2, None, None, None, 0, None) == 1
    assert cdll.slhc_slhc(None, 10, 4, 2, None, None, None, None, None, None, None, None, 0, None) == 1
    assert cdll.slhc_knn_graph_static(None, 10, 4, 2, None, None, None) == 1
    assert cdll.slhc_cross_1nn(None, 10, 4, None, None, 5, None, None, None, 0, None) == 1


def test_later_entry_points_check_arguments_on_the_host(cdll):
    out = ctypes.c_size_t(0)
    # flat clusters
    assert cdll.slhc_flat_clusters_workspace_bytes(1_000_000, ctypes.byref(out)) == 0
    assert out.value >= 3 * 8 * 1_000_000 and out.value % 256 == 0
    assert cdll.slhc_flat_clusters_workspace_bytes(1, ctypes.byref(out)) == 1
    assert cdll.slhc_flat_clusters_workspace_bytes(1 << 30, ctypes.byref(out)) == 2
    assert cdll.slhc_flat_clusters(None, 10, 2, None, None, 0, None) == 1
    one = ctypes.c_int32(0)
    ptr = ctypes.cast(ctypes.pointer(one), ctypes.c_void_p)          # never dereferenced: checks come first
    assert cdll.slhc_flat_clusters(ptr, 10, 0, ptr, ptr, 1 << 20, None) == 1       # n_clusters < 1
    assert cdll.slhc_flat_clusters(ptr, 10, 11, ptr, ptr, 1 << 20, None) == 1      # n_clusters > N
    assert cdll.slhc_flat_clusters(ptr, 10, 2, ptr, ptr, 16, None) == 3            # workspace too small
    # fused 1-NN between two matrices
    assert cdll.slhc_fused_1nn_workspace_bytes(1000, 100_000, 128, ctypes.byref(out)) == 0
    assert out.value >= 4 * 101_000 + 8 * 1000
    assert cdll.slhc_fused_1nn_workspace_bytes(0, 10, 4, ctypes.byref(out)) == 1
    assert cdll.slhc_fused_1nn_workspace_bytes(10, 1 << 29, 8, ctypes.byref(out)) == 2
    assert cdll.slhc_fused_1nn(None, 10, None, 10, 4, None, None, None, 0, None) == 1
    assert cdll.slhc_fused_1nn(ptr, 10, ptr, 10, 4, ptr, ptr, ptr, 16, None) == 3
    # spanning forest of a CSR graph
    assert cdll.slhc_csr_msf_workspace_bytes(1_000_000, 2_500_000, ctypes.byref(out)) == 0
    assert out.value >= 60 * 1_000_000
    assert cdll.slhc_csr_msf_workspace_bytes(0, 0, ctypes.byref(out)) == 1
    assert cdll.slhc_csr_msf_workspace_bytes(10, -1, ctypes.byref(out)) == 1
    assert cdll.slhc_csr_msf_workspace_bytes(1 << 31, 10, ctypes.byref(out)) == 2
    assert cdll.slhc_csr_msf(None, None, None, 10, 5, None, None, None, None, None, None, None, 0, None) == 1
    n = ctypes.c_int64(0)
    assert cdll.slhc_csr_msf(ptr, ptr, ptr, 10, 5, ptr, ptr, ptr, ctypes.byref(n), ptr, None, ptr, 16, None) == 3
    assert b"workspace" in cdll.slhc_last_error()


def test_binding_refuses_cpu_tensors():
    import torch
    import paper_2306_16354_amd as slhc
    with pytest.raises(TypeError):
        slhc.knn_graph(torch.zeros((8, 4)), 2)
