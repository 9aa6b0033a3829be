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
                 "slhc_knn_workspace_bytes", "slhc_last_error", "slhc_strerror", "slhc_abi_version"):
        assert must in names


def test_every_declared_symbol_is_exported(cdll):
    for name in declared_functions():
        assert hasattr(cdll, name), f"{name} declared in slhc.h but not exported"


def test_version_and_strings(cdll):
    assert cdll.slhc_abi_version() == 1
    assert cdll.slhc_strerror(0) == b"ok"
    assert cdll.slhc_strerror(3) == b"workspace too small"
    assert cdll.slhc_strerror(99) == b"unknown status"


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


def test_null_pointers_are_rejected_before_any_device_work(cdll):
    assert cdll.slhc_knn_graph(None, 10, 4, 2, None, None, None, 0, None) == 1
    assert cdll.slhc_slhc(None, 10, 4, 2, None, None, None, None, None, None, None, None, 0, None) == 1
    assert cdll.slhc_cross_1nn(None, 10, 4, None, None, 5, None, None, None, 0, None) == 1


def test_binding_refuses_cpu_tensors():
    import torch
    import paper_2306_16354_amd as slhc
    with pytest.raises(TypeError):
        slhc.knn_graph(torch.zeros((8, 4)), 2)
