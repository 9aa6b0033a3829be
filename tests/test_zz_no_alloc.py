"""slhc_knn_graph_static (the entry point that allocates nothing: its scratch is a fixed device array
inside the library) against slhc_knn_graph, through the C ABI, bit for bit: two calls in a row on the
same GPU, the second with a smaller input, so that what the first call left in the shared array must
not matter."""
import ctypes

import numpy as np
import pytest

import slhc_inputs as gen

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def test_static_scratch_knn_equals_workspace_knn():
    import paper_2306_16354_amd as slhc
    lib = slhc.load_library()
    assert torch.cuda.is_available()
    results = []
    for name, n, k in (("c2", 30_000, 32), ("c1", 3_000, 7)):        # the second input is smaller
        X, _, _ = gen.make(name, n=n)
        N, d = X.shape
        print(f"static scratch knn {name} N={N} d={d} k={k}", flush=True)
        Xd = torch.from_numpy(X).cuda()
        idx = torch.full((N, k), -7, dtype=torch.int32, device="cuda")
        dist = torch.full((N, k), -7.0, dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        rc = lib.slhc_knn_graph_static(Xd.data_ptr(), N, d, k, idx.data_ptr(), dist.data_ptr(),
                                       ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
        assert rc == 0, lib.slhc_last_error()
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        results.append((Xd, k, idx, dist))
    for Xd, k, idx, dist in results:                                  # the reference entry point, afterwards
        ref_idx, ref_dist = slhc.knn_graph(Xd, k)
        torch.cuda.synchronize()
        assert torch.equal(idx, ref_idx) and torch.equal(dist, ref_dist)
    # the larger input once more after the smaller one: stale half norms beyond the smaller N are overwritten
    Xd, k, idx, dist = results[0]
    again_i, again_d = torch.empty_like(idx), torch.empty_like(dist)
    slhc.knn_graph_static(Xd, k, (again_i, again_d))
    torch.cuda.synchronize()
    assert torch.equal(idx, again_i) and torch.equal(dist, again_d)


def test_static_scratch_rejects_oversize():
    import paper_2306_16354_amd as slhc
    lib = slhc.load_library()
    N = slhc.SLHC_STATIC_MAX_ROWS + 1
    one = ctypes.c_int32(0)
    ptr = ctypes.cast(ctypes.pointer(one), ctypes.c_void_p)          # never dereferenced: the size check comes first
    assert lib.slhc_knn_graph_static(ptr, N, 4, 2, ptr, ptr, None) == 2
    assert b"SLHC_STATIC_MAX_ROWS" in lib.slhc_last_error()
    assert lib.slhc_knn_graph_static(None, 100, 4, 2, ptr, ptr, None) == 1
