"""MI355X-native single-linkage clustering (the data-parallel path of cuSLINK).

Thin Python binding over the C ABI of ``libslhc.so`` (see ``include/slhc.h``): argument
marshalling only.  PyTorch supplies device memory and the current HIP stream; every step of the
computation runs in the library's own HIP kernels.  There is no CPU fallback: if the library has
not been built (``python -m paper_2306_16354_amd.build``) importing the binding's functions
raises.
"""
from .binding import (SlhcError, abi_version, cross_1nn, knn_graph, library_path, slhc,  # noqa: F401
                      knn_workspace_bytes, slhc_workspace_bytes, load_library, flat_clusters, fused_1nn, csr_msf,
                      flat_clusters_workspace_bytes, knn_graph_static, SLHC_STATIC_MAX_ROWS, probe_fp32_mfma, probe_bf16_mfma, probe_bf16_mfma_values,
                      probe_panel_loop)
