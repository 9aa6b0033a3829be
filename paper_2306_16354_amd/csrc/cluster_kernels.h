// Flat clusters from a dendrogram (cluster_kernels.hip): paper Sec. 3.3.2, Alg.
// "extract_flattened_clusters" and Alg. "inherit_labels".
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace slhc {

// Scratch of flat_clusters: `above`, `flag` and `rank` of 2N words each, plus the scan's own temporary.
size_t flat_clusters_scan_temp_bytes(int N);

// labels[v] for v < N: number of the cluster root above row v when the dendrogram is cut after
// its first N - n_clusters merges; roots are numbered in ascending order of their node id.
// children: [N-1, 2] linkage layout (ids below N are rows, N+i is merge i).
hipError_t flat_clusters(const int32_t* children, int N, int n_clusters, int32_t* labels,
                         int32_t* above, int32_t* flag, int32_t* rank, void* scan_temp,
                         size_t scan_temp_bytes, hipStream_t s);

}  // namespace slhc
