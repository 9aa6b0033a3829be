// Flat clusters from a dendrogram: cut after the first N - n_clusters merges, number the surviving
// roots by ascending node id, give every row the number of the root above it (paper Sec. 3.3.2,
// Alg. "extract_flattened_clusters", Alg. "inherit_labels").
//
// The paper's inherit_labels lets every node walk up its parents until it meets a labelled one.
// Single-linkage dendrograms are often chains thousands of levels deep, so here the walk is
// pointer doubling instead: ceil(log2(2N)) passes of above[v] = above[above[v]] over all nodes,
// each pass one coalesced read-modify-write of 8N bytes - HBM-bound and independent of the depth.
// The paper finds the roots by sorting the children of the last merges; here a node is a root iff
// it exists at the cut and nothing kept points above it, and the numbering is an exclusive prefix
// sum of that flag over the node ids (the same ascending order, no sort).
#include <hip/hip_runtime.h>
#include <cstring>
#include <rocprim/rocprim.hpp>
#include <stdint.h>
#include "cluster_kernels.h"

namespace slhc {

constexpr int TB = 256;
static inline int blocks_for(long long n) { return (int)((n + TB - 1) / TB); }

__global__ void __launch_bounds__(TB) k_above_self(int32_t* __restrict__ above, int nodes)
{
    const int v = blockIdx.x * TB + threadIdx.x;
    if (v < nodes) above[v] = v;
}

// merge i < kept puts node N+i above its two children
__global__ void __launch_bounds__(TB) k_above_kept(const int32_t* __restrict__ children, int N, int kept,
                                                   int32_t* __restrict__ above)
{
    const int i = blockIdx.x * TB + threadIdx.x;
    if (i >= kept) return;
    const int a = children[2 * i], b = children[2 * i + 1];
    // a well-formed dendrogram only joins nodes that already exist; anything else is ignored
    if ((unsigned int)a < (unsigned int)(N + i)) above[a] = N + i;
    if ((unsigned int)b < (unsigned int)(N + i)) above[b] = N + i;
}

// flag[v] = 1 for the nodes that exist at the cut (v < N + kept) and have nothing above them
__global__ void __launch_bounds__(TB) k_root_flags(const int32_t* __restrict__ above, int limit, int nodes,
                                                   int32_t* __restrict__ flag)
{
    const int v = blockIdx.x * TB + threadIdx.x;
    if (v < nodes) flag[v] = (v < limit && above[v] == v) ? 1 : 0;
}

// one doubling step; reading a value another thread has already advanced only gets there sooner
__global__ void __launch_bounds__(TB) k_above_double(int32_t* __restrict__ above, int nodes)
{
    const int v = blockIdx.x * TB + threadIdx.x;
    if (v >= nodes) return;
    const int a = above[v];
    if ((unsigned int)a < (unsigned int)nodes) {
        const int aa = above[a];
        if (aa != a) above[v] = aa;
    }
}

__global__ void __launch_bounds__(TB) k_labels(const int32_t* __restrict__ above, const int32_t* __restrict__ rank,
                                               int N, int nodes, int32_t* __restrict__ labels)
{
    const int v = blockIdx.x * TB + threadIdx.x;
    if (v >= N) return;
    const int r = above[v];
    labels[v] = (unsigned int)r < (unsigned int)nodes ? rank[r] : -1;
}

size_t flat_clusters_scan_temp_bytes(int N)
{
    size_t bytes = 0;
    const int32_t* in = nullptr;
    int32_t* out = nullptr;
    (void)rocprim::exclusive_scan(nullptr, bytes, in, out, 0, (size_t)(2 * (size_t)N), rocprim::plus<int32_t>());
    return bytes;
}

hipError_t flat_clusters(const int32_t* children, int N, int n_clusters, int32_t* labels, int32_t* above,
                         int32_t* flag, int32_t* rank, void* scan_temp, size_t scan_temp_bytes, hipStream_t s)
{
    const int nodes = 2 * N - 1;
    const int kept = N - n_clusters;
    hipLaunchKernelGGL(k_above_self, dim3(blocks_for(nodes)), dim3(TB), 0, s, above, nodes);
    if (kept > 0)
        hipLaunchKernelGGL(k_above_kept, dim3(blocks_for(kept)), dim3(TB), 0, s, children, N, kept, above);
    hipLaunchKernelGGL(k_root_flags, dim3(blocks_for(nodes)), dim3(TB), 0, s, above, N + kept, nodes, flag);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    e = rocprim::exclusive_scan(scan_temp, scan_temp_bytes, flag, rank, 0, (size_t)nodes, rocprim::plus<int32_t>(), s);
    if (e != hipSuccess) return e;
    int rounds = 1;
    while ((1LL << rounds) < (long long)nodes) ++rounds;
    for (int r = 0; r < rounds; ++r)
        hipLaunchKernelGGL(k_above_double, dim3(blocks_for(nodes)), dim3(TB), 0, s, above, nodes);
    hipLaunchKernelGGL(k_labels, dim3(blocks_for(N)), dim3(TB), 0, s, above, rank, N, nodes, labels);
    return hipGetLastError();
}

}  // namespace slhc
