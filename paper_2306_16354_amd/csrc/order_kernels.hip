// Row reordering helpers and tile bounding balls for the pruned sweeps.  All HBM-bound, one pass.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "order_kernels.h"

namespace slhc {

constexpr int TB = 256;
constexpr int TILE = 128;          // rows per candidate tile of the sweep kernels
static inline int blocks_for(long long n) { return (int)((n + TB - 1) / TB); }

__global__ void __launch_bounds__(TB) k_iota(int32_t* a, int n)
{
    const int i = blockIdx.x * TB + threadIdx.x;
    if (i < n) a[i] = i;
}

// one thread per output float4 (or float when d is not a multiple of 4)
template <bool VEC4>
__global__ void __launch_bounds__(TB) k_gather_rows(const float* __restrict__ X, const int32_t* __restrict__ perm,
                                                    int N, int d, int P, float* __restrict__ Xs)
{
    const int per_row = VEC4 ? d / 4 : d;
    const long long i = (long long)blockIdx.x * TB + threadIdx.x;
    const long long total = (long long)(perm ? N : P) * per_row;
    if (i >= total) return;
    const int r = (int)(i / per_row), c = (int)(i % per_row);
    const int src = perm ? perm[r] : (int)((long long)r * N / P);
    if ((unsigned int)src >= (unsigned int)N) return;
    if (VEC4) reinterpret_cast<float4*>(Xs)[i] = reinterpret_cast<const float4*>(X + (size_t)src * d)[c];
    else Xs[i] = X[(size_t)src * d + c];
}

__global__ void __launch_bounds__(TB) k_pick_f32(const float* __restrict__ a, int N, int P, float* __restrict__ out)
{
    const int j = blockIdx.x * TB + threadIdx.x;
    if (j < P) out[j] = a[(int)((long long)j * N / P)];
}

template <typename T>
__global__ void __launch_bounds__(TB) k_gather(const T* __restrict__ a, const int32_t* __restrict__ idx, int n,
                                               int limit, T fallback, T* __restrict__ out)
{
    const int i = blockIdx.x * TB + threadIdx.x;
    if (i >= n) return;
    const int j = idx[i];
    out[i] = (unsigned int)j < (unsigned int)limit ? a[j] : fallback;
}

// key[i] = 0 where dist[i] > tau (a row far from every pivot), else 1; *count += number of zeros
__global__ void __launch_bounds__(TB) k_mark_far(const float* __restrict__ dist, int n, float tau,
                                                 uint32_t* __restrict__ key, int32_t* __restrict__ count)
{
    const int i = blockIdx.x * TB + threadIdx.x;
    const bool far = i < n && dist[i] > tau;
    if (i < n) key[i] = far ? 0u : 1u;
    const unsigned long long mask = __ballot(far);
    if (mask && (threadIdx.x & 63) == (unsigned int)__builtin_ctzll(mask)) atomicAdd(count, __popcll(mask));
}

// Xp[j] = X[list[floor(j * m / P)]], hp likewise: P evenly spaced entries of a row list of length m
template <bool VEC4>
__global__ void __launch_bounds__(TB) k_pick_listed(const float* __restrict__ X, const float* __restrict__ h,
                                                    const uint32_t* __restrict__ list, int m, int N, int d, int P,
                                                    float* __restrict__ Xp, float* __restrict__ hp)
{
    const int per_row = VEC4 ? d / 4 : d;
    const long long i = (long long)blockIdx.x * TB + threadIdx.x;
    if (i >= (long long)P * per_row) return;
    const int r = (int)(i / per_row), c = (int)(i % per_row);
    const uint32_t src = list[(int)((long long)r * m / P)];
    if (src >= (uint32_t)N) return;
    if (VEC4) reinterpret_cast<float4*>(Xp)[i] = reinterpret_cast<const float4*>(X + (size_t)src * d)[c];
    else Xp[i] = X[(size_t)src * d + c];
    if (c == 0) hp[r] = h[src];
}

__global__ void __launch_bounds__(TB) k_invert(const int32_t* __restrict__ perm, int n, int32_t* __restrict__ inv)
{
    const int i = blockIdx.x * TB + threadIdx.x;
    if (i >= n) return;
    const int j = perm[i];
    if ((unsigned int)j < (unsigned int)n) inv[j] = i;
}

__global__ void __launch_bounds__(TB) k_fill_i32(int32_t* a, int n, int32_t v)
{
    const int i = blockIdx.x * TB + threadIdx.x;
    if (i < n) a[i] = v;
}

__global__ void __launch_bounds__(TB) k_histogram(const int32_t* __restrict__ pid, int n, int bins,
                                                  int32_t* __restrict__ counts)
{
    const int i = blockIdx.x * TB + threadIdx.x;
    if (i >= n) return;
    const int b = pid[i];
    if ((unsigned int)b < (unsigned int)bins) atomicAdd(&counts[b], 1);
}

__global__ void __launch_bounds__(TB) k_keys(const int32_t* __restrict__ pid, const int32_t* __restrict__ rank,
                                             int n, int bins, uint32_t* __restrict__ key)
{
    const int i = blockIdx.x * TB + threadIdx.x;
    if (i >= n) return;
    const int b = pid[i];
    key[i] = (unsigned int)b < (unsigned int)bins ? (uint32_t)rank[b] : 0u;
}

__global__ void __launch_bounds__(TB) k_scatter(const uint32_t* __restrict__ key_sorted,
                                                const uint32_t* __restrict__ row_sorted,
                                                const int32_t* __restrict__ shift, int n, int bins, int n_padded,
                                                int32_t* __restrict__ perm, int32_t* __restrict__ inv)
{
    const int j = blockIdx.x * TB + threadIdx.x;
    if (j >= n) return;
    const uint32_t r = key_sorted[j];
    const uint32_t row = row_sorted[j];
    if (r >= (uint32_t)bins || row >= (uint32_t)n) return;
    const int pos = j + shift[r];
    if ((unsigned int)pos >= (unsigned int)n_padded) return;
    perm[pos] = (int32_t)row;
    inv[row] = pos;
}

template <bool VEC4>
__global__ void __launch_bounds__(TB) k_gather_padded(const float* __restrict__ X, const float* __restrict__ h,
                                                      const int32_t* __restrict__ perm, int n_padded, int N, int d,
                                                      float* __restrict__ Xs, float* __restrict__ hs)
{
    const int per_row = VEC4 ? d / 4 : d;
    const long long i = (long long)blockIdx.x * TB + threadIdx.x;
    if (i >= (long long)n_padded * per_row) return;
    const int r = (int)(i / per_row), c = (int)(i % per_row);
    const int src = perm[r];
    const bool ok = (unsigned int)src < (unsigned int)N;
    if (VEC4) {
        float4 v = {0.f, 0.f, 0.f, 0.f};
        if (ok) v = reinterpret_cast<const float4*>(X + (size_t)src * d)[c];
        reinterpret_cast<float4*>(Xs)[i] = v;
    } else {
        Xs[i] = ok ? X[(size_t)src * d + c] : 0.f;
    }
    if (c == 0) hs[r] = ok ? h[src] : __builtin_inff();
}

// one workgroup per tile; dynamic LDS: d floats (centre) + 2 words (radius bits, valid rows)
__global__ void __launch_bounds__(TB) k_tile_balls(const float* __restrict__ Xs, const int32_t* __restrict__ perm,
                                                   int n_padded, int d, float* __restrict__ tile_c,
                                                   float* __restrict__ tile_r)
{
    extern __shared__ float ball_smem[];
    float* cen = ball_smem;
    unsigned int* rbits = reinterpret_cast<unsigned int*>(ball_smem + d);
    int* nvalid = reinterpret_cast<int*>(ball_smem + d + 1);
    const int t = blockIdx.x;
    const int row0 = t * TILE;
    const int rows = (n_padded - row0) < TILE ? (n_padded - row0) : TILE;
    if (threadIdx.x == 0) { *rbits = 0u; *nvalid = 0; }
    __syncthreads();
    const bool mine = (int)threadIdx.x < rows && perm[row0 + threadIdx.x] >= 0;
    if (mine) atomicAdd(nvalid, 1);
    __syncthreads();
    const int cnt = *nvalid;
    for (int c = threadIdx.x; c < d; c += TB) {
        float sum = 0.f;                               // padding rows are all zero
        for (int r = 0; r < rows; ++r) sum += Xs[(size_t)(row0 + r) * d + c];
        const float m = cnt > 0 ? sum / (float)cnt : 0.f;
        cen[c] = m;
        tile_c[(size_t)t * d + c] = m;
    }
    __syncthreads();
    if (mine) {
        const float* x = Xs + (size_t)(row0 + threadIdx.x) * d;
        float s2 = 0.f;
        for (int c = 0; c < d; ++c) { const float e = x[c] - cen[c]; s2 = __builtin_fmaf(e, e, s2); }
        atomicMax(rbits, __float_as_uint(__builtin_sqrtf(s2)));
    }
    __syncthreads();
    if (threadIdx.x == 0) tile_r[t] = cnt > 0 ? __uint_as_float(*rbits) : -3.0e38f;
}

// Lower bounds between all pairs of tile balls: gaps[p * T + t] = max(0, |c_p - c_t| - r_p - r_t)^2, rounded
// towards zero (the centre distance may come out 2e-5 too large, the radii 2e-5 too small), NaN where tile t
// has no valid row (r_t < 0): the table a pruned sweep otherwise computes for every query panel.
// One workgroup per patch of 64 x 64 pairs; feature columns pass through LDS 32 at a time.
__global__ void __launch_bounds__(TB) k_tile_gaps(const float* __restrict__ tile_c, const float* __restrict__ tile_r,
                                                  int T, int d, float* __restrict__ gaps)
{
    __shared__ float P[64][33];
    __shared__ float Q[64][33];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;        // 16 x 16 threads, 4 x 4 pairs each
    const int p0 = blockIdx.y * 64, t0 = blockIdx.x * 64;
    float s2[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) s2[i][j] = 0.f;
    for (int c0 = 0; c0 < d; c0 += 32) {
        __syncthreads();
        for (int e = threadIdx.x; e < 64 * 32; e += TB) {
            const int r = e >> 5, c = e & 31;
            const bool live = c0 + c < d;
            P[r][c] = (live && p0 + r < T) ? tile_c[(size_t)(p0 + r) * d + c0 + c] : 0.f;
            Q[r][c] = (live && t0 + r < T) ? tile_c[(size_t)(t0 + r) * d + c0 + c] : 0.f;
        }
        __syncthreads();
#pragma unroll 4
        for (int c = 0; c < 32; ++c) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = P[ty + 16 * i][c]; b[i] = Q[tx + 16 * i][c]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) { const float e = a[i] - b[j]; s2[i][j] = __builtin_fmaf(e, e, s2[i][j]); }
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int pr = p0 + ty + 16 * i;
        if (pr >= T) continue;
        const float rp = tile_r[pr];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int tc = t0 + tx + 16 * j;
            if (tc >= T) continue;
            const float rt = tile_r[tc];
            const float g = __builtin_sqrtf(s2[i][j]) * (1.f - 2e-5f) - (rp + rt) * (1.f + 2e-5f);
            float lb = g > 0.f ? g * g * (1.f - 1e-5f) : 0.f;
            if (rt < 0.f || rp < 0.f) lb = __builtin_nanf("");
            gaps[(size_t)pr * T + tc] = lb;
        }
    }
}

static bool vec4_ok(const void* a, const void* b, int d)
{
    return d % 4 == 0 && ((reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b)) & 15) == 0;
}

// row = list[j] adopts pivot base + new_idx[j] when that pivot is closer than its current one
__global__ void __launch_bounds__(TB) k_adopt_pivots(const uint32_t* __restrict__ list, int m, int N,
                                                     const int32_t* __restrict__ new_idx,
                                                     const float* __restrict__ new_dist, int base, int count,
                                                     int32_t* __restrict__ pid, float* __restrict__ pdist)
{
    const int j = blockIdx.x * TB + threadIdx.x;
    if (j >= m) return;
    const uint32_t row = list[j];
    const int c = new_idx[j];
    if (row >= (uint32_t)N || (unsigned int)c >= (unsigned int)count) return;
    if (new_dist[j] < pdist[row]) { pid[row] = base + c; pdist[row] = new_dist[j]; }
}

// one wavefront per tile: the colour shared by all valid rows (colour >= 0), else -1
__global__ void __launch_bounds__(TB) k_tile_colours(const int32_t* __restrict__ colour_s, int n_padded, int T,
                                                     int32_t* __restrict__ tile_colour)
{
    const int lane = threadIdx.x & 63;
    const int t = (int)(((long long)blockIdx.x * TB + threadIdx.x) >> 6);
    if (t >= T) return;                                  // whole wavefronts leave together
    int lo = 0x7fffffff, hi = -1;
    for (int r = lane; r < TILE; r += 64) {
        const int row = t * TILE + r;
        const int c = row < n_padded ? colour_s[row] : -1;
        if (c >= 0) { lo = c < lo ? c : lo; hi = c > hi ? c : hi; }
    }
    for (int o = 1; o < 64; o <<= 1) {
        const int l2 = __shfl_xor(lo, o), h2 = __shfl_xor(hi, o);
        lo = l2 < lo ? l2 : lo;
        hi = h2 > hi ? h2 : hi;
    }
    if (lane == 0) tile_colour[t] = (hi >= 0 && lo == hi) ? lo : -1;
}

// slot[inv[list[q]]] = q
__global__ void __launch_bounds__(TB) k_scatter_slots(const int32_t* __restrict__ inv, const int32_t* __restrict__ list,
                                                      int m, int N, int n_padded, int32_t* __restrict__ slot)
{
    const int q = blockIdx.x * TB + threadIdx.x;
    if (q >= m) return;
    const int v = list[q];
    if ((unsigned int)v >= (unsigned int)N) return;
    const int pos = inv[v];
    if ((unsigned int)pos < (unsigned int)n_padded) slot[pos] = q;
}

hipError_t order_iota(int32_t* a, int n, hipStream_t s)
{
    hipLaunchKernelGGL(k_iota, dim3(blocks_for(n)), dim3(TB), 0, s, a, n);
    return hipGetLastError();
}

hipError_t order_pick_rows(const float* X, const float* h, int N, int d, int P, float* Xp, float* hp, hipStream_t s)
{
    if (vec4_ok(X, Xp, d))
        hipLaunchKernelGGL(k_gather_rows<true>, dim3(blocks_for((long long)P * (d / 4))), dim3(TB), 0, s, X, (const int32_t*)nullptr, N, d, P, Xp);
    else
        hipLaunchKernelGGL(k_gather_rows<false>, dim3(blocks_for((long long)P * d)), dim3(TB), 0, s, X, (const int32_t*)nullptr, N, d, P, Xp);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_pick_f32, dim3(blocks_for(P)), dim3(TB), 0, s, h, N, P, hp);
    return hipGetLastError();
}

hipError_t order_gather_rows(const float* X, const int32_t* perm, int N, int d, float* Xs, hipStream_t s)
{
    if (vec4_ok(X, Xs, d))
        hipLaunchKernelGGL(k_gather_rows<true>, dim3(blocks_for((long long)N * (d / 4))), dim3(TB), 0, s, X, perm, N, d, N, Xs);
    else
        hipLaunchKernelGGL(k_gather_rows<false>, dim3(blocks_for((long long)N * d)), dim3(TB), 0, s, X, perm, N, d, N, Xs);
    return hipGetLastError();
}

hipError_t order_gather_f32(const float* a, const int32_t* idx, int n, int limit, float fallback, float* out,
                            hipStream_t s)
{
    hipLaunchKernelGGL(k_gather<float>, dim3(blocks_for(n)), dim3(TB), 0, s, a, idx, n, limit, fallback, out);
    return hipGetLastError();
}

hipError_t order_gather_i32(const int32_t* a, const int32_t* idx, int n, int limit, int32_t fallback, int32_t* out,
                            hipStream_t s)
{
    hipLaunchKernelGGL(k_gather<int32_t>, dim3(blocks_for(n)), dim3(TB), 0, s, a, idx, n, limit, fallback, out);
    return hipGetLastError();
}

hipError_t order_pick_f32(const float* a, int N, int P, float* out, hipStream_t s)
{
    hipLaunchKernelGGL(k_pick_f32, dim3(blocks_for(P)), dim3(TB), 0, s, a, N, P, out);
    return hipGetLastError();
}

hipError_t order_mark_far(const float* dist, int n, float tau, uint32_t* key, int32_t* count, hipStream_t s)
{
    hipLaunchKernelGGL(k_mark_far, dim3(blocks_for(n)), dim3(TB), 0, s, dist, n, tau, key, count);
    return hipGetLastError();
}

hipError_t order_pick_listed_rows(const float* X, const float* h, const uint32_t* list, int m, int N, int d, int P,
                                  float* Xp, float* hp, hipStream_t s)
{
    if (vec4_ok(X, Xp, d))
        hipLaunchKernelGGL(k_pick_listed<true>, dim3(blocks_for((long long)P * (d / 4))), dim3(TB), 0, s, X, h, list, m, N, d, P, Xp, hp);
    else
        hipLaunchKernelGGL(k_pick_listed<false>, dim3(blocks_for((long long)P * d)), dim3(TB), 0, s, X, h, list, m, N, d, P, Xp, hp);
    return hipGetLastError();
}

hipError_t order_invert(const int32_t* perm, int n, int32_t* inv, hipStream_t s)
{
    hipLaunchKernelGGL(k_invert, dim3(blocks_for(n)), dim3(TB), 0, s, perm, n, inv);
    return hipGetLastError();
}

hipError_t order_fill_i32(int32_t* a, int n, int32_t value, hipStream_t s)
{
    hipLaunchKernelGGL(k_fill_i32, dim3(blocks_for(n)), dim3(TB), 0, s, a, n, value);
    return hipGetLastError();
}

hipError_t order_histogram(const int32_t* pid, int n, int bins, int32_t* counts, hipStream_t s)
{
    hipLaunchKernelGGL(k_histogram, dim3(blocks_for(n)), dim3(TB), 0, s, pid, n, bins, counts);
    return hipGetLastError();
}

hipError_t order_keys(const int32_t* pid, const int32_t* rank, int n, int bins, uint32_t* key, hipStream_t s)
{
    hipLaunchKernelGGL(k_keys, dim3(blocks_for(n)), dim3(TB), 0, s, pid, rank, n, bins, key);
    return hipGetLastError();
}

hipError_t order_scatter(const uint32_t* key_sorted, const uint32_t* row_sorted, const int32_t* shift,
                         int n, int bins, int n_padded, int32_t* perm, int32_t* inv, hipStream_t s)
{
    hipLaunchKernelGGL(k_scatter, dim3(blocks_for(n)), dim3(TB), 0, s, key_sorted, row_sorted, shift, n, bins,
                       n_padded, perm, inv);
    return hipGetLastError();
}

hipError_t order_gather_padded(const float* X, const float* h, const int32_t* perm, int n_padded, int N,
                               int d, float* Xs, float* hs, hipStream_t s)
{
    if (vec4_ok(X, Xs, d))
        hipLaunchKernelGGL(k_gather_padded<true>, dim3(blocks_for((long long)n_padded * (d / 4))), dim3(TB), 0, s,
                           X, h, perm, n_padded, N, d, Xs, hs);
    else
        hipLaunchKernelGGL(k_gather_padded<false>, dim3(blocks_for((long long)n_padded * d)), dim3(TB), 0, s,
                           X, h, perm, n_padded, N, d, Xs, hs);
    return hipGetLastError();
}

hipError_t order_tile_balls(const float* Xs, const int32_t* perm, int n_padded, int d, float* tile_c,
                            float* tile_r, hipStream_t s)
{
    const int T = (n_padded + TILE - 1) / TILE;
    hipLaunchKernelGGL(k_tile_balls, dim3(T), dim3(TB), (size_t)(d + 4) * sizeof(float), s, Xs, perm, n_padded, d,
                       tile_c, tile_r);
    return hipGetLastError();
}

hipError_t order_adopt_pivots(const uint32_t* list, int m, int N, const int32_t* new_idx, const float* new_dist,
                              int base, int count, int32_t* pid, float* pdist, hipStream_t s)
{
    hipLaunchKernelGGL(k_adopt_pivots, dim3(blocks_for(m)), dim3(TB), 0, s, list, m, N, new_idx, new_dist, base, count,
                       pid, pdist);
    return hipGetLastError();
}

// *count += tiles of 128 slots that hold at least one slot >= 0 (one wavefront per tile); their numbers go to
// list[old *count ...] in no particular order
__global__ void __launch_bounds__(TB) k_count_used_tiles(const int32_t* __restrict__ slot, int n_padded, int T,
                                                         int32_t* __restrict__ count, int32_t* __restrict__ list)
{
    const int t = (blockIdx.x * TB + threadIdx.x) >> 6, lane = threadIdx.x & 63;
    if (t >= T) return;
    const int r0 = t * TILE + lane, r1 = r0 + 64;
    const bool any = (r0 < n_padded && slot[r0] >= 0) || (r1 < n_padded && slot[r1] >= 0);
    if (__ballot(any) != 0ull && lane == 0) {
        const int at = atomicAdd(count, 1);
        if (list) list[at] = t;
    }
}

hipError_t order_count_used_tiles(const int32_t* slot, int n_padded, int32_t* count, int32_t* list, hipStream_t s)
{
    const int T = (n_padded + TILE - 1) / TILE;
    hipLaunchKernelGGL(k_count_used_tiles, dim3(blocks_for((long long)T * 64)), dim3(TB), 0, s, slot, n_padded, T, count, list);
    return hipGetLastError();
}

hipError_t order_tile_gaps(const float* tile_c, const float* tile_r, int T, int d, float* gaps, hipStream_t s)
{
    if (T < 1) return hipSuccess;
    const int patches = (T + 63) / 64;
    hipLaunchKernelGGL(k_tile_gaps, dim3(patches, patches), dim3(TB), 0, s, tile_c, tile_r, T, d, gaps);
    return hipGetLastError();
}

hipError_t order_tile_colours(const int32_t* colour_s, int n_padded, int32_t* tile_colour, hipStream_t s)
{
    const int T = (n_padded + TILE - 1) / TILE;
    hipLaunchKernelGGL(k_tile_colours, dim3(blocks_for((long long)T * 64)), dim3(TB), 0, s, colour_s, n_padded, T, tile_colour);
    return hipGetLastError();
}

hipError_t order_scatter_slots(const int32_t* inv, const int32_t* list, int m, int N, int n_padded, int32_t* slot,
                               hipStream_t s)
{
    hipLaunchKernelGGL(k_scatter_slots, dim3(blocks_for(m)), dim3(TB), 0, s, inv, list, m, N, n_padded, slot);
    return hipGetLastError();
}

}  // namespace slhc
