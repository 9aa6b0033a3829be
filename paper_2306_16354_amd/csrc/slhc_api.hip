// C ABI of the library (see include/slhc.h) and the host orchestration of the cuSLINK pipeline:
// Alg. "cuSLINK Algorithm" (k-NN graph -> MST -> connect -> relabel), Alg. "connect_graph",
// Alg. "MST Algorithm" of the paper, restructured as one certified Boruvka loop (see
// forest_kernels.hip for what "certified" means).
#include <hip/hip_runtime.h>
#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <exception>
#include <mutex>
#include <memory>
#include <new>
#include <thread>
#include <vector>

#include "../../include/slhc.h"
#include "cluster_kernels.h"
#include "forest_kernels.h"
#include "order_kernels.h"
#include "sweep_kernels.h"

namespace {

thread_local char g_err[512] = "";

void set_err(const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

int hip_fail(hipError_t e, const char* what)
{
    set_err("%s: %s", what, hipGetErrorString(e));
    return SLHC_HIP_ERROR;
}

#define HIP_TRY(expr)                                                  \
    do {                                                               \
        hipError_t _e = (expr);                                        \
        if (_e != hipSuccess) return hip_fail(_e, #expr);              \
    } while (0)

// Runs the body of an exported function; no C++ exception leaves the library.
template <typename F>
int guarded(F&& body) noexcept
{
    try {
        return body();
    } catch (const std::bad_alloc&) {
        set_err("a host allocation failed");
        return SLHC_HOST_MEMORY;
    } catch (const std::exception& e) {
        set_err("unexpected exception: %s", e.what());
        return SLHC_INTERNAL;
    } catch (...) {
        set_err("unexpected exception");
        return SLHC_INTERNAL;
    }
}

constexpr size_t ALIGN = 256;
inline size_t up(size_t b) { return (b + ALIGN - 1) & ~(ALIGN - 1); }

// Bump allocator over the caller's workspace (layout only; nothing is allocated).
struct Carver {
    unsigned char* base;
    size_t off = 0;
    explicit Carver(void* b) : base(static_cast<unsigned char*>(b)) {}
    template <typename T>
    T* take(size_t count)
    {
        T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
        off += up(count * sizeof(T));
        return p;
    }
};

int check_shape(int64_t N, int32_t d, int32_t k, bool need_k)
{
    if (N < 2 || d < 1) { set_err("need N >= 2 and d >= 1 (N=%lld d=%d)", (long long)N, d); return SLHC_INVALID_ARG; }
    if (need_k) {
        if (k < 1 || (int64_t)k > N - 1) { set_err("need 1 <= k <= N-1 (k=%d N=%lld)", k, (long long)N); return SLHC_INVALID_ARG; }
        if (k > SLHC_MAX_K) { set_err("k=%d exceeds SLHC_MAX_K=%d", k, SLHC_MAX_K); return SLHC_UNSUPPORTED; }
        if (N * (int64_t)k > 2147483647LL) { set_err("N*k exceeds 2^31-1"); return SLHC_UNSUPPORTED; }
    }
    if (N * (int64_t)d > 2147483647LL) { set_err("N*d exceeds 2^31-1"); return SLHC_UNSUPPORTED; }
    return SLHC_OK;
}

__global__ void k_zero_words(uint32_t* p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// Columns the sweeps work on.  A zero column adds fma(0, 0, s) = s to a distance and to a norm, so appending
// zero columns changes no bit of any output; it does change which kernels apply.  Up to 128 features the rows are
// padded to whole chunks of 32 columns (register-resident queries, split bfloat16 products, tile pruning for
// every d), beyond that to a multiple of 4 (vector loads and split products in the streaming kernel).  The
// padded copy lives at the head of the caller's workspace.  d is kept where the padded matrix would pass the
// 2^31-1 element limit.
int32_t working_columns(int64_t N, int32_t d)
{
    const int32_t dw = d <= 128 ? (d + 31) / 32 * 32 : (d + 3) / 4 * 4;
    return N * (int64_t)dw > 2147483647LL ? d : dw;
}
size_t padded_copy_bytes(int64_t N, int32_t d)
{
    const int32_t dw = working_columns(N, d);
    return dw == d ? 0 : up((size_t)N * (size_t)dw * sizeof(float));
}

// out[row][c] = c < d ? X[row][c] : 0 for c < dw (dw a multiple of 4); one thread per four output columns
__global__ void __launch_bounds__(256) k_pad_columns(const float* __restrict__ X, long long quads, int d, int dw,
                                                     float* __restrict__ out)
{
    const long long q = (long long)blockIdx.x * 256 + threadIdx.x;
    if (q >= quads) return;
    const int per_row = dw >> 2;
    const long long row = q / per_row;
    const int c0 = 4 * (int)(q - row * per_row);
    const float* src = X + row * d;
    float4 v;
    v.x = c0 < d ? src[c0] : 0.f;
    v.y = c0 + 1 < d ? src[c0 + 1] : 0.f;
    v.z = c0 + 2 < d ? src[c0 + 2] : 0.f;
    v.w = c0 + 3 < d ? src[c0 + 3] : 0.f;
    *reinterpret_cast<float4*>(out + row * dw + c0) = v;
}

int pad_columns(const float* X, int64_t N, int32_t d, int32_t dw, float* out, hipStream_t s)
{
    const long long quads = (long long)N * (dw >> 2);
    hipLaunchKernelGGL(k_pad_columns, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, s, X, quads, d, dw, out);
    HIP_TRY(hipGetLastError());
    return SLHC_OK;
}

// Regions of the reordered copy: runs of consecutive tiles whose centres stay close.  boundary[t] = 1 when tile t
// starts a region: the first tile, a tile without valid rows (radius < 0) or next to one, or a tile whose centre lies
// farther from the previous tile's than twice the larger of the two radii.
__global__ void __launch_bounds__(256) k_region_boundaries(const float* __restrict__ tile_c, const float* __restrict__ tile_r,
                                                           int T, int d, int32_t* __restrict__ boundary)
{
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= T) return;
    int b = 1;
    if (t > 0) {
        const float r0 = tile_r[t - 1], r1 = tile_r[t];
        if (r0 >= 0.f && r1 >= 0.f) {
            const float* c0 = tile_c + (size_t)(t - 1) * d;
            const float* c1 = tile_c + (size_t)t * d;
            float s2 = 0.f;
            for (int j = 0; j < d; ++j) { const float e = c1[j] - c0[j]; s2 = __builtin_fmaf(e, e, s2); }
            const float reach = 2.f * fmaxf(r0, r1);
            b = (s2 <= reach * reach) ? 0 : 1;           // NaN: a boundary
        }
    }
    boundary[t] = b;
}
// region[t] = number of the region tile t lies in, first[t] = the first tile of that region (one workgroup)
__global__ void __launch_bounds__(1024) k_region_scan(const int32_t* __restrict__ boundary, int T, int32_t* __restrict__ region,
                                                      int32_t* __restrict__ first)
{
    __shared__ int cnt[1024], last[1024];
    const int tid = threadIdx.x;
    const int per = (T + 1023) / 1024;
    const int t0 = tid * per < T ? tid * per : T, t1 = t0 + per < T ? t0 + per : T;
    int c = 0, l = -1;
    for (int t = t0; t < t1; ++t) if (boundary[t]) { ++c; l = t; }
    cnt[tid] = c; last[tid] = l;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {
        const int cv = tid >= off ? cnt[tid - off] : 0, lv = tid >= off ? last[tid - off] : -1;
        __syncthreads();
        cnt[tid] += cv; last[tid] = last[tid] > lv ? last[tid] : lv;
        __syncthreads();
    }
    int rc = tid > 0 ? cnt[tid - 1] : 0, rl = tid > 0 ? last[tid - 1] : -1;
    for (int t = t0; t < t1; ++t) {
        if (boundary[t]) { ++rc; rl = t; }
        region[t] = rc > 0 ? rc - 1 : 0;
        first[t] = rl >= 0 ? rl : 0;
    }
}
// last[t] = the last tile of tile t's region: the thread of a region's last tile writes the whole run
__global__ void __launch_bounds__(256) k_region_last(const int32_t* __restrict__ boundary, const int32_t* __restrict__ first, int T,
                                                     int32_t* __restrict__ last)
{
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= T) return;
    if (t == T - 1 || boundary[t + 1] != 0) {
        int u = first[t];
        if (u < 0) u = 0;
        for (; u <= t; ++u) last[u] = t;
    }
}
// out[row] = the smallest lower bound in row `row` of the table of tile pairs among the tiles of other regions
// (+inf: none; NaN entries mark tiles that are never needed)
__global__ void __launch_bounds__(256) k_region_other_min(const float* __restrict__ tile_gap, const int32_t* __restrict__ region,
                                                          int T, float* __restrict__ out)
{
    __shared__ float part[256];
    const int row = blockIdx.x;
    const int mine = region[row];
    const float* g = tile_gap + (size_t)row * T;
    float m = __builtin_inff();
    for (int t = threadIdx.x; t < T; t += 256) {
        const float v = g[t];
        if (region[t] != mine && v < m) m = v;          // false for NaN
    }
    part[threadIdx.x] = m;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) part[threadIdx.x] = fminf(part[threadIdx.x], part[threadIdx.x + w]);
        __syncthreads();
    }
    if (threadIdx.x == 0) out[row] = part[0];
}
// h[i] = +inf for the padding rows of the reordered copy (perm[i] < 0)
__global__ void __launch_bounds__(256) k_mask_padding(const int32_t* __restrict__ perm, int n, float* __restrict__ h)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n && perm[i] < 0) h[i] = __builtin_inff();
}

// out[0], out[1] = sums of a[i] and b[i] over at most 16384 evenly spaced i < n (one workgroup, fixed order)
__global__ void __launch_bounds__(256) k_sample_sums(const float* __restrict__ a, const float* __restrict__ b, int n,
                                                     float* __restrict__ out)
{
    __shared__ float sa[256], sb[256];
    const int samples = n < 16384 ? n : 16384;
    float xa = 0.f, xb = 0.f;
    for (int i = threadIdx.x; i < samples; i += 256) {
        const long long at = (long long)i * n / samples;
        xa += a[at]; xb += b[at];
    }
    sa[threadIdx.x] = xa; sb[threadIdx.x] = xb;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) { sa[threadIdx.x] += sa[threadIdx.x + w]; sb[threadIdx.x] += sb[threadIdx.x + w]; }
        __syncthreads();
    }
    if (threadIdx.x == 0) { out[0] = sa[0]; out[1] = sb[0]; }
}

// Pinned host staging for device<->host copies (freed when the call returns).
struct PinnedHost {
    void* p = nullptr;
    hipError_t alloc(size_t bytes) { return hipHostMalloc(&p, bytes, hipHostMallocDefault); }
    ~PinnedHost() { if (p) (void)hipHostFree(p); }
};

// A pair of HIP events bracketing work on a stream.
struct EventPair {
    hipEvent_t a = nullptr, b = nullptr;
    hipError_t create() { hipError_t e = hipEventCreate(&a); return e != hipSuccess ? e : hipEventCreate(&b); }
    ~EventPair() { if (a) (void)hipEventDestroy(a); if (b) (void)hipEventDestroy(b); }
    float ms() const { float t = 0.f; return hipEventElapsedTime(&t, a, b) == hipSuccess ? t : -1.f; }
};

double now_ms()
{
    using clk = std::chrono::steady_clock;
    return std::chrono::duration<double, std::milli>(clk::now().time_since_epoch()).count();
}

// SLHC_LOG=1 in the environment: phase times and per-round counters on stderr (each mark waits for
// the stream, so the logged run is slower than a normal one).
struct PhaseLog {
    bool on;
    hipStream_t s;
    double t;
    explicit PhaseLog(hipStream_t stream) : s(stream), t(0.0)
    {
        const char* e = std::getenv("SLHC_LOG");
        on = e && e[0] && e[0] != '0';
        if (on) t = now_ms();
    }
    void mark(const char* fmt, ...)
    {
        if (!on) return;
        (void)hipStreamSynchronize(s);
        const double now = now_ms();
        char text[256];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(text, sizeof(text), fmt, ap);
        va_end(ap);
        std::fprintf(stderr, "[slhc] %8.2f ms  %s\n", now - t, text);
        t = now_ms();
    }
};

// Tile pruning is implemented by the register-resident-query sweep only (d <= 128, d % 4 == 0), and
// pays off only when there are enough rows to form several tiles per cluster.
#ifndef SLHC_PRUNE_MIN_ROWS
#define SLHC_PRUNE_MIN_ROWS 512      // compile-time knob so that small harnesses can exercise the reordered path
#endif
constexpr int64_t PRUNE_MIN_ROWS = SLHC_PRUNE_MIN_ROWS;
// two-phase pruned connection sweeps (see run_slhc): rows, tile steps per panel of the round before
#ifndef SLHC_TWO_PHASE_MIN_ROWS
#define SLHC_TWO_PHASE_MIN_ROWS 262144
#endif
constexpr int64_t TWO_PHASE_MIN_ROWS = SLHC_TWO_PHASE_MIN_ROWS;
#ifndef SLHC_TWO_PHASE_MIN_STEPS
#define SLHC_TWO_PHASE_MIN_STEPS 128.0
#endif
constexpr double TWO_PHASE_MIN_STEPS = SLHC_TWO_PHASE_MIN_STEPS;
constexpr int TWO_PHASE_STRIDE = 16;
// pruned connection sweeps lower a component's shared threshold to this multiple of the lightest edge its
// queries have found so far (squared distance; see SweepParams::comp_lower_factor)
#ifndef SLHC_LOWER_FACTOR
#define SLHC_LOWER_FACTOR 1.0f
#endif
constexpr float LOWER_FACTOR = SLHC_LOWER_FACTOR;
#ifndef SLHC_LOWER_MIN_ROWS
#define SLHC_LOWER_MIN_ROWS 4096
#endif
constexpr int LOWER_MIN_ROWS = SLHC_LOWER_MIN_ROWS;
constexpr int NESTED_K = 8;
// pruned connection sweeps: a launch with fewer non-empty panels than this splits every panel's scan into parts
// so that about this many work items result, at most SPLIT_MAX_PARTS per panel
#ifndef SLHC_SPLIT_ITEMS_TARGET
#define SLHC_SPLIT_ITEMS_TARGET 32768
#endif
constexpr int SPLIT_ITEMS_TARGET = SLHC_SPLIT_ITEMS_TARGET;
constexpr int SPLIT_MAX_PARTS = 16;
// ... and only as far as a part still has about this many tiles to multiply, going by the steps per panel of the
// sweep before
#ifndef SLHC_SPLIT_MIN_STEPS
#define SLHC_SPLIT_MIN_STEPS 8.0
#endif
constexpr double SPLIT_MIN_STEPS = SLHC_SPLIT_MIN_STEPS;
// up to this many tiles of the reordered copy the lower bounds between all pairs of tiles are tabulated once
// (T x T floats: 4 GiB at the limit) instead of being computed for every query panel of every pruned sweep
#ifndef SLHC_TILE_GAP_MAX_TILES
#define SLHC_TILE_GAP_MAX_TILES 32768
#endif
constexpr int TILE_GAP_MAX_TILES = SLHC_TILE_GAP_MAX_TILES;
// dendrogram: from this many rows on, host threads share the light edges (see build_dendrogram_parallel)
#ifndef SLHC_DENDROGRAM_THREADS_MIN_ROWS
#define SLHC_DENDROGRAM_THREADS_MIN_ROWS 200000
#endif
constexpr int64_t DENDROGRAM_THREADS_MIN_ROWS = SLHC_DENDROGRAM_THREADS_MIN_ROWS;
bool prunable(int64_t N, int32_t d) { return d % 4 == 0 && d <= 128 && N >= PRUNE_MIN_ROWS; }
#ifndef SLHC_PIVOT_STRIDE
#define SLHC_PIVOT_STRIDE 64
#endif
int first_level_pivots(int64_t N) { return (int)((N + SLHC_PIVOT_STRIDE - 1) / SLHC_PIVOT_STRIDE); }
// The reordered copy inserts padding rows so that well separated clusters start on a tile
// boundary; padding is limited to N/2 rows.
int64_t padded_rows_limit(int64_t N) { return N + N / 2 + 256; }

size_t slhc_ws_bytes(int64_t N, int32_t d, int32_t k, bool with_order);

// tile products from split bfloat16 halves: whole chunks of 32 columns up to 128 features (the
// register-resident-query kernel); beyond 128 features the streaming kernel takes any multiple of 4 columns,
// its split copy padded to whole chunks
bool split_products_ok(int32_t d) { return (d % 32 == 0 && d >= 32 && d <= 128) || (d > 128 && d % 4 == 0); }
// ... in the pruned sweeps from two chunks on only: at 32 features a tile's multiplies are too short for the
// wider filter to pay (2M x 32: pruned connection sweeps 30 ms with float32 products, 60 ms with split ones)
bool split_products_pruned_ok(int32_t d) { return d % 32 == 0 && d >= 64 && d <= 128; }

// Buffers of the spatially coherent row order (see build_order).
struct OrderWs {
    float *Xp, *hp, *pdist, *sample, *Xs, *hs, *tile_c, *tile_r, *gap_ws, *tile_gap, *n_w, *n_heights;
    float *Xs_split, *hs_split;      // the reordered copy in split bfloat16 halves and its half norms (nullptr: d does not allow it)
    // a second split copy, every tile relative to the centre of the first tile of its region, with its half norms;
    // region number, first tile and boundary flag per tile (see run_knn; nullptr: the pruned sweeps keep float32 products)
    float *Xs_local, *hs_local, *region_other_min;
    int32_t *tile_region, *tile_first, *tile_last, *tile_boundary;
    int32_t *pid, *perm, *inv, *colour_s, *qslot, *tile_colour, *tile_list, *counts, *rank, *shift, *far_count;
    int32_t *n_src, *n_dst, *n_children, *n_sizes;
    uint32_t *tmp_a, *tmp_b, *tmp_c;
    void* sort_temp; size_t sort_temp_bytes;
    void* nested_ws; size_t nested_bytes;
    int P1, Pmax, Tmax;
    int64_t Nmax;
    int P = 0;        // pivots in use          (set by build_order)
    int Ns = 0;       // rows of the padded copy (set by build_order)
    static constexpr int SAMPLE = 4096;
    void carve(Carver& c, int64_t N, int32_t d)
    {
        const size_t n = (size_t)N;
        P1 = first_level_pivots(N);
        Pmax = 4 * P1;            // budget for pivots added for clusters the first level missed
        Nmax = padded_rows_limit(N);
        Tmax = (int)((Nmax + 127) / 128);
        const size_t nm = (size_t)Nmax, pm = (size_t)Pmax;
        Xp = c.take<float>(pm * d); hp = c.take<float>(pm);
        pdist = c.take<float>(n); sample = c.take<float>(SAMPLE);
        Xs = c.take<float>(nm * d); hs = c.take<float>(nm);
        Xs_split = nullptr; hs_split = nullptr;
        if (split_products_ok(d)) { Xs_split = c.take<float>(nm * d); hs_split = c.take<float>(nm); }
        Xs_local = nullptr; hs_local = nullptr; region_other_min = nullptr; tile_region = nullptr; tile_first = nullptr; tile_last = nullptr; tile_boundary = nullptr;
        if (split_products_ok(d) && d <= 128) {
            Xs_local = c.take<float>(nm * d); hs_local = c.take<float>(nm);
            tile_region = c.take<int32_t>((size_t)Tmax); tile_first = c.take<int32_t>((size_t)Tmax);
            tile_last = c.take<int32_t>((size_t)Tmax);
            region_other_min = c.take<float>((size_t)Tmax);
            tile_boundary = c.take<int32_t>((size_t)Tmax);
        }
        tile_c = c.take<float>((size_t)Tmax * d); tile_r = c.take<float>((size_t)Tmax);
        int grid = slhc::sweep_grid_limit();
        if (grid < 1) grid = 512;
        gap_ws = c.take<float>((size_t)grid * Tmax);
        // lower bounds between all pairs of tiles (order_tile_gaps), as long as the table stays moderate
        tile_gap = Tmax <= TILE_GAP_MAX_TILES ? c.take<float>((size_t)Tmax * Tmax) : nullptr;
        pid = c.take<int32_t>(n); perm = c.take<int32_t>(nm); inv = c.take<int32_t>(n); colour_s = c.take<int32_t>(nm);
        qslot = c.take<int32_t>(nm); tile_colour = c.take<int32_t>((size_t)Tmax); tile_list = c.take<int32_t>((size_t)Tmax);
        counts = c.take<int32_t>(pm); rank = c.take<int32_t>(pm); shift = c.take<int32_t>(pm); far_count = c.take<int32_t>(64);
        tmp_a = c.take<uint32_t>(n); tmp_b = c.take<uint32_t>(n); tmp_c = c.take<uint32_t>(n);
        sort_temp_bytes = slhc::pair_sort_temp_bytes((int)N);
        sort_temp = c.take<unsigned char>(sort_temp_bytes);
        n_src = c.take<int32_t>(pm); n_dst = c.take<int32_t>(pm); n_w = c.take<float>(pm);
        n_children = c.take<int32_t>(2 * pm); n_heights = c.take<float>(pm); n_sizes = c.take<int32_t>(pm);
        const int32_t kp = Pmax - 1 < NESTED_K ? Pmax - 1 : NESTED_K;
        // (the clustering runs on the pivots in use, fewer than Pmax: a k-NN sweep of few panels then also wants
        // its scratch for candidate ranges, which the layout for Pmax rows may not contain)
        nested_bytes = slhc_ws_bytes(Pmax, d, kp, false) + (size_t)grid * 128 * (size_t)kp * 8 + 1024;
        nested_ws = c.take<unsigned char>(nested_bytes);
    }
};

struct KnnWs {
    unsigned long long* counters;    // [0] k-NN survivors [1] connect survivors [2] k-NN tile steps [3] connect tile steps
                                     // [4] non-finite flag (low word) [8] panel hand-out counter (low word)
    float* hn;
    bool has_order;
    OrderWs order;
    // lists per candidate range of a k-NN sweep with few panels (see launch_knn_sweep); k = 0: none
    int32_t* part_idx; float* part_dist; long long part_rows;
    // every-tile sweeps on the bf16 MFMA: X split into bfloat16 halves (see SweepParams::Xq_split) and the half
    // norms with the slack that goes with it; nullptr when d does not allow it
    float* Xsplit; float* hn_split;
    // the split copies hold the rows relative to the column means of X (a sample's): shift [d], and the scratch of
    // the two-pass mean
    float* shift; float* shift_scratch;
    // scratch of the every-tile sweeps that go range by range (see SweepParams::carry_ws): 2 + panels words
    unsigned int* carry_ws; long long carry_ws_words;
    bool split_ready = false;        // filled in this call
    bool order_split_ready = false;  // likewise the split copy of the reordered rows
    bool offset_heavy = false;       // the rows' norms are mostly a common offset (see run_knn): split products everywhere
    bool order_split_connect = false;   // the pruned connection sweeps multiply the split copy of the reordered rows too
    size_t bytes;
    KnnWs(void* ws, int64_t N, int32_t d, bool with_order, int32_t k = 0)
    {
        Carver c(ws);
        counters = c.take<unsigned long long>(32);
        hn = c.take<float>((size_t)N);
        part_idx = nullptr; part_dist = nullptr; part_rows = 0;
        Xsplit = nullptr; hn_split = nullptr; shift = nullptr; shift_scratch = nullptr;
        if (split_products_ok(d) && k > 0) {
            Xsplit = c.take<float>((size_t)N * (size_t)slhc::split_row_stride(d));
            hn_split = c.take<float>((size_t)N);
            shift = c.take<float>((size_t)d);
            shift_scratch = c.take<float>(slhc::column_means_scratch_floats(d));
        }
        {
            // ranges x rows never exceeds the workgroup slots x 128: a sweep is only split while its panels
            // fill less than half the slots
            int grid = slhc::sweep_grid_limit();
            if (grid < 1) grid = 512;
            if (k > 1 && ((N + 127) / 128) * 2 <= grid) {
                part_rows = (long long)grid * 128;
                part_idx = c.take<int32_t>((size_t)part_rows * k);
                part_dist = c.take<float>((size_t)part_rows * k);
            }
        }
        carry_ws_words = 2 + (long long)((N + 127) / 128);
        carry_ws = c.take<unsigned int>((size_t)carry_ws_words);
        has_order = with_order && prunable(N, d);
        if (has_order) order.carve(c, N, d);
        bytes = c.off;
    }
};

struct SlhcWs {
    void* knn_ws;
    int32_t* nbr_idx; float* nbr_dist;
    int32_t *colour, *ptr, *ext_idx, *cand_u, *hook, *qlist, *q_idx, *counters, *e_lo, *e_hi;
    float *ext_dist, *cand_w, *q_dist, *e_w;
    uint32_t *best_w, *min_lb, *vals_a, *vals_b;
    unsigned long long *best_e, *keys_a, *keys_b;
    void* sort_temp; size_t sort_temp_bytes;
    size_t bytes;
    SlhcWs(void* ws, int64_t N, int32_t d, int32_t k, bool with_order)
    {
        Carver c(ws);
        const size_t n = (size_t)N;
        knn_ws = c.take<unsigned char>(KnnWs(nullptr, N, d, with_order, k).bytes);
        nbr_idx = c.take<int32_t>(n * k);
        nbr_dist = c.take<float>(n * k);
        colour = c.take<int32_t>(n); ptr = c.take<int32_t>(n); ext_idx = c.take<int32_t>(n);
        cand_u = c.take<int32_t>(n); hook = c.take<int32_t>(n); qlist = c.take<int32_t>(n);
        q_idx = c.take<int32_t>(n); counters = c.take<int32_t>(64);
        e_lo = c.take<int32_t>(n); e_hi = c.take<int32_t>(n);
        ext_dist = c.take<float>(n); cand_w = c.take<float>(n); q_dist = c.take<float>(n); e_w = c.take<float>(n);
        best_w = c.take<uint32_t>(n); min_lb = c.take<uint32_t>(n);
        vals_a = c.take<uint32_t>(n); vals_b = c.take<uint32_t>(n);
        best_e = c.take<unsigned long long>(n); keys_a = c.take<unsigned long long>(n); keys_b = c.take<unsigned long long>(n);
        sort_temp_bytes = std::max(slhc::edge_sort_temp_bytes((int)(N - 1)), slhc::pair_sort_temp_bytes((int)N));   // the second: grouping the dendrogram's edges
        sort_temp = c.take<unsigned char>(sort_temp_bytes);
        bytes = c.off;
    }
};

size_t slhc_ws_bytes(int64_t N, int32_t d, int32_t k, bool with_order) { return SlhcWs(nullptr, N, d, k, with_order).bytes; }

int run_slhc(const float* X, int64_t N, int32_t d, int32_t k, int32_t* mst_src, int32_t* mst_dst, float* mst_w,
             int32_t* children, float* heights, int32_t* sizes, slhc_stats* stats, void* workspace,
             hipStream_t s, uint32_t flags, bool with_order);

int bits_for(long long n) { int b = 1; while (b < 32 && (1LL << b) < n) ++b; return b; }

// X in split bfloat16 halves, taken relative to the column means of a sample of its rows (a translation changes no
// distance and keeps a common offset of the data out of the filter's slack), with the half norms that go with it.
int make_split_copy(const float* X, int64_t N, int32_t d, KnnWs& ws, hipStream_t s)
{
    HIP_TRY(slhc::launch_column_means(X, (int)N, d, ws.shift_scratch, ws.shift, s));
    HIP_TRY(slhc::launch_split_bf16(X, (int)N, d, ws.Xsplit, s, ws.shift));
    HIP_TRY(slhc::launch_half_norms(X, (int)N, d, ws.hn_split, s, nullptr, true, ws.shift));
    ws.split_ready = true;
    return SLHC_OK;
}

// Nearest pivot of every row by the fused sweep (k = 1 against the P pivot rows).
// `x_split` / `hn_split` / `shift` (optional): X in split bfloat16 halves, the half norms that go with it and the
// shift both were taken relative to; the pivots
// then get a split copy of their own (in the buffers of the reordered copy's, which are free until step 4).
int assign_to_pivots(const float* X, int64_t N, int32_t d, const float* hn, OrderWs& o, int P, hipStream_t s,
                     const float* x_split = nullptr, const float* hn_split = nullptr, const float* shift = nullptr)
{
    slhc::SweepParams p{};
    p.Xq = X; p.hq = hn; p.NQ = (int)N;
    p.Xc = o.Xp; p.hc = o.hp; p.NC = P;
    p.d = d; p.k = 1;
    p.out_idx = o.pid; p.out_dist = o.pdist;
    if (x_split && hn_split && o.Xs_split && o.hs_split) {
        HIP_TRY(slhc::launch_split_bf16(o.Xp, P, d, o.Xs_split, s, shift));
        HIP_TRY(slhc::launch_half_norms(o.Xp, P, d, o.hs_split, s, nullptr, true, shift));
        p.Xq_split = x_split; p.hq_split = hn_split;
        p.Xc_split = o.Xs_split; p.hc_split = o.hs_split;
    }
    HIP_TRY(slhc::launch_knn_sweep(p, s));
    return SLHC_OK;
}

// Spatially coherent order of the rows (not in the paper, whose sweeps multiply every tile).
//   1. Every 64th row is a pivot; each row is assigned to its nearest pivot by the fused 1-NN sweep.
//      Rows much farther from their pivot than the typical row belong to clusters that received no
//      pivot; a sample of those rows becomes a second set of pivots and the assignment is repeated.
//   2. The pivots are clustered by this library's own single-linkage path (without reordering); the
//      leaf order of their dendrogram puts pivots of one cluster next to each other at every scale.
//   3. Rows are sorted by the position of their pivot in that order.  Where consecutive pivots are
//      joined only far above the typical cell scale, the next row starts a new tile of 128 (padding
//      rows: perm = -1, zero features, +inf half norm), so tiles do not straddle distant clusters.
//   4. One bounding ball per tile of the reordered copy.
// The order only affects which tiles the sweeps can skip, never a result.
// `nonfinite`: device word the norm kernel set when a row is not finite; checked first, because
// nothing below is defined for such rows.
int build_order(const float* X, int64_t N, int32_t d, const float* hn, const unsigned int* nonfinite, OrderWs& o,
                hipStream_t s, const float* x_split = nullptr, const float* hn_split = nullptr, const float* shift = nullptr)
{
    const int n = (int)N;
    const int P1 = o.P1;
    PhaseLog log(s);
    PinnedHost pin;
    HIP_TRY(pin.alloc(((size_t)OrderWs::SAMPLE + 16 + 6 * (size_t)o.Pmax) * 4));
    float* h_sample = static_cast<float*>(pin.p);
    int32_t* h_count = reinterpret_cast<int32_t*>(h_sample + OrderWs::SAMPLE);
    int32_t* h_src = h_count + 16;
    int32_t* h_dst = h_src + o.Pmax;
    float* h_w = reinterpret_cast<float*>(h_dst + o.Pmax);
    int32_t* h_cells = reinterpret_cast<int32_t*>(h_w + o.Pmax);
    int32_t* h_rank = h_cells + o.Pmax;
    int32_t* h_shift = h_rank + o.Pmax;

    HIP_TRY(hipMemcpyAsync(h_count + 8, nonfinite, 4, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    if (h_count[8] != 0) { set_err("a row of X is not finite (NaN, infinity, or a squared norm beyond float32)"); return SLHC_NONFINITE; }

    // ---- 1. pivots and assignment
    HIP_TRY(slhc::order_pick_rows(X, hn, n, d, P1, o.Xp, o.hp, s));
    int rc = assign_to_pivots(X, N, d, hn, o, P1, s, x_split, hn_split, shift);
    if (rc != SLHC_OK) return rc;
    const int S = n < OrderWs::SAMPLE ? n : OrderWs::SAMPLE;
    HIP_TRY(slhc::order_pick_f32(o.pdist, n, S, o.sample, s));
    HIP_TRY(hipMemcpyAsync(h_sample, o.sample, (size_t)S * 4, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    log.mark("row order: %d pivots, nearest pivot of every row", P1);
    // Scale of a well-placed cell: 4 x the median positive squared distance to the pivot.  (When the
    // clusters are much smaller than the pivot spacing the median is an inter-cluster distance and no
    // row counts as far; such data cannot be pruned at tile granularity anyway, and the connection
    // sweeps then fall back to multiplying every tile, see run_slhc.)
    float tau = __builtin_inff();
    {
        std::vector<float> v;
        for (int i = 0; i < S; ++i) if (h_sample[i] > 0.f && std::isfinite(h_sample[i])) v.push_back(h_sample[i]);
        if (!v.empty()) {
            std::nth_element(v.begin(), v.begin() + v.size() / 2, v.end());
            tau = 4.f * v[v.size() / 2];
        }
    }
    // Rows much farther from their pivot than the typical row: clusters without a pivot.  Every 16th
    // of them (in row order) becomes a pivot and the far rows alone are re-assigned among the new
    // pivots; repeated until no row is far, the pivot budget is used, or four rounds are done.
    int P = P1;
    for (int round = 0; round < 4 && std::isfinite(tau) && P < o.Pmax; ++round) {
        hipLaunchKernelGGL(k_zero_words, dim3(1), dim3(64), 0, s, reinterpret_cast<uint32_t*>(o.far_count), 64);
        HIP_TRY(hipGetLastError());
        HIP_TRY(slhc::order_mark_far(o.pdist, n, tau, o.tmp_a, o.far_count, s));
        HIP_TRY(hipMemcpyAsync(h_count, o.far_count, 4, hipMemcpyDeviceToHost, s));
        HIP_TRY(hipStreamSynchronize(s));
        const int far = h_count[0];
        if (far < 0 || far > n) { set_err("row order: bad far-row count %d", far); return SLHC_INTERNAL; }
        if (far == 0) break;
        // far rows first, in row order (stable 1-bit sort)
        uint32_t* far_rows = reinterpret_cast<uint32_t*>(o.perm);
        HIP_TRY(slhc::order_iota(reinterpret_cast<int32_t*>(o.tmp_b), n, s));
        HIP_TRY(slhc::pair_sort_u32(o.tmp_a, o.tmp_c, o.tmp_b, far_rows, n, 1, o.sort_temp, o.sort_temp_bytes, s));
        int P2 = (far + 15) / 16;
        if (P2 > o.Pmax - P) P2 = o.Pmax - P;
        HIP_TRY(slhc::order_pick_listed_rows(X, hn, far_rows, far, n, d, P2, o.Xp + (size_t)P * d, o.hp + P, s));
        // the far rows as a compact query matrix (the buffer of the reordered copy is still free)
        HIP_TRY(slhc::order_pick_listed_rows(X, hn, far_rows, far, n, d, far, o.Xs, o.hs, s));
        slhc::SweepParams p{};
        p.Xq = o.Xs; p.hq = o.hs; p.NQ = far;
        p.Xc = o.Xp + (size_t)P * d; p.hc = o.hp + P; p.NC = P2;
        p.d = d; p.k = 1;
        p.out_idx = reinterpret_cast<int32_t*>(o.tmp_b); p.out_dist = reinterpret_cast<float*>(o.tmp_c);
        HIP_TRY(slhc::launch_knn_sweep(p, s));
        HIP_TRY(slhc::order_adopt_pivots(far_rows, far, n, reinterpret_cast<const int32_t*>(o.tmp_b),
                                         reinterpret_cast<const float*>(o.tmp_c), P, P2, o.pid, o.pdist, s));
        P += P2;
        log.mark("row order: %d far rows -> %d more pivots", far, P2);
    }
    o.P = P;

    // ---- 2. hierarchy of the pivots: concatenating the two sides of every merge, in merge order,
    // yields a leaf order of the dendrogram; `joined[i]` is the height at which pivot i's successor
    // in that order was attached.
    std::vector<int32_t> order((size_t)P), head((size_t)P), tail((size_t)P), nxt((size_t)P, -1), up_set((size_t)P);
    std::vector<float> joined((size_t)P, 0.f);
    for (int i = 0; i < P; ++i) head[(size_t)i] = tail[(size_t)i] = up_set[(size_t)i] = i;
    if (P >= 2) {
        const int32_t kp = P - 1 < NESTED_K ? P - 1 : NESTED_K;
        rc = run_slhc(o.Xp, P, d, kp, o.n_src, o.n_dst, o.n_w, o.n_children, o.n_heights, o.n_sizes, nullptr,
                      o.nested_ws, s, 0u, false);
        if (rc != SLHC_OK) return rc;
        const size_t E = (size_t)(P - 1);
        HIP_TRY(hipMemcpyAsync(h_src, o.n_src, E * 4, hipMemcpyDeviceToHost, s));
        HIP_TRY(hipMemcpyAsync(h_dst, o.n_dst, E * 4, hipMemcpyDeviceToHost, s));
        HIP_TRY(hipMemcpyAsync(h_w, o.n_w, E * 4, hipMemcpyDeviceToHost, s));
        HIP_TRY(hipStreamSynchronize(s));
        auto top = [&](int32_t a) {
            while (up_set[(size_t)a] != a) {
                up_set[(size_t)a] = up_set[(size_t)up_set[(size_t)a]];
                a = up_set[(size_t)a];
            }
            return a;
        };
        for (size_t e = 0; e < E; ++e) {
            if ((uint32_t)h_src[e] >= (uint32_t)P || (uint32_t)h_dst[e] >= (uint32_t)P) { set_err("row order: bad pivot edge"); return SLHC_INTERNAL; }
            const int32_t a = top(h_src[e]), b = top(h_dst[e]);
            if (a == b) { set_err("row order: pivot tree has a cycle"); return SLHC_INTERNAL; }
            nxt[(size_t)tail[(size_t)a]] = head[(size_t)b];
            joined[(size_t)tail[(size_t)a]] = h_w[e];
            tail[(size_t)a] = tail[(size_t)b];
            up_set[(size_t)b] = a;
        }
        int32_t at = head[(size_t)top(0)];
        for (int r = 0; r < P; ++r) {
            if (at < 0) { set_err("row order: pivot chain ends early"); return SLHC_INTERNAL; }
            order[(size_t)r] = at;
            at = nxt[(size_t)at];
        }
    } else {
        order[0] = 0;
    }
    for (int r = 0; r < P; ++r) h_rank[order[(size_t)r]] = r;
    log.mark("row order: single linkage of %d pivots, leaf order", P);

    // ---- 3. cell sizes and the padded layout
    HIP_TRY(slhc::order_fill_i32(o.counts, P, 0, s));
    HIP_TRY(slhc::order_histogram(o.pid, n, P, o.counts, s));
    HIP_TRY(hipMemcpyAsync(h_cells, o.counts, (size_t)P * 4, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    {
        long long total = 0;
        for (int i = 0; i < P; ++i) { if (h_cells[i] < 0) { total = -1; break; } total += h_cells[i]; }
        if (total != (long long)N) { set_err("row order: cells hold %lld of %lld rows", total, (long long)N); return SLHC_INTERNAL; }
    }
    const long long budget = (long long)(N / 2);
    float tau_pad = tau;
    long long Ns = 0;
    for (int attempt = 0; attempt < 200; ++attempt) {
        long long pos = 0, plain = 0;
        for (int r = 0; r < P; ++r) {
            const int pv = order[(size_t)r];
            h_shift[r] = (int32_t)(pos - plain);
            pos += h_cells[pv];
            plain += h_cells[pv];
            if (r + 1 < P && joined[(size_t)pv] > tau_pad) pos = (pos + 127) / 128 * 128;
        }
        Ns = pos;
        if (Ns - (long long)N <= budget) break;
        tau_pad = attempt < 190 ? tau_pad * 2.f : __builtin_inff();
    }
    if (Ns < (long long)N || Ns > (long long)o.Nmax) { set_err("row order: padded size %lld out of range", Ns); return SLHC_INTERNAL; }
    o.Ns = (int)Ns;

    // ---- 4. place the rows, gather the copy, bound the tiles
    HIP_TRY(hipMemcpyAsync(o.rank, h_rank, (size_t)P * 4, hipMemcpyHostToDevice, s));
    HIP_TRY(hipMemcpyAsync(o.shift, h_shift, (size_t)P * 4, hipMemcpyHostToDevice, s));
    uint32_t* keys = reinterpret_cast<uint32_t*>(o.colour_s);        // free until the connection rounds
    HIP_TRY(slhc::order_keys(o.pid, o.rank, n, P, keys, s));
    HIP_TRY(slhc::order_iota(reinterpret_cast<int32_t*>(o.tmp_a), n, s));
    HIP_TRY(slhc::pair_sort_u32(keys, o.tmp_b, o.tmp_a, o.tmp_c, n, bits_for(P), o.sort_temp, o.sort_temp_bytes, s));
    HIP_TRY(slhc::order_fill_i32(o.perm, o.Ns, -1, s));
    HIP_TRY(slhc::order_scatter(o.tmp_b, o.tmp_c, o.shift, n, P, o.Ns, o.perm, o.inv, s));
    HIP_TRY(slhc::order_gather_padded(X, hn, o.perm, o.Ns, n, d, o.Xs, o.hs, s));
    HIP_TRY(slhc::order_tile_balls(o.Xs, o.perm, o.Ns, d, o.tile_c, o.tile_r, s));
    if (o.tile_gap) HIP_TRY(slhc::order_tile_gaps(o.tile_c, o.tile_r, (o.Ns + 127) / 128, d, o.tile_gap, s));
    HIP_TRY(hipStreamSynchronize(s));        // the pinned staging buffer is released on return
    log.mark("row order: %d rows placed in %d (tau %.4g, padding above %.4g), tile balls", n, o.Ns, (double)tau, (double)tau_pad);
    return SLHC_OK;
}

int run_knn(const float* X, int64_t N, int32_t d, int32_t k, int32_t* nbr_idx, float* nbr_dist,
            KnnWs& ws, hipStream_t stream, uint32_t flags, bool* pruned_out = nullptr,
            EventPair* ev_norm = nullptr, EventPair* ev_order = nullptr, EventPair* ev_sweep = nullptr)
{
    hipLaunchKernelGGL(k_zero_words, dim3(1), dim3(64), 0, stream, reinterpret_cast<uint32_t*>(ws.counters), 64);
    HIP_TRY(hipGetLastError());
    if (ev_norm) HIP_TRY(hipEventRecord(ev_norm->a, stream));
    HIP_TRY(slhc::launch_half_norms(X, (int)N, d, ws.hn, stream, reinterpret_cast<unsigned int*>(ws.counters + 4)));
    if (ev_norm) HIP_TRY(hipEventRecord(ev_norm->b, stream));
    const bool prune = (flags & SLHC_PRUNE) && ws.has_order;
    if (pruned_out) *pruned_out = prune;
    if (ev_order) HIP_TRY(hipEventRecord(ev_order->a, stream));
    if (prune) {
        const bool split = ws.Xsplit && ws.hn_split && !(flags & SLHC_FP32_FILTER);
        if (split) {        // X in split halves: for the nearest-pivot sweep here and for every-tile sweeps later
            const int rs = make_split_copy(X, N, d, ws, stream);
            if (rs != SLHC_OK) return rs;
            if (!split_products_pruned_ok(d)) {
                // Below 64 features the pruned sweeps multiply in float32, on the rows as they are: fine unless the
                // rows share an offset far larger than their distances, which then fills the filter's slack and
                // lets every pair of a tile through.  The split copy is taken relative to the column means; when
                // that shrinks the norms eightfold or more, the pruned sweeps multiply it too.
                PinnedHost pin;
                HIP_TRY(pin.alloc(2 * sizeof(float)));
                float* h_sums = static_cast<float*>(pin.p);
                hipLaunchKernelGGL(k_sample_sums, dim3(1), dim3(256), 0, stream, ws.hn, ws.hn_split, (int)N, ws.shift_scratch);
                HIP_TRY(hipGetLastError());
                HIP_TRY(hipMemcpyAsync(h_sums, ws.shift_scratch, 2 * sizeof(float), hipMemcpyDeviceToHost, stream));
                HIP_TRY(hipStreamSynchronize(stream));
                ws.offset_heavy = h_sums[0] >= 8.f * h_sums[1];          // false when either sum is NaN
            }
        }
        const int rc = build_order(X, N, d, ws.hn, reinterpret_cast<const unsigned int*>(ws.counters + 4), ws.order, stream,
                                   split ? ws.Xsplit : nullptr, split ? ws.hn_split : nullptr, split ? ws.shift : nullptr);
        if (rc != SLHC_OK) return rc;
    }
    if (ev_order) HIP_TRY(hipEventRecord(ev_order->b, stream));
    if (ev_sweep) HIP_TRY(hipEventRecord(ev_sweep->a, stream));
    slhc::SweepParams p{};
    p.d = d; p.k = k;
    p.out_idx = nbr_idx; p.out_dist = nbr_dist;
    p.exclude_self = 1;
    p.survivors = ws.counters;
    p.tiles_done = ws.counters + 2;
    if (prune) {
        const OrderWs& o = ws.order;
        p.Xq = p.Xc = o.Xs; p.hq = p.hc = o.hs; p.NQ = p.NC = o.Ns;
        if (o.Xs_split && ws.hn_split && (split_products_pruned_ok(d) || ws.offset_heavy || (o.Xs_local && !(flags & SLHC_ONE_SHIFT))) &&
            !(flags & SLHC_FP32_FILTER)) {
            // the reordered copy in split halves too; its half norms are those of the rows (padding: +inf)
            HIP_TRY(slhc::launch_split_bf16(o.Xs, o.Ns, d, o.Xs_split, stream, ws.shift));
            HIP_TRY(slhc::order_gather_f32(ws.hn_split, o.perm, o.Ns, (int)N, __builtin_inff(), o.hs_split, stream));
            p.Xq_split = p.Xc_split = o.Xs_split; p.hq_split = p.hc_split = o.hs_split;
            ws.order_split_ready = true;
            // (at 32 features the connection sweeps keep float32 products unless the data has a large common offset:
            // the wider filter costs them more than the multiplies save; the k-NN sweep, in local coordinates for the
            // tiles that matter, gains)
            ws.order_split_connect = split_products_pruned_ok(d) || ws.offset_heavy;
        }
        p.q_out_row = o.perm; p.c_id = o.perm;
        p.tile_c = o.tile_c; p.tile_r = o.tile_r; p.gap_ws = o.gap_ws;
        p.tile_gap = (flags & SLHC_NO_TILE_TABLE) ? nullptr : o.tile_gap;
        p.own_tile_first = 1;
        p.panel_counter = reinterpret_cast<unsigned int*>(ws.counters + 8);     // zeroed above
#ifdef SLHC_STUDY_PANEL_STEPS
        p.panel_steps = reinterpret_cast<int*>(o.qslot);       // free until the connection rounds
        HIP_TRY(hipMemsetAsync(o.qslot, 0, (size_t)((o.Ns + 127) / 128) * 8, stream));
#endif
#ifdef SLHC_PHASE_TIMERS
        p.phase_cycles = ws.counters + 16;
#endif
    } else {
        p.Xq = p.Xc = X; p.hq = p.hc = ws.hn; p.NQ = p.NC = (int)N;
        p.part_idx = ws.part_idx; p.part_dist = ws.part_dist; p.part_rows = ws.part_rows;
        if (!(flags & SLHC_PANEL_ORDER)) {
            p.carry_ws = ws.carry_ws; p.carry_ws_words = ws.carry_ws_words;
            p.carry_fault = reinterpret_cast<unsigned int*>(ws.counters + 4);
        }
        if (ws.Xsplit && !(flags & SLHC_FP32_FILTER)) {
            const int rs = make_split_copy(X, N, d, ws, stream);
            if (rs != SLHC_OK) return rs;
            p.Xq_split = p.Xc_split = ws.Xsplit; p.hq_split = p.hc_split = ws.hn_split;
        }
#ifdef SLHC_PHASE_TIMERS
        p.phase_cycles = ws.counters + 16;
#endif
    }
    if (prune && ws.order_split_ready && ws.order.Xs_local && !(flags & SLHC_ONE_SHIFT)) {
        // Two launches (see SweepParams::region_mode).  The rows of a cluster share their centre as an offset that
        // the common shift does not remove, and the filter's slack is a fraction of the squared norms: 1M x 128
        // passes 660 pairs per row on to the exact evaluation for 217 list updates.  The row order keeps a cluster
        // in consecutive tiles, so the tiles are cut into regions where consecutive centres part (farther than
        // twice the larger radius), a second split copy takes every tile relative to the centre of its region's
        // first tile, and the first launch multiplies that copy for the tiles of the panel's own region; the
        // second launch starts from those lists and visits the other tiles with the common shift.
        const OrderWs& o = ws.order;
        const int T = (o.Ns + 127) / 128;
        hipLaunchKernelGGL(k_region_boundaries, dim3((unsigned)((T + 255) / 256)), dim3(256), 0, stream, o.tile_c, o.tile_r, T, d,
                           o.tile_boundary);
        hipLaunchKernelGGL(k_region_scan, dim3(1), dim3(1024), 0, stream, o.tile_boundary, T, o.tile_region, o.tile_first);
        hipLaunchKernelGGL(k_region_last, dim3((unsigned)((T + 255) / 256)), dim3(256), 0, stream, o.tile_boundary, o.tile_first, T,
                           o.tile_last);
        HIP_TRY(hipGetLastError());
        HIP_TRY(slhc::launch_split_bf16(o.Xs, o.Ns, d, o.Xs_local, stream, o.tile_c, o.tile_first));
        HIP_TRY(slhc::launch_half_norms(o.Xs, o.Ns, d, o.hs_local, stream, nullptr, true, o.tile_c, o.tile_first));
        hipLaunchKernelGGL(k_mask_padding, dim3((unsigned)((o.Ns + 255) / 256)), dim3(256), 0, stream, o.perm, o.Ns, o.hs_local);
        HIP_TRY(hipGetLastError());
        slhc::SweepParams own = p;
        own.Xq_split = own.Xc_split = o.Xs_local; own.hq_split = own.hc_split = o.hs_local;
        own.tile_region = o.tile_region; own.region_mode = 1;
        own.tile_first = o.tile_first; own.tile_last = o.tile_last;
        HIP_TRY(slhc::launch_knn_sweep(own, stream));
        hipLaunchKernelGGL(k_zero_words, dim3(1), dim3(64), 0, stream, p.panel_counter, 2);
        HIP_TRY(hipGetLastError());
        p.tile_region = o.tile_region; p.region_mode = 2;
        if (p.tile_gap) {
            hipLaunchKernelGGL(k_region_other_min, dim3((unsigned)T), dim3(256), 0, stream, p.tile_gap, o.tile_region, T, o.region_other_min);
            HIP_TRY(hipGetLastError());
            p.region_other_min = o.region_other_min;
        }
    }
    HIP_TRY(slhc::launch_knn_sweep(p, stream));
    if (ev_sweep) HIP_TRY(hipEventRecord(ev_sweep->b, stream));
    return SLHC_OK;
}

// Linkage arrays from weight-sorted tree edges (paper Sec. 3.3.1): a union-find over the N points
// (union by size, path halving) in which every set carries the dendrogram node created by its last
// merge; merge i creates node N+i.  The edges arrive in weight order, so their end points are
// scattered over the whole array: one 16-byte record per point keeps a find step to one cache
// line, and the records of the edges a few iterations ahead, then their parents, are prefetched.
//
// Merges inside different components of the forest made of the first R edges do not see each other, so
// those components can be worked through by different threads, each in edge order, on one shared array (no
// two of them touch the same record); the edges from R on follow on one thread.  `listed`: those first R
// edge indices grouped by component, ascending inside a component.
struct DendrogramBuilder {
    struct PointSet { int32_t up, count, node, unused; };
    std::unique_ptr<PointSet[]> set;
    int64_t N;
    static constexpr int64_t AHEAD = 16;

    explicit DendrogramBuilder(int64_t N_) : set(new PointSet[(size_t)N_]), N(N_) {}
    void init(int64_t v0, int64_t v1) { for (int64_t v = v0; v < v1; ++v) set[(size_t)v] = PointSet{(int32_t)v, 1, (int32_t)v, 0}; }
    int32_t root(int32_t a)
    {
        while (set[(size_t)a].up != a) {
            set[(size_t)a].up = set[(size_t)set[(size_t)a].up].up;
            a = set[(size_t)a].up;
        }
        return a;
    }
    // Edges j0 .. j1-1 of the streams lo / hi, in order; edge j is merge `first_merge + j`, or merge ids[j]
    // when `ids` is given; its children go to children[2 j ..], its size to sizes[j].  End points outside
    // [0, N) (never produced by a correct caller) are skipped and reported by `false`.
    bool run(const int32_t* lo, const int32_t* hi, const uint32_t* ids, int64_t first_merge, int64_t j0, int64_t j1,
             int32_t* children, int32_t* sizes)
    {
        bool good = true;
        const uint32_t n = (uint32_t)N;
        for (int64_t j = j0; j < j1; ++j) {
            if (j + AHEAD < j1 && (uint32_t)lo[j + AHEAD] < n && (uint32_t)hi[j + AHEAD] < n) {
                __builtin_prefetch(&set[(size_t)lo[j + AHEAD]]);
                __builtin_prefetch(&set[(size_t)hi[j + AHEAD]]);
                // and, half way, the records those point to (their own have arrived by now)
                __builtin_prefetch(&set[(size_t)set[(size_t)lo[j + AHEAD / 2]].up]);
                __builtin_prefetch(&set[(size_t)set[(size_t)hi[j + AHEAD / 2]].up]);
            }
            if ((uint32_t)lo[j] >= n || (uint32_t)hi[j] >= n) { good = false; continue; }
            int32_t ra = root(lo[j]), rb = root(hi[j]);
            const int32_t a = set[(size_t)ra].node, b = set[(size_t)rb].node;
            children[2 * j] = a < b ? a : b;
            children[2 * j + 1] = a < b ? b : a;
            if (set[(size_t)ra].count < set[(size_t)rb].count) std::swap(ra, rb);
            set[(size_t)rb].up = ra;
            set[(size_t)ra].count += set[(size_t)rb].count;
            set[(size_t)ra].node = (int32_t)(N + (ids ? (int64_t)ids[j] : first_merge + j));
            sizes[j] = set[(size_t)ra].count;
        }
        return good;
    }
};

bool build_dendrogram(const int32_t* lo, const int32_t* hi, int64_t N, int32_t* children, int32_t* sizes)
{
    DendrogramBuilder b(N);
    b.init(0, N);
    return b.run(lo, hi, nullptr, 0, 0, N - 1, children, sizes);
}

// The same with `threads` host threads for the first R merges.  Those come grouped by component (`key`,
// equal keys adjacent) and in merge order inside a group: glo / ghi / ids [R] are their end points and merge
// numbers in that order, and their children and sizes are written in that order too (cj [2R], sj [R]).
// Thread t takes the t-th share of the list, moved forward at both ends to the next group boundary.
// The merges from R on follow on one thread: tlo / thi are their end points, tc / ts their output.
bool build_dendrogram_parallel(int64_t N, int64_t R, const uint32_t* key, const int32_t* glo, const int32_t* ghi,
                               const uint32_t* ids, int32_t* cj, int32_t* sj, const int32_t* tlo, const int32_t* thi,
                               int32_t* tc, int32_t* ts, int threads)
{
    // joins what was started even when starting another thread throws
    struct Pool {
        std::vector<std::thread> v;
        void join() { for (auto& th : v) if (th.joinable()) th.join(); }
        ~Pool() { join(); }
    };
    DendrogramBuilder b(N);
    {
        Pool pool;
        for (int t = 0; t < threads; ++t)
            pool.v.emplace_back([&b, N, t, threads] { b.init(N * t / threads, N * (t + 1) / threads); });
        pool.join();
    }
    {
        auto boundary = [&](int64_t j) { while (j > 0 && j < R && key[j] == key[j - 1]) ++j; return j; };
        std::vector<char> good((size_t)threads, 1);
        Pool pool;
        for (int t = 0; t < threads; ++t) {
            const int64_t j0 = boundary(R * t / threads), j1 = t + 1 == threads ? R : boundary(R * (t + 1) / threads);
            char* mine = &good[(size_t)t];
            pool.v.emplace_back([&b, glo, ghi, ids, cj, sj, j0, j1, mine] { *mine = b.run(glo, ghi, ids, 0, j0, j1, cj, sj) ? 1 : 0; });
        }
        pool.join();
        for (char g : good) if (!g) return false;
    }
    return b.run(tlo, thi, nullptr, R, 0, N - 1 - R, tc, ts);
}

int host_threads()
{
    int t = (int)std::thread::hardware_concurrency();
    if (const char* e = std::getenv("SLHC_HOST_THREADS")) { const int v = std::atoi(e); if (v >= 1) t = v; }
    return t < 1 ? 1 : (t > 16 ? 16 : t);
}

// ---- scratch of slhc_knn_graph_static: the workspace of the unpruned k-NN path (counters + one
// half norm per row) for up to SLHC_STATIC_MAX_ROWS rows, as a fixed device array.  Every GPU the
// library runs on holds its own copy at its own address until the process ends; host code never
// uses the array's name as an address, only what hipGetSymbolAddress returns for the current device.
constexpr size_t STATIC_SCRATCH_BYTES = 256 + (size_t)SLHC_STATIC_MAX_ROWS * sizeof(float);
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[MAX_DEVICES] = {};

// Device address of `scratch` on the current device (looked up once per device).
int static_scratch(void** out)
{
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) { set_err("device ordinal %d beyond %d", dev, MAX_DEVICES - 1); return SLHC_UNSUPPORTED; }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) { set_err("hipGetSymbolAddress returned a null address"); return SLHC_HIP_ERROR; }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return SLHC_OK;
}

}  // namespace

extern "C" {

int slhc_abi_version(void) { return SLHC_ABI_VERSION; }

const char* slhc_strerror(int status)
{
    switch (status) {
        case SLHC_OK: return "ok";
        case SLHC_INVALID_ARG: return "invalid argument";
        case SLHC_UNSUPPORTED: return "unsupported size";
        case SLHC_WORKSPACE_TOO_SMALL: return "workspace too small";
        case SLHC_HIP_ERROR: return "HIP error";
        case SLHC_NONFINITE: return "input not finite";
        case SLHC_INTERNAL: return "internal error";
        case SLHC_HOST_MEMORY: return "host allocation failed";
        default: return "unknown status";
    }
}

const char* slhc_last_error(void) { return g_err; }

int slhc_knn_workspace_bytes(int64_t N, int32_t d, int32_t k, size_t* bytes)
{
    return guarded([&]() -> int {
        if (!bytes) { set_err("bytes is NULL"); return SLHC_INVALID_ARG; }
        const int rc = check_shape(N, d, k, true);
        if (rc != SLHC_OK) return rc;
        *bytes = padded_copy_bytes(N, d) + KnnWs(nullptr, N, working_columns(N, d), true, k).bytes;
        return SLHC_OK;
    });
}

int slhc_knn_graph_opt(const float* X, int64_t N, int32_t d, int32_t k, int32_t* nbr_idx, float* nbr_dist,
                       void* workspace, size_t workspace_bytes, void* stream, uint32_t flags)
{
    return guarded([&]() -> int {
        if (!X || !nbr_idx || !nbr_dist || !workspace) { set_err("NULL pointer argument"); return SLHC_INVALID_ARG; }
        const int rc = check_shape(N, d, k, true);
        if (rc != SLHC_OK) return rc;
        const int32_t dw = working_columns(N, d);
        const size_t head = padded_copy_bytes(N, d);
        KnnWs ws(static_cast<unsigned char*>(workspace) + head, N, dw, true, k);
        if (workspace_bytes < head + ws.bytes) { set_err("workspace %zu < %zu bytes", workspace_bytes, head + ws.bytes); return SLHC_WORKSPACE_TOO_SMALL; }
        if (dw != d) {
            const int rp = pad_columns(X, N, d, dw, static_cast<float*>(workspace), static_cast<hipStream_t>(stream));
            if (rp != SLHC_OK) return rp;
            X = static_cast<const float*>(workspace);
        }
        return run_knn(X, N, dw, k, nbr_idx, nbr_dist, ws, static_cast<hipStream_t>(stream), flags);
    });
}

int slhc_knn_graph(const float* X, int64_t N, int32_t d, int32_t k, int32_t* nbr_idx, float* nbr_dist,
                   void* workspace, size_t workspace_bytes, void* stream)
{
    return guarded([&]() -> int {
        return slhc_knn_graph_opt(X, N, d, k, nbr_idx, nbr_dist, workspace, workspace_bytes, stream, 0u);
    });
}

int slhc_knn_graph_static(const float* X, int64_t N, int32_t d, int32_t k, int32_t* nbr_idx, float* nbr_dist,
                          void* stream)
{
    return guarded([&]() -> int {
        if (!X || !nbr_idx || !nbr_dist) { set_err("NULL pointer argument"); return SLHC_INVALID_ARG; }
        const int rc = check_shape(N, d, k, true);
        if (rc != SLHC_OK) return rc;
        if (N > (int64_t)SLHC_STATIC_MAX_ROWS) {
            set_err("N=%lld exceeds SLHC_STATIC_MAX_ROWS=%lld of the fixed scratch array; use slhc_knn_graph with a workspace",
                    (long long)N, (long long)SLHC_STATIC_MAX_ROWS);
            return SLHC_UNSUPPORTED;
        }
        void* ptr = nullptr;
        const int rs = static_scratch(&ptr);
        if (rs != SLHC_OK) return rs;
        KnnWs ws(ptr, N, d, false);                 // counters (cleared by run_knn) + half norms (all N written)
        if (ws.bytes > STATIC_SCRATCH_BYTES) { set_err("scratch layout %zu > %zu bytes", ws.bytes, STATIC_SCRATCH_BYTES); return SLHC_INTERNAL; }
        return run_knn(X, N, d, k, nbr_idx, nbr_dist, ws, static_cast<hipStream_t>(stream), 0u);
    });
}

int slhc_probe_fp32_mfma(double* tflops, void* workspace, size_t workspace_bytes, void* stream)
{
    return guarded([&]() -> int {
        if (!tflops || !workspace) { set_err("NULL pointer argument"); return SLHC_INVALID_ARG; }
        if (workspace_bytes < 256) { set_err("workspace %zu < 256 bytes", workspace_bytes); return SLHC_WORKSPACE_TOO_SMALL; }
        hipStream_t s = static_cast<hipStream_t>(stream);
        EventPair ev;
        HIP_TRY(ev.create());
        double flop = 0.0;
        HIP_TRY(slhc::launch_mfma_probe(2000, static_cast<float*>(workspace), s, &flop));      // warm-up: clocks settle
        HIP_TRY(hipEventRecord(ev.a, s));
        HIP_TRY(slhc::launch_mfma_probe(40000, static_cast<float*>(workspace), s, &flop));     // ~40 ms
        HIP_TRY(hipEventRecord(ev.b, s));
        HIP_TRY(hipStreamSynchronize(s));
        const float ms = ev.ms();
        if (!(ms > 0.f)) { set_err("probe timing failed"); return SLHC_HIP_ERROR; }
        *tflops = flop / (ms * 1e-3) / 1e12;
        return SLHC_OK;
    });
}

int slhc_probe_bf16_mfma(double* tflops, void* workspace, size_t workspace_bytes, void* stream)
{
    return guarded([&]() -> int {
        if (!tflops || !workspace) { set_err("NULL pointer argument"); return SLHC_INVALID_ARG; }
        if (workspace_bytes < 256) { set_err("workspace %zu < 256 bytes", workspace_bytes); return SLHC_WORKSPACE_TOO_SMALL; }
        hipStream_t s = static_cast<hipStream_t>(stream);
        EventPair ev;
        HIP_TRY(ev.create());
        double flop = 0.0;
        HIP_TRY(slhc::launch_mfma_bf16_probe(2000, static_cast<float*>(workspace), s, &flop));     // warm-up: clocks settle
        HIP_TRY(hipEventRecord(ev.a, s));
        HIP_TRY(slhc::launch_mfma_bf16_probe(80000, static_cast<float*>(workspace), s, &flop));    // ~40 ms
        HIP_TRY(hipEventRecord(ev.b, s));
        HIP_TRY(hipStreamSynchronize(s));
        const float ms = ev.ms();
        if (!(ms > 0.f)) { set_err("probe timing failed"); return SLHC_HIP_ERROR; }
        *tflops = flop / (ms * 1e-3) / 1e12;
        return SLHC_OK;
    });
}

int slhc_probe_bf16_mfma_values(const float* A, const float* B, const float* C, float* D, int32_t trials, void* stream)
{
    return guarded([&]() -> int {
        if (!A || !B || !C || !D) { set_err("NULL pointer argument"); return SLHC_INVALID_ARG; }
        if (trials < 0 || trials > (1 << 24)) { set_err("trials must be 0..2^24 (trials=%d)", trials); return SLHC_INVALID_ARG; }
        HIP_TRY(slhc::launch_mfma_bf16_values(A, B, C, D, trials, static_cast<hipStream_t>(stream)));
        return SLHC_OK;
    });
}

int slhc_probe_panel_loop(int32_t steps, double* tflops, void* workspace, size_t workspace_bytes, void* stream)
{
    return guarded([&]() -> int {
        if (!tflops || !workspace) { set_err("NULL pointer argument"); return SLHC_INVALID_ARG; }
        if (steps < 0 || steps > 11) { set_err("steps must be 0..11 (steps=%d)", steps); return SLHC_INVALID_ARG; }
        // a sink word, then the rows to stream from: the largest power of two of 512-byte rows that fits
        if (workspace_bytes < 256 + 512 * 256) { set_err("workspace %zu < %d bytes", workspace_bytes, 256 + 512 * 256); return SLHC_WORKSPACE_TOO_SMALL; }
        int rows = 256;
        while ((size_t)rows * 2 * 512 + 256 <= workspace_bytes && rows < (1 << 22)) rows *= 2;
        float* sink = static_cast<float*>(workspace);
        const float* rows_ptr = reinterpret_cast<const float*>(static_cast<unsigned char*>(workspace) + 256);
        hipStream_t s = static_cast<hipStream_t>(stream);
        EventPair ev;
        HIP_TRY(ev.create());
        double flop = 0.0;
        HIP_TRY(slhc::launch_loop_probe(steps, 500, rows_ptr, rows, sink, s, &flop));           // warm-up: clocks settle
        HIP_TRY(hipEventRecord(ev.a, s));
        HIP_TRY(slhc::launch_loop_probe(steps, 10000, rows_ptr, rows, sink, s, &flop));         // ~40 ms
        HIP_TRY(hipEventRecord(ev.b, s));
        HIP_TRY(hipStreamSynchronize(s));
        const float ms = ev.ms();
        if (!(ms > 0.f)) { set_err("probe timing failed"); return SLHC_HIP_ERROR; }
        *tflops = flop / (ms * 1e-3) / 1e12;
        return SLHC_OK;
    });
}

int slhc_cross_1nn_workspace_bytes(int64_t N, int32_t d, int64_t m, size_t* bytes)
{
    return guarded([&]() -> int {
        if (!bytes) { set_err("bytes is NULL"); return SLHC_INVALID_ARG; }
        const int rc = check_shape(N, d, 1, false);
        if (rc != SLHC_OK) return rc;
        if (m < 0 || m > 2147483647LL) { set_err("bad m"); return SLHC_INVALID_ARG; }
        *bytes = up(32 * sizeof(unsigned long long)) + up((size_t)N * sizeof(float));
        return SLHC_OK;
    });
}

int slhc_cross_1nn(const float* X, int64_t N, int32_t d, const int32_t* colour, const int32_t* rows,
                   int64_t m, int32_t* out_idx, float* out_dist, void* workspace,
                   size_t workspace_bytes, void* stream)
{
    return guarded([&]() -> int {
        if (!X || !colour || !out_idx || !out_dist || !workspace) { set_err("NULL pointer argument"); return SLHC_INVALID_ARG; }
        const int rc = check_shape(N, d, 1, false);
        if (rc != SLHC_OK) return rc;
        if (m < 0 || m > 2147483647LL || (!rows && m > N)) { set_err("bad m=%lld", (long long)m); return SLHC_INVALID_ARG; }
        Carver c(workspace);
        unsigned long long* counters = c.take<unsigned long long>(32);
        float* hn = c.take<float>((size_t)N);
        if (workspace_bytes < c.off) { set_err("workspace %zu < %zu bytes", workspace_bytes, c.off); return SLHC_WORKSPACE_TOO_SMALL; }
        if (m == 0) return SLHC_OK;
        hipStream_t s = static_cast<hipStream_t>(stream);
        hipLaunchKernelGGL(k_zero_words, dim3(1), dim3(64), 0, s, reinterpret_cast<uint32_t*>(counters), 64);
        HIP_TRY(hipGetLastError());
        HIP_TRY(slhc::launch_half_norms(X, (int)N, d, hn, s));
        slhc::SweepParams p{};
        p.Xq = p.Xc = X; p.hq = p.hc = hn; p.NQ = p.NC = (int)N; p.d = d; p.k = 1;
        p.out_idx = out_idx; p.out_dist = out_dist;
        p.qcolour = p.ccolour = colour; p.rows = rows; p.m = (int)m;
        p.survivors = counters;
        HIP_TRY(slhc::launch_cross_1nn_sweep(p, s));
        return SLHC_OK;
    });
}

struct CsrWs {
    int32_t *colour, *ptr, *ext_idx, *cand_u, *hook, *counters, *e_lo, *e_hi;
    float *ext_dist, *cand_w, *e_w;
    uint32_t *best_w, *min_lb, *vals_a, *vals_b;
    unsigned long long *best_e, *keys_a, *keys_b;
    void* sort_temp; size_t sort_temp_bytes;
    size_t bytes;
    CsrWs(void* ws, int64_t V)
    {
        Carver c(ws);
        const size_t n = (size_t)V;
        colour = c.take<int32_t>(n); ptr = c.take<int32_t>(n); ext_idx = c.take<int32_t>(n);
        cand_u = c.take<int32_t>(n); hook = c.take<int32_t>(n); counters = c.take<int32_t>(64);
        e_lo = c.take<int32_t>(n); e_hi = c.take<int32_t>(n);
        ext_dist = c.take<float>(n); cand_w = c.take<float>(n); e_w = c.take<float>(n);
        best_w = c.take<uint32_t>(n); min_lb = c.take<uint32_t>(n);
        vals_a = c.take<uint32_t>(n); vals_b = c.take<uint32_t>(n);
        best_e = c.take<unsigned long long>(n); keys_a = c.take<unsigned long long>(n); keys_b = c.take<unsigned long long>(n);
        sort_temp_bytes = slhc::edge_sort_temp_bytes((int)(V > 1 ? V - 1 : 1));
        sort_temp = c.take<unsigned char>(sort_temp_bytes);
        bytes = c.off;
    }
};

static int csr_shape(int64_t V, int64_t E)
{
    if (V < 1 || E < 0) { set_err("need V >= 1 and E >= 0 (V=%lld E=%lld)", (long long)V, (long long)E); return SLHC_INVALID_ARG; }
    if (V > 2147483646LL || E > 2147483647LL) { set_err("V or E exceeds 2^31-1"); return SLHC_UNSUPPORTED; }
    return SLHC_OK;
}

int slhc_csr_msf_workspace_bytes(int64_t V, int64_t E, size_t* bytes)
{
    return guarded([&]() -> int {
        if (!bytes) { set_err("bytes is NULL"); return SLHC_INVALID_ARG; }
        const int rc = csr_shape(V, E);
        if (rc != SLHC_OK) return rc;
        *bytes = CsrWs(nullptr, V).bytes;
        return SLHC_OK;
    });
}

int slhc_csr_msf(const int32_t* offsets, const int32_t* indices, const float* weights, int64_t V, int64_t E,
                 int32_t* mst_src, int32_t* mst_dst, float* mst_w, int64_t* n_edges, int32_t* colours,
                 int32_t* rounds, void* workspace, size_t workspace_bytes, void* stream)
{
    return guarded([&]() -> int {
        if (!offsets || (E > 0 && (!indices || !weights)) || !mst_src || !mst_dst || !mst_w || !n_edges || !colours || !workspace) {
            set_err("NULL pointer argument");
            return SLHC_INVALID_ARG;
        }
        const int rc = csr_shape(V, E);
        if (rc != SLHC_OK) return rc;
        CsrWs ws(workspace, V);
        if (workspace_bytes < ws.bytes) { set_err("workspace %zu < %zu bytes", workspace_bytes, ws.bytes); return SLHC_WORKSPACE_TOO_SMALL; }
        hipStream_t s = static_cast<hipStream_t>(stream);
        slhc::ForestState f{};
        f.N = (int)V; f.k = 1;
        f.colour = ws.colour; f.ptr = ws.ptr; f.ext_idx = ws.ext_idx; f.ext_dist = ws.ext_dist;
        f.cand_w = ws.cand_w; f.cand_u = ws.cand_u; f.best_w = ws.best_w; f.best_e = ws.best_e;
        f.min_lb = ws.min_lb; f.hook = ws.hook; f.qlist = ws.ptr; f.counters = ws.counters;
        f.e_lo = ws.e_lo; f.e_hi = ws.e_hi; f.e_w = ws.e_w;
        HIP_TRY(slhc::forest_init(f, s));
        HIP_TRY(slhc::forest_csr_check(offsets, indices, weights, (int)V, (int)E, ws.counters, s));
        PinnedHost pin_cnt;
        HIP_TRY(pin_cnt.alloc(64));
        int32_t* h_cnt = static_cast<int32_t*>(pin_cnt.p);
        HIP_TRY(hipMemcpyAsync(h_cnt, ws.counters, 4 * sizeof(int32_t), hipMemcpyDeviceToHost, s));
        HIP_TRY(hipStreamSynchronize(s));
        if (h_cnt[3] != 0) {
            set_err("CSR input check %d failed (20-22: offsets, 23: index out of range, 24: weight negative or not finite)", h_cnt[3]);
            return SLHC_INVALID_ARG;
        }
        int edges = 0, nrounds = 0;
        int max_rounds = 2;
        for (int64_t t = 1; t < V; t *= 2) ++max_rounds;
        // Alg. "MST Algorithm": min edge per vertex, min edge per supervertex, label propagation, until a
        // round adds no edge (the graph's components are then the forest's trees)
        while (edges < V - 1) {
            if (nrounds >= max_rounds) { set_err("no steady state after %d rounds", max_rounds); return SLHC_INTERNAL; }
            ++nrounds;
            HIP_TRY(slhc::forest_round_reset(f, s));
            HIP_TRY(slhc::forest_csr_scan(offsets, indices, weights, (int)E, f, s));
            HIP_TRY(slhc::forest_select_edges(f, s));
            HIP_TRY(slhc::forest_commit(f, s));
            HIP_TRY(slhc::forest_jump(f, 32, false, s));
            HIP_TRY(slhc::forest_jump(f, 32, true, s));
            HIP_TRY(slhc::forest_relabel(f, true, s));
            HIP_TRY(hipMemcpyAsync(h_cnt, ws.counters, 4 * sizeof(int32_t), hipMemcpyDeviceToHost, s));
            HIP_TRY(hipStreamSynchronize(s));
            if (h_cnt[3] != 0) { set_err("forest state check %d failed", h_cnt[3]); return SLHC_INTERNAL; }
            if (h_cnt[2] != 0) {
                // hook chains longer than the two device passes cover: finish them with the host in the loop
                for (int jumps = 0; h_cnt[2] != 0; ++jumps) {
                    if (jumps > 64) { set_err("component hooks do not form a forest (is every edge stored in both rows with one weight?)"); return SLHC_INTERNAL; }
                    hipLaunchKernelGGL(k_zero_words, dim3(1), dim3(64), 0, s, reinterpret_cast<uint32_t*>(ws.counters + 2), 1);
                    HIP_TRY(hipGetLastError());
                    HIP_TRY(slhc::forest_jump(f, 32, true, s));
                    HIP_TRY(hipMemcpyAsync(h_cnt, ws.counters, 4 * sizeof(int32_t), hipMemcpyDeviceToHost, s));
                    HIP_TRY(hipStreamSynchronize(s));
                    if (h_cnt[3] != 0) { set_err("forest state check %d failed", h_cnt[3]); return SLHC_INTERNAL; }
                }
                HIP_TRY(slhc::forest_relabel(f, false, s));
            }
            if (h_cnt[1] < edges || h_cnt[1] > V - 1) { set_err("round left %d edges (had %d)", h_cnt[1], edges); return SLHC_INTERNAL; }
            if (h_cnt[1] == edges) break;                 // steady state: a spanning forest
            edges = h_cnt[1];
        }
        if (edges > 0)
            HIP_TRY(slhc::edge_sort(ws.e_lo, ws.e_hi, ws.e_w, edges, ws.keys_a, ws.keys_b, ws.vals_a, ws.vals_b,
                                    ws.sort_temp, ws.sort_temp_bytes, mst_src, mst_dst, mst_w, s));
        HIP_TRY(hipMemcpyAsync(colours, ws.colour, (size_t)V * sizeof(int32_t), hipMemcpyDeviceToDevice, s));
        HIP_TRY(hipStreamSynchronize(s));
        *n_edges = edges;
        if (rounds) *rounds = nrounds;
        return SLHC_OK;
    });
}

static size_t fused_1nn_layout(void* ws, int64_t m, int64_t n, float** hq, float** hy, unsigned long long** keys)
{
    Carver c(ws);
    *hq = c.take<float>((size_t)m);
    *hy = c.take<float>((size_t)n);
    *keys = c.take<unsigned long long>((size_t)m);
    return c.off;
}

int slhc_fused_1nn_workspace_bytes(int64_t m, int64_t n, int32_t d, size_t* bytes)
{
    return guarded([&]() -> int {
        if (!bytes) { set_err("bytes is NULL"); return SLHC_INVALID_ARG; }
        if (m < 1 || n < 1 || d < 1) { set_err("need m >= 1, n >= 1, d >= 1"); return SLHC_INVALID_ARG; }
        if (m * (int64_t)d > 2147483647LL || n * (int64_t)d > 2147483647LL) { set_err("m*d or n*d exceeds 2^31-1"); return SLHC_UNSUPPORTED; }
        float *hq, *hy; unsigned long long* keys;
        *bytes = fused_1nn_layout(nullptr, m, n, &hq, &hy, &keys);
        return SLHC_OK;
    });
}

int slhc_fused_1nn(const float* Q, int64_t m, const float* Y, int64_t n, int32_t d, int32_t* out_idx,
                   float* out_dist, void* workspace, size_t workspace_bytes, void* stream)
{
    return guarded([&]() -> int {
        if (!Q || !Y || !out_idx || !out_dist || !workspace) { set_err("NULL pointer argument"); return SLHC_INVALID_ARG; }
        if (m < 1 || n < 1 || d < 1) { set_err("need m >= 1, n >= 1, d >= 1"); return SLHC_INVALID_ARG; }
        if (m * (int64_t)d > 2147483647LL || n * (int64_t)d > 2147483647LL) { set_err("m*d or n*d exceeds 2^31-1"); return SLHC_UNSUPPORTED; }
        float *hq, *hy; unsigned long long* keys;
        const size_t need = fused_1nn_layout(workspace, m, n, &hq, &hy, &keys);
        if (workspace_bytes < need) { set_err("workspace %zu < %zu bytes", workspace_bytes, need); return SLHC_WORKSPACE_TOO_SMALL; }
        hipStream_t s = static_cast<hipStream_t>(stream);
        HIP_TRY(slhc::launch_half_norms(Q, (int)m, d, hq, s));
        HIP_TRY(slhc::launch_half_norms(Y, (int)n, d, hy, s));
        slhc::SweepParams p{};
        p.Xq = Q; p.hq = hq; p.NQ = (int)m;
        p.Xc = Y; p.hc = hy; p.NC = (int)n;
        p.d = d; p.k = 1;
        p.out_idx = out_idx; p.out_dist = out_dist;
        HIP_TRY(slhc::launch_segmented_1nn(p, keys, s));
        return SLHC_OK;
    });
}

static int flat_clusters_layout(void* ws, int64_t N, int32_t** above, int32_t** flag, int32_t** rank, void** temp,
                                size_t* temp_bytes, size_t* total)
{
    Carver c(ws);
    const size_t nodes = 2 * (size_t)N;
    *above = c.take<int32_t>(nodes);
    *flag = c.take<int32_t>(nodes);
    *rank = c.take<int32_t>(nodes);
    *temp_bytes = slhc::flat_clusters_scan_temp_bytes((int)N);
    *temp = c.take<unsigned char>(*temp_bytes);
    *total = c.off;
    return SLHC_OK;
}

int slhc_flat_clusters_workspace_bytes(int64_t N, size_t* bytes)
{
    return guarded([&]() -> int {
        if (!bytes) { set_err("bytes is NULL"); return SLHC_INVALID_ARG; }
        if (N < 2) { set_err("need N >= 2 (N=%lld)", (long long)N); return SLHC_INVALID_ARG; }
        if (N > 1073741823LL) { set_err("2N exceeds 2^31-1"); return SLHC_UNSUPPORTED; }
        int32_t *a, *f, *r; void* t; size_t tb;
        return flat_clusters_layout(nullptr, N, &a, &f, &r, &t, &tb, bytes);
    });
}

int slhc_flat_clusters(const int32_t* children, int64_t N, int64_t n_clusters, int32_t* labels,
                       void* workspace, size_t workspace_bytes, void* stream)
{
    return guarded([&]() -> int {
        if (!children || !labels || !workspace) { set_err("NULL pointer argument"); return SLHC_INVALID_ARG; }
        if (N < 2) { set_err("need N >= 2 (N=%lld)", (long long)N); return SLHC_INVALID_ARG; }
        if (N > 1073741823LL) { set_err("2N exceeds 2^31-1"); return SLHC_UNSUPPORTED; }
        if (n_clusters < 1 || n_clusters > N) { set_err("need 1 <= n_clusters <= N (n_clusters=%lld)", (long long)n_clusters); return SLHC_INVALID_ARG; }
        int32_t *above, *flag, *rank; void* temp; size_t temp_bytes, total;
        flat_clusters_layout(workspace, N, &above, &flag, &rank, &temp, &temp_bytes, &total);
        if (workspace_bytes < total) { set_err("workspace %zu < %zu bytes", workspace_bytes, total); return SLHC_WORKSPACE_TOO_SMALL; }
        HIP_TRY(slhc::flat_clusters(children, (int)N, (int)n_clusters, labels, above, flag, rank, temp, temp_bytes,
                                    static_cast<hipStream_t>(stream)));
        return SLHC_OK;
    });
}

int slhc_workspace_bytes(int64_t N, int32_t d, int32_t k, size_t* bytes)
{
    return guarded([&]() -> int {
        if (!bytes) { set_err("bytes is NULL"); return SLHC_INVALID_ARG; }
        const int rc = check_shape(N, d, k, true);
        if (rc != SLHC_OK) return rc;
        *bytes = padded_copy_bytes(N, d) + SlhcWs(nullptr, N, working_columns(N, d), k, true).bytes;
        return SLHC_OK;
    });
}

int slhc_slhc(const float* X, int64_t N, int32_t d, int32_t k, int32_t* mst_src, int32_t* mst_dst,
              float* mst_w, int32_t* children, float* heights, int32_t* sizes, slhc_stats* stats,
              void* workspace, size_t workspace_bytes, void* stream)
{
    return guarded([&]() -> int {
        // below this size the row order costs more than the skipped tiles save (measured on four kinds of data
        // between 4096 and 65 536 rows: the two paths cross between 24 000 and 32 000 rows)
        return slhc_slhc_opt(X, N, d, k, mst_src, mst_dst, mst_w, children, heights, sizes, stats, workspace,
                             workspace_bytes, stream, N >= SLHC_AUTO_PRUNE_MIN_ROWS ? SLHC_PRUNE : 0u);
    });
}

int slhc_slhc_opt(const float* X, int64_t N, int32_t d, int32_t k, int32_t* mst_src, int32_t* mst_dst,
                  float* mst_w, int32_t* children, float* heights, int32_t* sizes, slhc_stats* stats,
                  void* workspace, size_t workspace_bytes, void* stream, uint32_t flags)
{
    return guarded([&]() -> int {
        if (!X || !mst_src || !mst_dst || !mst_w || !children || !heights || !sizes || !workspace) {
            set_err("NULL pointer argument");
            return SLHC_INVALID_ARG;
        }
        const int rc = check_shape(N, d, k, true);
        if (rc != SLHC_OK) return rc;
        const int32_t dw = working_columns(N, d);
        const size_t head = padded_copy_bytes(N, d);
        const size_t need = head + slhc_ws_bytes(N, dw, k, true);
        if (workspace_bytes < need) { set_err("workspace %zu < %zu bytes", workspace_bytes, need); return SLHC_WORKSPACE_TOO_SMALL; }
        if (dw != d) {
            const int rp = pad_columns(X, N, d, dw, static_cast<float*>(workspace), static_cast<hipStream_t>(stream));
            if (rp != SLHC_OK) return rp;
            X = static_cast<const float*>(workspace);
        }
        return run_slhc(X, N, dw, k, mst_src, mst_dst, mst_w, children, heights, sizes, stats,
                        static_cast<unsigned char*>(workspace) + head, static_cast<hipStream_t>(stream), flags, true);
    });
}

}  // extern "C"

namespace {

// The whole pipeline on validated arguments.  `with_order` selects the workspace layout (the
// nested call that clusters the pivots of the row order runs without one).
int run_slhc(const float* X, int64_t N, int32_t d, int32_t k, int32_t* mst_src, int32_t* mst_dst, float* mst_w,
             int32_t* children, float* heights, int32_t* sizes, slhc_stats* stats, void* workspace,
             hipStream_t s, uint32_t flags, bool with_order)
{
    int rc = SLHC_OK;
    SlhcWs ws(workspace, N, d, k, with_order);
    slhc_stats st;
    std::memset(&st, 0, sizeof(st));
    const double t_begin = now_ms();
    PhaseLog log(s);

    // ---- k-NN graph (Alg. "cuSLINK Algorithm", first step)
    EventPair ev_norm, ev_order, ev_knn, ev_conn;
    HIP_TRY(ev_norm.create());
    HIP_TRY(ev_order.create());
    HIP_TRY(ev_knn.create());
    HIP_TRY(ev_conn.create());
    bool pruned = false;
    KnnWs kws(ws.knn_ws, N, d, with_order, k);   // half norms and row order are reused by the connection sweeps
    rc = run_knn(X, N, d, k, ws.nbr_idx, ws.nbr_dist, kws, s, flags, &pruned, &ev_norm, &ev_order, &ev_knn);
    if (rc != SLHC_OK) return rc;
    // The pinned staging of the dendrogram pass is taken here, while the k-NN sweep runs: pinning 28 bytes per row
    // takes the host 2 to 3 ms at a million rows, which would otherwise stand between the edge sort and the pass.
    PinnedHost pin_edges;
    HIP_TRY(pin_edges.alloc((7 * (size_t)(N - 1) + 16) * sizeof(int32_t)));
    PinnedHost pin_surv;
    HIP_TRY(pin_surv.alloc(64));
    unsigned long long* h_surv = static_cast<unsigned long long*>(pin_surv.p);
    HIP_TRY(hipMemcpyAsync(h_surv, kws.counters, 5 * sizeof(unsigned long long), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    if ((h_surv[4] & 2ull) != 0) { set_err("a work item of the k-NN sweep waited for its predecessor in vain"); return SLHC_INTERNAL; }
    if ((h_surv[4] & 0xffffffffull) != 0) { set_err("a row of X is not finite (NaN, infinity, or a squared norm beyond float32)"); return SLHC_NONFINITE; }
    st.knn_filter_survivors = (int64_t)h_surv[0];
    st.knn_tile_steps = (int64_t)h_surv[2];
#ifdef SLHC_STUDY_PANEL_STEPS
    if (pruned) {
        const int T_ = (kws.order.Ns + 127) / 128;
        std::vector<int> hs((size_t)T_ * 2);
        HIP_TRY(hipMemcpy(hs.data(), kws.order.qslot, hs.size() * 4, hipMemcpyDeviceToHost));
        long long tot = 0; int longest = 0, most = 0;
        for (int i = 0; i < T_; ++i) { tot += hs[(size_t)T_ + i]; if (hs[(size_t)T_ + i] > longest) longest = hs[(size_t)T_ + i]; if (hs[(size_t)i] > most) most = hs[(size_t)i]; }
        std::fprintf(stderr, "[study] k-NN sweep: %d panels, kcycles %lld (per WG slot %.0f), longest panel %d kcycles, most steps %d, kernel %.2f ms\n",
                     T_, tot, tot / 512.0, longest, most, ev_knn.ms());
    }
#endif
    st.ms_norm_kernel = ev_norm.ms();
    st.ms_order = ev_order.ms();
    st.ms_knn_kernel = ev_knn.ms();
    log.mark("k-NN graph of %lld rows: order %.2f ms, sweep %.2f ms, %llu tile steps", (long long)N, st.ms_order,
             st.ms_knn_kernel, h_surv[2]);
    const double t_knn = now_ms();
    st.ms_knn = (float)(t_knn - t_begin);

    // ---- certified Boruvka with connection queries (Alg. "MST Algorithm" + "connect_graph")
    slhc::ForestState f{};
    f.N = (int)N; f.k = k;
    f.nbr_idx = ws.nbr_idx; f.nbr_dist = ws.nbr_dist;
    f.colour = ws.colour; f.ptr = ws.ptr; f.ext_idx = ws.ext_idx; f.ext_dist = ws.ext_dist;
    f.cand_w = ws.cand_w; f.cand_u = ws.cand_u; f.best_w = ws.best_w; f.best_e = ws.best_e;
    f.min_lb = ws.min_lb; f.hook = ws.hook; f.qlist = ws.qlist; f.counters = ws.counters;
    f.e_lo = ws.e_lo; f.e_hi = ws.e_hi; f.e_w = ws.e_w;
    HIP_TRY(slhc::forest_init(f, s));
    PinnedHost pin_cnt;
    HIP_TRY(pin_cnt.alloc(64));
    int32_t* h_cnt = static_cast<int32_t*>(pin_cnt.p);
    h_cnt[0] = h_cnt[1] = h_cnt[2] = h_cnt[3] = 0;
    int edges = 0;
    int max_rounds = 2;
    for (int64_t t = 1; t < N; t *= 2) ++max_rounds;
    double ms_connect = 0.0;
    bool first_connect = true;
    // cleared when pruning stops paying: at once when the k-NN sweep already had to multiply more
    // than a quarter of all tile pairs (the data has no structure at the scale of a tile), else by
    // the per-round test below
    const unsigned long long tiles_1d = (unsigned long long)((N + 127) / 128);
    bool connect_pruned = (unsigned long long)st.knn_tile_steps * 4 <= tiles_1d * tiles_1d;
    unsigned long long conn_steps_seen = 0;
    double prev_steps_per_panel = 0.0;     // tile steps per query panel in the last pruned round
    // tile steps per panel that holds a queried row, as far as known: the k-NN sweep's at first, then the last
    // pruned round's; decides into how many parts a panel's scan is worth splitting
    double steps_per_used_panel = pruned ? (double)st.knn_tile_steps / (double)((kws.order.Ns + 127) / 128) : 0.0;
    long long used_panels_round = 0;
    st.components_after_knn = 1;
    // One read-back per round: the scan of the lists for round r+1 is enqueued right behind the relabelling
    // of round r, so the counters that come back carry the edges committed so far, whether the hook
    // chains were followed to their end, and the number of rows the next round has to query.
    auto enqueue_scan = [&]() -> int {
        HIP_TRY(slhc::forest_round_reset(f, s));
        HIP_TRY(slhc::forest_scan_lists(f, s));
        HIP_TRY(slhc::forest_classify(f, s));
        return SLHC_OK;
    };
    auto read_counters = [&]() -> int {
        HIP_TRY(hipMemcpyAsync(h_cnt, ws.counters, 4 * sizeof(int32_t), hipMemcpyDeviceToHost, s));
        HIP_TRY(hipStreamSynchronize(s));
        if (h_cnt[3] != 0) {
            // what the failed check saw (counters[16..22], written by the thread whose report came first)
            HIP_TRY(hipMemcpyAsync(h_cnt + 8, ws.counters + 16, 7 * sizeof(int32_t), hipMemcpyDeviceToHost, s));
            HIP_TRY(hipStreamSynchronize(s));
            set_err("forest state check %d failed in round %d (%s rounds, %d connection rounds): %d %d %d %d %d %d", h_cnt[3],
                    st.boruvka_rounds, pruned ? "pruned" : "every-tile", st.connect_rounds,
                    h_cnt[9], h_cnt[10], h_cnt[11], h_cnt[12], h_cnt[13], h_cnt[14]);
            return SLHC_INTERNAL;
        }
        return SLHC_OK;
    };
    rc = enqueue_scan();
    if (rc != SLHC_OK) return rc;
    for (;;) {
        rc = read_counters();
        if (rc != SLHC_OK) return rc;
        if (st.boruvka_rounds > 0) {
            if (h_cnt[2] != 0) {
                // a hook chain longer than the two device passes cover (a path of > 1000 components): finish
                // it with the host in the loop, relabel, and scan again under the final colours
                for (int jumps = 0; h_cnt[2] != 0; ++jumps) {
                    if (jumps > 64) { set_err("component hooks do not form a forest"); return SLHC_INTERNAL; }
                    hipLaunchKernelGGL(k_zero_words, dim3(1), dim3(64), 0, s, reinterpret_cast<uint32_t*>(ws.counters + 2), 1);
                    HIP_TRY(hipGetLastError());
                    HIP_TRY(slhc::forest_jump(f, 32, true, s));
                    rc = read_counters();
                    if (rc != SLHC_OK) return rc;
                }
                HIP_TRY(slhc::forest_relabel(f, false, s));
                rc = enqueue_scan();
                if (rc != SLHC_OK) return rc;
                rc = read_counters();
                if (rc != SLHC_OK) return rc;
            }
            if (h_cnt[1] <= edges || h_cnt[1] > N - 1) { set_err("round added %d edges (total %d)", h_cnt[1] - edges, h_cnt[1]); return SLHC_INTERNAL; }
            edges = h_cnt[1];
            if (edges == N - 1) break;
        }
        if (st.boruvka_rounds >= max_rounds) { set_err("no single component after %d rounds", max_rounds); return SLHC_INTERNAL; }
        ++st.boruvka_rounds;
        const int nq = h_cnt[0];
        if (h_cnt[3] != 0 || nq < 0 || nq > N) { set_err("forest state check %d failed (nq=%d)", h_cnt[3], nq); return SLHC_INTERNAL; }
        if (nq > 0) {
            const double tc0 = now_ms();
            if (first_connect) { st.components_after_knn = (int32_t)(N - edges); first_connect = false; }
            ++st.connect_rounds;
            const bool round_pruned = pruned && connect_pruned;
            if (round_pruned) {
                // colours in the reordered copy and one colour summary per tile
                const OrderWs& o = kws.order;
                HIP_TRY(slhc::order_gather_i32(ws.colour, o.perm, o.Ns, (int)N, -1, o.colour_s, s));
                HIP_TRY(slhc::order_tile_colours(o.colour_s, o.Ns, o.tile_colour, s));
                // rows per component (vals_b is free until the edge sort): which components may lower
                // their shared threshold during the sweep
                HIP_TRY(slhc::order_fill_i32(reinterpret_cast<int32_t*>(ws.vals_b), (int)N, 0, s));
                HIP_TRY(slhc::forest_component_sizes(o.colour_s, o.Ns, (int)N, reinterpret_cast<int32_t*>(ws.vals_b), s));
            }
            float ms_round_kernels = 0.f;
            // one cross-colour 1-NN sweep for `n` listed rows, and its answers applied to the forest
            auto sweep_rows = [&](const int32_t* rows, int n) -> int {
                slhc::SweepParams p{};
                p.d = d; p.k = 1;
                p.out_idx = ws.q_idx; p.out_dist = ws.q_dist;
                p.m = n;
                p.survivors = kws.counters + 1;
                p.tiles_done = kws.counters + 3;
                if (round_pruned) {
                    // the queried rows marked in place so that query panels coincide with candidate tiles
                    const OrderWs& o = kws.order;
                    HIP_TRY(slhc::order_fill_i32(o.qslot, o.Ns, -1, s));
                    HIP_TRY(slhc::order_scatter_slots(o.inv, rows, n, (int)N, o.Ns, o.qslot, s));
                    // A launch with few panels is as long as its longest panel, and a panel whose queries admit
                    // thousands of tiles outlasts the others several times over: with fewer non-empty panels
                    // than SPLIT_ITEMS_TARGET, every panel's scan is split into parts (see the kernel).
                    int32_t* used = ws.counters + 12;
                    hipLaunchKernelGGL(k_zero_words, dim3(1), dim3(64), 0, s, reinterpret_cast<uint32_t*>(used), 1);
                    HIP_TRY(hipGetLastError());
                    HIP_TRY(slhc::order_count_used_tiles(o.qslot, o.Ns, used, o.tile_list, s));
                    HIP_TRY(hipMemcpyAsync(h_cnt + 6, used, sizeof(int32_t), hipMemcpyDeviceToHost, s));
                    HIP_TRY(hipStreamSynchronize(s));
                    const int used_panels = h_cnt[6] > 0 ? h_cnt[6] : 1;
                    used_panels_round += used_panels;
                    int parts = SPLIT_ITEMS_TARGET / used_panels;
                    const int worth = (int)(steps_per_used_panel / SPLIT_MIN_STEPS);      // a part should have some tiles to multiply
                    if (parts > worth) parts = worth;
                    p.segments = parts < 2 ? 1 : (parts > SPLIT_MAX_PARTS ? SPLIT_MAX_PARTS : parts);
                    if (flags & SLHC_SPLIT_SCANS) p.segments = 5;
                    if (h_cnt[6] < 0 || h_cnt[6] > (o.Ns + 127) / 128) { set_err("bad count of queried tiles %d", h_cnt[6]); return SLHC_INTERNAL; }
                    p.panel_list = o.tile_list; p.panel_list_n = h_cnt[6];
                    p.Xq = p.Xc = o.Xs; p.hq = p.hc = o.hs; p.NQ = p.NC = o.Ns;
                    if (kws.order_split_connect) { p.Xq_split = p.Xc_split = o.Xs_split; p.hq_split = p.hc_split = o.hs_split; }
                    p.qcolour = p.ccolour = o.colour_s;
                    p.qslot = o.qslot;
                    p.c_id = o.perm;
                    p.tile_c = o.tile_c; p.tile_r = o.tile_r; p.gap_ws = o.gap_ws;
                    p.tile_gap = (flags & SLHC_NO_TILE_TABLE) ? nullptr : o.tile_gap;
                    p.tile_colour = o.tile_colour;
                    // thresholds shared by the queries of a component: what the forest already knows (a
                    // working copy that the sweep lowers further as its queries find lighter edges;
                    // vals_a is free until the edge sort)
                    HIP_TRY(hipMemcpyAsync(ws.vals_a, ws.best_w, (size_t)N * sizeof(uint32_t), hipMemcpyDeviceToDevice, s));
                    p.comp_best = ws.vals_a;
#ifndef SLHC_STUDY_NO_LOWERING
                    p.comp_best_lower = ws.vals_a;      // lowered in place; forest_apply_queries reads the final values
                    p.comp_lower_factor = LOWER_FACTOR;
                    p.comp_size = reinterpret_cast<const int32_t*>(ws.vals_b);
                    p.comp_lower_min_size = LOWER_MIN_ROWS;
#endif
                    p.comp_count = (int)N;
                    p.panel_counter = reinterpret_cast<unsigned int*>(kws.counters + 8);
#ifdef SLHC_PHASE_TIMERS
                    p.phase_cycles = kws.counters + 24;
#endif
                    hipLaunchKernelGGL(k_zero_words, dim3(1), dim3(64), 0, s, p.panel_counter, 1);
                    HIP_TRY(hipGetLastError());
                } else {
                    p.Xq = p.Xc = X; p.hq = p.hc = kws.hn; p.NQ = p.NC = (int)N;
                    p.qcolour = p.ccolour = ws.colour;
                    p.rows = rows;
                    if (!(flags & SLHC_PANEL_ORDER)) {
                        p.carry_ws = kws.carry_ws; p.carry_ws_words = kws.carry_ws_words;
                        p.carry_fault = reinterpret_cast<unsigned int*>(kws.counters + 4);
                    }
                    if (kws.Xsplit && !(flags & SLHC_FP32_FILTER)) {
                        if (!kws.split_ready) {          // (a pruned k-NN sweep did not need it)
                            const int rs = make_split_copy(X, N, d, kws, s);
                            if (rs != SLHC_OK) return rs;
                        }
                        // (a launch that ends in a kernel with float32 products takes hq / hc)
                        p.Xq_split = p.Xc_split = kws.Xsplit; p.hq_split = p.hc_split = kws.hn_split;
                    }
                }
#ifdef SLHC_STUDY_PANEL_STEPS
                int* study_steps = reinterpret_cast<int*>(kws.order.gap_ws);    // unused while the table of tile pairs serves
                const int study_panels = (kws.order.Ns + 127) / 128;
                if (round_pruned) { HIP_TRY(hipMemsetAsync(study_steps, 0, (size_t)study_panels * 8, s)); p.panel_steps = study_steps; }
#endif
                HIP_TRY(hipEventRecord(ev_conn.a, s));
                // keys_a / keys_b are free until the edge sort (the two-phase split above keeps its row lists in keys_a,
                // in pruned rounds only)
                HIP_TRY(slhc::launch_segmented_cross_1nn(p, round_pruned ? ws.keys_b : ws.keys_a, s));
                HIP_TRY(hipEventRecord(ev_conn.b, s));
                HIP_TRY(slhc::forest_apply_queries(f, rows, ws.q_idx, ws.q_dist, n, round_pruned ? ws.vals_a : nullptr, s));
                HIP_TRY(hipMemcpyAsync(h_cnt + 7, ws.counters + 3, sizeof(int32_t), hipMemcpyDeviceToHost, s));
                HIP_TRY(hipStreamSynchronize(s));
                if (h_cnt[7] == 14) {
                    // an answer inside the query's own component: say what the sweep was given
                    HIP_TRY(hipMemcpy(h_cnt + 8, ws.counters + 16, 7 * sizeof(int32_t), hipMemcpyDeviceToHost));
                    const int q = h_cnt[9], v = h_cnt[10], u = h_cnt[11];
                    int dv[12] = {-9, -9, -9, -9, -9, -9, -9, -9, -9, -9, -9, -9};
                    auto peek = [&](const void* base, long long index, int* out) {
                        if (base && index >= 0) (void)hipMemcpy(out, static_cast<const int32_t*>(base) + index, 4, hipMemcpyDeviceToHost);
                    };
                    peek(ws.colour, v, &dv[0]); peek(ws.colour, u, &dv[1]);
                    peek(ws.q_idx, q, &dv[2]); peek(rows, q, &dv[3]);
                    if (round_pruned) {
                        const OrderWs& o = kws.order;
                        peek(o.inv, v, &dv[4]); peek(o.inv, u, &dv[5]);
                        if (dv[4] >= 0 && dv[4] < o.Ns) { peek(o.colour_s, dv[4], &dv[6]); peek(o.qslot, dv[4], &dv[8]); peek(o.perm, dv[4], &dv[10]); }
                        if (dv[5] >= 0 && dv[5] < o.Ns) { peek(o.colour_s, dv[5], &dv[7]); peek(o.qslot, dv[5], &dv[9]); peek(o.perm, dv[5], &dv[11]); }
                    }
                    set_err("sweep answer inside the query's component: round %d, %s sweep of %d rows in %d parts, q %d v %d u %d; "
                            "colour v %d u %d, q_idx[q] %d rows[q] %d, position v %d u %d, colour_s %d %d, qslot %d %d, perm %d %d",
                            st.boruvka_rounds, round_pruned ? "pruned" : "every-tile", n, p.segments, q, v, u,
                            dv[0], dv[1], dv[2], dv[3], dv[4], dv[5], dv[6], dv[7], dv[8], dv[9], dv[10], dv[11]);
                    return SLHC_INTERNAL;
                }
#ifdef SLHC_STUDY_PANEL_STEPS
                if (round_pruned) {
                    std::vector<int> hs((size_t)study_panels * 2);
                    HIP_TRY(hipMemcpy(hs.data(), study_steps, hs.size() * 4, hipMemcpyDeviceToHost));
                    std::vector<int> order_((size_t)study_panels);
                    for (int i = 0; i < study_panels; ++i) order_[(size_t)i] = i;
                    std::sort(order_.begin(), order_.end(), [&](int a, int b) { return hs[(size_t)study_panels + a] > hs[(size_t)study_panels + b]; });
                    long long tot_steps = 0, tot_cyc = 0; int used = 0;
                    for (int i = 0; i < study_panels; ++i) { tot_steps += hs[(size_t)i]; tot_cyc += hs[(size_t)study_panels + i]; used += hs[(size_t)study_panels + i] > 0; }
                    std::fprintf(stderr, "[study] %d rows, %d panels used, parts %d, steps %lld, kcycles %lld (per WG slot %.0f), kernel %.2f ms\n", n, used, p.segments, tot_steps, tot_cyc, tot_cyc / 512.0, ev_conn.ms());
                    for (int r = 0; r < 12; ++r) { const int i = order_[(size_t)r]; std::fprintf(stderr, "[study]   panel %d: steps %d kcycles %d\n", i, hs[(size_t)i], hs[(size_t)study_panels + i]); }
                }
#endif
                ms_round_kernels += ev_conn.ms();
                return SLHC_OK;
            };
            int queried = nq;
            const bool split_round = (flags & SLHC_SPLIT_ROUNDS)
                                         ? nq >= 256
                                         : ((int64_t)nq * 2 >= N && (int64_t)nq >= TWO_PHASE_MIN_ROWS &&
                                            prev_steps_per_panel >= TWO_PHASE_MIN_STEPS);
            if (round_pruned && split_round) {
                // Two phases, for a round that queries most rows while the thresholds the forest has
                // are loose (the last pruned round multiplied hundreds of tiles per panel).  The rows
                // of every 16th panel go first; what they find lowers their components' best
                // weights, and the other rows (those the lower weights still leave on the list) then
                // run under thresholds close to the final ones, which lets their panels skip tiles.
                int32_t* part_a = reinterpret_cast<int32_t*>(ws.keys_a);      // free until the edge sort
                int32_t* part_b = part_a + N;
                int32_t* counts = ws.counters + 8;
                hipLaunchKernelGGL(k_zero_words, dim3(1), dim3(64), 0, s, reinterpret_cast<uint32_t*>(counts), 3);
                HIP_TRY(hipGetLastError());
                HIP_TRY(slhc::forest_split_queries(f, ws.qlist, nq, kws.order.inv, TWO_PHASE_STRIDE, part_a, part_b, counts, s));
                HIP_TRY(hipMemcpyAsync(h_cnt + 4, counts, 2 * sizeof(int32_t), hipMemcpyDeviceToHost, s));
                HIP_TRY(hipStreamSynchronize(s));
                const int na = h_cnt[4], nb = h_cnt[5];
                if (na < 0 || nb < 0 || na + nb != nq) { set_err("query split lost rows (%d + %d of %d)", na, nb, nq); return SLHC_INTERNAL; }
                if (na > 0) { const int rc = sweep_rows(part_a, na); if (rc != SLHC_OK) return rc; }
                int nb_left = 0;
                if (nb > 0) {
                    HIP_TRY(slhc::forest_still_needed(f, part_b, nb, ws.qlist, counts + 2, s));
                    HIP_TRY(hipMemcpyAsync(h_cnt + 4, counts + 2, sizeof(int32_t), hipMemcpyDeviceToHost, s));
                    HIP_TRY(hipStreamSynchronize(s));
                    nb_left = h_cnt[4];
                    if (nb_left < 0 || nb_left > nb) { set_err("query re-filter kept %d of %d rows", nb_left, nb); return SLHC_INTERNAL; }
                    if (nb_left > 0) { const int rc = sweep_rows(ws.qlist, nb_left); if (rc != SLHC_OK) return rc; }
                }
                queried = na + nb_left;
            } else {
                const int rc = sweep_rows(ws.qlist, nq);
                if (rc != SLHC_OK) return rc;
            }
            st.connect_query_rows += queried;
            if (round_pruned) HIP_TRY(hipMemcpyAsync(h_surv, kws.counters, 4 * sizeof(unsigned long long), hipMemcpyDeviceToHost, s));
            HIP_TRY(hipStreamSynchronize(s));
            st.ms_connect_kernels += ms_round_kernels;
            ms_connect += now_ms() - tc0;
            if (round_pruned) {
                // Did skipping pay?  A pruned tile step costs more than an every-tile one (queries
                // stay aligned with tiles, so panels are partly empty, and the surviving tiles are
                // the dense ones); when a large round still multiplied more than a third of what the
                // every-tile sweep would, the remaining rounds run without pruning.
                const unsigned long long steps = h_surv[3] - conn_steps_seen;
                conn_steps_seen = h_surv[3];
                prev_steps_per_panel = (double)steps / (double)((queried + 127) / 128 > 0 ? (queried + 127) / 128 : 1);
                if (used_panels_round > 0) steps_per_used_panel = (double)steps / (double)used_panels_round;
                used_panels_round = 0;
                const unsigned long long every = (unsigned long long)((nq + 127) / 128) * (unsigned long long)((N + 127) / 128);
                if ((int64_t)nq * 8 >= N && steps * 3 > every) connect_pruned = false;
            }
            if (log.on) {
                HIP_TRY(hipMemcpyAsync(h_surv, kws.counters, 4 * sizeof(unsigned long long), hipMemcpyDeviceToHost, s));
                HIP_TRY(hipStreamSynchronize(s));
                log.mark("round %d: %d components, %d of %d listed rows queried, sweeps %.2f ms, %llu tile steps so far",
                         st.boruvka_rounds, (int)(N - edges), queried, nq, ms_round_kernels, h_surv[3]);
            }
        }
        HIP_TRY(slhc::forest_select_edges(f, s));
        HIP_TRY(slhc::forest_commit(f, s));
        HIP_TRY(slhc::forest_jump(f, 32, false, s));          // hooks -> new roots
        HIP_TRY(slhc::forest_jump(f, 32, true, s));
        HIP_TRY(slhc::forest_relabel(f, true, s));
        rc = enqueue_scan();                                  // next round's scan; its counters are read at the top
        if (rc != SLHC_OK) return rc;
    }
    HIP_TRY(hipMemcpyAsync(h_surv, kws.counters, 5 * sizeof(unsigned long long), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    if ((h_surv[4] & 2ull) != 0) { set_err("a work item of a connection sweep waited for its predecessor in vain"); return SLHC_INTERNAL; }
#ifdef SLHC_PHASE_TIMERS
    if (log.on) {
        unsigned long long* h_ph = h_surv + 4;           // 64-byte staging buffer: not enough, use two copies
        for (int part = 0; part < 4; ++part) {
            HIP_TRY(hipMemcpyAsync(h_ph, kws.counters + 16 + 4 * part, 4 * sizeof(unsigned long long), hipMemcpyDeviceToHost, s));
            HIP_TRY(hipStreamSynchronize(s));
            std::fprintf(stderr, "[slhc] %s phase cycles %d..%d: %llu %llu %llu %llu\n", part < 2 ? "k-NN" : "connect",
                         4 * (part & 1), 4 * (part & 1) + 3, h_ph[0], h_ph[1], h_ph[2], h_ph[3]);
        }
    }
#endif
    st.connect_filter_survivors = (int64_t)h_surv[1];
    st.connect_tile_steps = (int64_t)h_surv[3];
    st.pruned = pruned ? 1 : 0;
    st.split_products = (kws.split_ready || kws.order_split_ready) ? 1 : 0;
    if (pruned) { st.order_pivots = kws.order.P; st.order_padded_rows = kws.order.Ns; }
    const double t_forest = now_ms();
    st.ms_connect = (float)ms_connect;
    st.ms_boruvka = (float)(t_forest - t_knn - ms_connect);

    // ---- sort by weight (Sec. 3.3.1), then the sequential relabelling on the host
    HIP_TRY(slhc::edge_sort(ws.e_lo, ws.e_hi, ws.e_w, (int)(N - 1), ws.keys_a, ws.keys_b, ws.vals_a, ws.vals_b,
                            ws.sort_temp, ws.sort_temp_bytes, mst_src, mst_dst, mst_w, s));
    HIP_TRY(hipMemcpyAsync(heights, mst_w, (size_t)(N - 1) * sizeof(float), hipMemcpyDeviceToDevice, s));
    HIP_TRY(hipStreamSynchronize(s));
    const double t_sort = now_ms();
    st.ms_sort = (float)(t_sort - t_forest);

    const size_t E = (size_t)(N - 1);
    // Large trees: all but the heaviest sixteenth of the edges are grouped by the component they lie in when
    // only those edges are there (labels on the device, a stable sort by label), and host threads share the
    // groups; see build_dendrogram_parallel.  The arrays of the forest rounds are free by now.
    const int threads = host_threads();
    int64_t R = 0;
    uint32_t* key_sorted = reinterpret_cast<uint32_t*>(ws.ptr);
    uint32_t* listed = reinterpret_cast<uint32_t*>(ws.hook);
    int32_t* glo = ws.qlist;
    int32_t* ghi = ws.cand_u;
    if (N >= DENDROGRAM_THREADS_MIN_ROWS && threads >= 2) {
        const int64_t heavy = (int64_t)E / 16 > 4096 ? (int64_t)E / 16 : 4096;
        R = (int64_t)E - heavy;
        int32_t* changed = ws.counters + 8;
        int32_t* h_changed = reinterpret_cast<int32_t*>(h_surv + 7);      // last word of the 64-byte staging buffer
        bool settled = false;
        for (int pass = 0; pass < 64 && !settled; ++pass) {
            hipLaunchKernelGGL(k_zero_words, dim3(1), dim3(64), 0, s, reinterpret_cast<uint32_t*>(changed), 1);
            HIP_TRY(hipGetLastError());
            HIP_TRY(slhc::prefix_forest_pass(mst_src, mst_dst, (int)R, (int)N, ws.colour, changed, pass == 0, s));
            HIP_TRY(hipMemcpyAsync(h_changed, changed, 4, hipMemcpyDeviceToHost, s));
            HIP_TRY(hipStreamSynchronize(s));
            settled = *h_changed == 0;
        }
        if (settled) {
            HIP_TRY(slhc::prefix_forest_keys(mst_src, ws.colour, (int)R, (int)N, ws.vals_a, ws.vals_b, s));
            HIP_TRY(slhc::pair_sort_u32(ws.vals_a, key_sorted, ws.vals_b, listed, (int)R, bits_for(N), ws.sort_temp,
                                        ws.sort_temp_bytes, s));
            HIP_TRY(slhc::prefix_forest_gather(mst_src, mst_dst, listed, (int)R, glo, ghi, s));
        } else {
            R = 0;
        }
    }
    // host staging: end points (grouped part in list order, then the rest in edge order), keys and merge numbers
    // of the grouped part, children and sizes in the same two parts
    const size_t Rz = (size_t)R, Tz = E - Rz;
    int32_t* h_lo = static_cast<int32_t*>(pin_edges.p);     // [R] grouped, [E - R] rest (5 E + 2 R words in all)
    int32_t* h_hi = h_lo + E;
    int32_t* h_children = h_hi + E;                         // 2E entries, same two parts
    int32_t* h_sizes = h_children + 2 * E;
    uint32_t* h_key = reinterpret_cast<uint32_t*>(h_sizes + E);
    uint32_t* h_ids = h_key + Rz;
    if (Rz) {
        HIP_TRY(hipMemcpyAsync(h_lo, glo, Rz * 4, hipMemcpyDeviceToHost, s));
        HIP_TRY(hipMemcpyAsync(h_hi, ghi, Rz * 4, hipMemcpyDeviceToHost, s));
        HIP_TRY(hipMemcpyAsync(h_key, key_sorted, Rz * 4, hipMemcpyDeviceToHost, s));
        HIP_TRY(hipMemcpyAsync(h_ids, listed, Rz * 4, hipMemcpyDeviceToHost, s));
    }
    HIP_TRY(hipMemcpyAsync(h_lo + Rz, mst_src + Rz, Tz * 4, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipMemcpyAsync(h_hi + Rz, mst_dst + Rz, Tz * 4, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    log.mark("dendrogram: %zu edges staged on the host (%lld grouped for %d threads)", E, (long long)R, threads);
    const bool good = Rz ? build_dendrogram_parallel(N, R, h_key, h_lo, h_hi, h_ids, h_children, h_sizes, h_lo + Rz, h_hi + Rz,
                                                     h_children + 2 * Rz, h_sizes + Rz, threads)
                         : build_dendrogram(h_lo, h_hi, N, h_children, h_sizes);
    if (!good) { set_err("dendrogram: an edge of the sorted tree has an end point outside [0, N)"); return SLHC_INTERNAL; }
    log.mark("dendrogram: union-find");
    if (Rz) {
        // the grouped part goes back to edge order on the device (the sort's scratch arrays are free again)
        int32_t* cj = reinterpret_cast<int32_t*>(ws.keys_a);            // 2R words of the N 64-bit words
        int32_t* sj = reinterpret_cast<int32_t*>(ws.vals_a);
        HIP_TRY(hipMemcpyAsync(cj, h_children, Rz * 8, hipMemcpyHostToDevice, s));
        HIP_TRY(hipMemcpyAsync(sj, h_sizes, Rz * 4, hipMemcpyHostToDevice, s));
        HIP_TRY(slhc::prefix_forest_scatter(listed, cj, sj, (int)R, children, sizes, s));
    }
    HIP_TRY(hipMemcpyAsync(children + 2 * Rz, h_children + 2 * Rz, Tz * 8, hipMemcpyHostToDevice, s));
    HIP_TRY(hipMemcpyAsync(sizes + Rz, h_sizes + Rz, Tz * 4, hipMemcpyHostToDevice, s));
    HIP_TRY(hipStreamSynchronize(s));
    const double t_end = now_ms();
    st.ms_dendrogram = (float)(t_end - t_sort);
    st.ms_total = (float)(t_end - t_begin);
    if (stats) *stats = st;
    return SLHC_OK;
}

}  // namespace
