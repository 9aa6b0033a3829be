// C ABI of the library (see include/slhc.h) and the host orchestration of the cuSLINK pipeline:
// Alg. "cuSLINK Algorithm" (k-NN graph -> MST -> connect -> relabel), Alg. "connect_graph",
// Alg. "MST Algorithm" of the paper, restructured as one certified Boruvka loop (see
// forest_kernels.hip for what "certified" means).
#include <hip/hip_runtime.h>
#include <chrono>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <vector>

#include "../../include/slhc.h"
#include "forest_kernels.h"
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

struct KnnWs {
    unsigned long long* survivors;
    float* hn;
    size_t bytes;
    KnnWs(void* ws, int64_t N)
    {
        Carver c(ws);
        survivors = c.take<unsigned long long>(32);
        hn = c.take<float>((size_t)N);
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
    SlhcWs(void* ws, int64_t N, int32_t k)
    {
        Carver c(ws);
        const size_t n = (size_t)N;
        knn_ws = c.take<unsigned char>(KnnWs(nullptr, N).bytes);
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
        sort_temp_bytes = slhc::edge_sort_temp_bytes((int)(N - 1));
        sort_temp = c.take<unsigned char>(sort_temp_bytes);
        bytes = c.off;
    }
};

int run_knn(const float* X, int64_t N, int32_t d, int32_t k, int32_t* nbr_idx, float* nbr_dist,
            void* workspace, hipStream_t stream, unsigned long long** survivors_out,
            EventPair* ev_norm = nullptr, EventPair* ev_sweep = nullptr)
{
    KnnWs ws(workspace, N);
    hipLaunchKernelGGL(k_zero_words, dim3(1), dim3(64), 0, stream, reinterpret_cast<uint32_t*>(ws.survivors), 64);
    HIP_TRY(hipGetLastError());
    if (ev_norm) HIP_TRY(hipEventRecord(ev_norm->a, stream));
    HIP_TRY(slhc::launch_half_norms(X, (int)N, d, ws.hn, stream));
    if (ev_norm) HIP_TRY(hipEventRecord(ev_norm->b, stream));
    if (ev_sweep) HIP_TRY(hipEventRecord(ev_sweep->a, stream));
    slhc::SweepParams p{};
    p.X = X; p.hn = ws.hn; p.N = (int)N; p.d = d; p.k = k;
    p.out_idx = nbr_idx; p.out_dist = nbr_dist;
    p.colour = nullptr; p.rows = nullptr; p.m = 0;
    p.survivors = ws.survivors;
    HIP_TRY(slhc::launch_knn_sweep(p, stream));
    if (ev_sweep) HIP_TRY(hipEventRecord(ev_sweep->b, stream));
    if (survivors_out) *survivors_out = ws.survivors;
    return SLHC_OK;
}

double now_ms()
{
    using clk = std::chrono::steady_clock;
    return std::chrono::duration<double, std::milli>(clk::now().time_since_epoch()).count();
}

// Linkage arrays from weight-sorted tree edges (paper Sec. 3.3.1): a union-find over the
// 2N-1 dendrogram nodes in which the representative of a set is the node created by its last
// merge; merge i creates node N+i.
void build_dendrogram(const int32_t* lo, const int32_t* hi, int64_t N, int32_t* children, int32_t* sizes)
{
    const int64_t total = 2 * N - 1;
    std::vector<int32_t> up_node((size_t)total);
    std::vector<int32_t> count((size_t)total, 1);
    for (int64_t i = 0; i < total; ++i) up_node[(size_t)i] = (int32_t)i;
    auto top = [&](int32_t a) {
        while (up_node[(size_t)a] != a) {                       // path halving
            up_node[(size_t)a] = up_node[(size_t)up_node[(size_t)a]];
            a = up_node[(size_t)a];
        }
        return a;
    };
    for (int64_t i = 0; i < N - 1; ++i) {
        const int32_t a = top(lo[i]), b = top(hi[i]);
        const int32_t node = (int32_t)(N + i);
        children[2 * i] = a < b ? a : b;
        children[2 * i + 1] = a < b ? b : a;
        up_node[(size_t)a] = node;
        up_node[(size_t)b] = node;
        count[(size_t)node] = count[(size_t)a] + count[(size_t)b];
        sizes[i] = count[(size_t)node];
    }
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
        case SLHC_INTERNAL: return "internal error";
        default: return "unknown status";
    }
}

const char* slhc_last_error(void) { return g_err; }

int slhc_knn_workspace_bytes(int64_t N, int32_t d, int32_t k, size_t* bytes)
{
    if (!bytes) { set_err("bytes is NULL"); return SLHC_INVALID_ARG; }
    const int rc = check_shape(N, d, k, true);
    if (rc != SLHC_OK) return rc;
    *bytes = KnnWs(nullptr, N).bytes;
    return SLHC_OK;
}

int slhc_knn_graph(const float* X, int64_t N, int32_t d, int32_t k, int32_t* nbr_idx, float* nbr_dist,
                   void* workspace, size_t workspace_bytes, void* stream)
{
    if (!X || !nbr_idx || !nbr_dist || !workspace) { set_err("NULL pointer argument"); return SLHC_INVALID_ARG; }
    const int rc = check_shape(N, d, k, true);
    if (rc != SLHC_OK) return rc;
    const size_t need = KnnWs(nullptr, N).bytes;
    if (workspace_bytes < need) { set_err("workspace %zu < %zu bytes", workspace_bytes, need); return SLHC_WORKSPACE_TOO_SMALL; }
    return run_knn(X, N, d, k, nbr_idx, nbr_dist, workspace, static_cast<hipStream_t>(stream), nullptr);
}

int slhc_cross_1nn_workspace_bytes(int64_t N, int32_t d, int64_t m, size_t* bytes)
{
    if (!bytes) { set_err("bytes is NULL"); return SLHC_INVALID_ARG; }
    const int rc = check_shape(N, d, 1, false);
    if (rc != SLHC_OK) return rc;
    if (m < 0 || m > 2147483647LL) { set_err("bad m"); return SLHC_INVALID_ARG; }
    *bytes = KnnWs(nullptr, N).bytes;
    return SLHC_OK;
}

int slhc_cross_1nn(const float* X, int64_t N, int32_t d, const int32_t* colour, const int32_t* rows,
                   int64_t m, int32_t* out_idx, float* out_dist, void* workspace,
                   size_t workspace_bytes, void* stream)
{
    if (!X || !colour || !out_idx || !out_dist || !workspace) { set_err("NULL pointer argument"); return SLHC_INVALID_ARG; }
    const int rc = check_shape(N, d, 1, false);
    if (rc != SLHC_OK) return rc;
    if (m < 0 || m > 2147483647LL || (!rows && m > N)) { set_err("bad m=%lld", (long long)m); return SLHC_INVALID_ARG; }
    const size_t need = KnnWs(nullptr, N).bytes;
    if (workspace_bytes < need) { set_err("workspace %zu < %zu bytes", workspace_bytes, need); return SLHC_WORKSPACE_TOO_SMALL; }
    if (m == 0) return SLHC_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    KnnWs ws(workspace, N);
    hipLaunchKernelGGL(k_zero_words, dim3(1), dim3(64), 0, s, reinterpret_cast<uint32_t*>(ws.survivors), 64);
    HIP_TRY(hipGetLastError());
    HIP_TRY(slhc::launch_half_norms(X, (int)N, d, ws.hn, s));
    slhc::SweepParams p{};
    p.X = X; p.hn = ws.hn; p.N = (int)N; p.d = d; p.k = 1;
    p.out_idx = out_idx; p.out_dist = out_dist;
    p.colour = colour; p.rows = rows; p.m = (int)m;
    p.survivors = ws.survivors;
    HIP_TRY(slhc::launch_cross_1nn_sweep(p, s));
    return SLHC_OK;
}

int slhc_workspace_bytes(int64_t N, int32_t d, int32_t k, size_t* bytes)
{
    if (!bytes) { set_err("bytes is NULL"); return SLHC_INVALID_ARG; }
    const int rc = check_shape(N, d, k, true);
    if (rc != SLHC_OK) return rc;
    *bytes = SlhcWs(nullptr, N, k).bytes;
    return SLHC_OK;
}

int slhc_slhc(const float* X, int64_t N, int32_t d, int32_t k, int32_t* mst_src, int32_t* mst_dst,
              float* mst_w, int32_t* children, float* heights, int32_t* sizes, slhc_stats* stats,
              void* workspace, size_t workspace_bytes, void* stream)
{
    if (!X || !mst_src || !mst_dst || !mst_w || !children || !heights || !sizes || !workspace) {
        set_err("NULL pointer argument");
        return SLHC_INVALID_ARG;
    }
    int rc = check_shape(N, d, k, true);
    if (rc != SLHC_OK) return rc;
    SlhcWs ws(workspace, N, k);
    if (workspace_bytes < ws.bytes) { set_err("workspace %zu < %zu bytes", workspace_bytes, ws.bytes); return SLHC_WORKSPACE_TOO_SMALL; }
    hipStream_t s = static_cast<hipStream_t>(stream);
    slhc_stats st;
    std::memset(&st, 0, sizeof(st));
    const double t_begin = now_ms();

    // ---- k-NN graph (Alg. "cuSLINK Algorithm", first step)
    unsigned long long* d_surv = nullptr;
    EventPair ev_norm, ev_knn, ev_conn;
    HIP_TRY(ev_norm.create());
    HIP_TRY(ev_knn.create());
    HIP_TRY(ev_conn.create());
    rc = run_knn(X, N, d, k, ws.nbr_idx, ws.nbr_dist, ws.knn_ws, s, &d_surv, &ev_norm, &ev_knn);
    if (rc != SLHC_OK) return rc;
    PinnedHost pin_surv;
    HIP_TRY(pin_surv.alloc(64));
    unsigned long long* h_surv = static_cast<unsigned long long*>(pin_surv.p);
    HIP_TRY(hipMemcpyAsync(h_surv, d_surv, sizeof(unsigned long long), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    st.knn_filter_survivors = (int64_t)h_surv[0];
    st.ms_norm_kernel = ev_norm.ms();
    st.ms_knn_kernel = ev_knn.ms();
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
    KnnWs kws(ws.knn_ws, N);       // the half norms computed for the k-NN sweep are reused
    PinnedHost pin_cnt;
    HIP_TRY(pin_cnt.alloc(64));
    int32_t* h_cnt = static_cast<int32_t*>(pin_cnt.p);
    h_cnt[0] = h_cnt[1] = h_cnt[2] = h_cnt[3] = 0;
    int edges = 0;
    int max_rounds = 2;
    for (int64_t t = 1; t < N; t *= 2) ++max_rounds;
    double ms_connect = 0.0;
    bool first_connect = true;
    st.components_after_knn = 1;
    while (edges < N - 1) {
        if (st.boruvka_rounds >= max_rounds) { set_err("no single component after %d rounds", max_rounds); return SLHC_INTERNAL; }
        ++st.boruvka_rounds;
        HIP_TRY(slhc::forest_round_reset(f, s));
        HIP_TRY(slhc::forest_scan_lists(f, s));
        HIP_TRY(slhc::forest_classify(f, s));
        HIP_TRY(hipMemcpyAsync(h_cnt, ws.counters, 4 * sizeof(int32_t), hipMemcpyDeviceToHost, s));
        HIP_TRY(hipStreamSynchronize(s));
        const int nq = h_cnt[0];
        if (h_cnt[3] != 0 || nq < 0 || nq > N) { set_err("forest state check %d failed (nq=%d)", h_cnt[3], nq); return SLHC_INTERNAL; }
        if (nq > 0) {
            const double tc0 = now_ms();
            if (first_connect) { st.components_after_knn = (int32_t)(N - edges); first_connect = false; }
            ++st.connect_rounds;
            st.connect_query_rows += nq;
            slhc::SweepParams p{};
            p.X = X; p.hn = kws.hn; p.N = (int)N; p.d = d; p.k = 1;
            p.out_idx = ws.q_idx; p.out_dist = ws.q_dist;
            p.colour = ws.colour; p.rows = ws.qlist; p.m = nq;
            p.survivors = kws.survivors + 1;
            HIP_TRY(hipEventRecord(ev_conn.a, s));
            HIP_TRY(slhc::launch_cross_1nn_sweep(p, s));
            HIP_TRY(hipEventRecord(ev_conn.b, s));
            HIP_TRY(slhc::forest_apply_queries(f, ws.q_idx, ws.q_dist, nq, s));
            HIP_TRY(hipStreamSynchronize(s));
            st.ms_connect_kernels += ev_conn.ms();
            ms_connect += now_ms() - tc0;
        }
        HIP_TRY(slhc::forest_select_edges(f, s));
        HIP_TRY(slhc::forest_commit(f, s));
        int jumps = 0;
        do {                                                  // pointer doubling to the new roots
            hipLaunchKernelGGL(k_zero_words, dim3(1), dim3(64), 0, s, reinterpret_cast<uint32_t*>(ws.counters + 2), 1);
            HIP_TRY(hipGetLastError());
            HIP_TRY(slhc::forest_jump(f, s));
            HIP_TRY(hipMemcpyAsync(h_cnt, ws.counters, 4 * sizeof(int32_t), hipMemcpyDeviceToHost, s));
            HIP_TRY(hipStreamSynchronize(s));
            if (++jumps > 64) { set_err("component hooks do not form a forest"); return SLHC_INTERNAL; }
            if (h_cnt[3] != 0) { set_err("forest state check %d failed", h_cnt[3]); return SLHC_INTERNAL; }
        } while (h_cnt[2] != 0);
        HIP_TRY(slhc::forest_relabel(f, s));
        if (h_cnt[1] <= edges || h_cnt[1] > N - 1) { set_err("round added %d edges (total %d)", h_cnt[1] - edges, h_cnt[1]); return SLHC_INTERNAL; }
        edges = h_cnt[1];
    }
    HIP_TRY(hipMemcpyAsync(h_surv, kws.survivors + 1, sizeof(unsigned long long), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    st.connect_filter_survivors = (int64_t)h_surv[0];
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
    PinnedHost pin_edges;
    HIP_TRY(pin_edges.alloc(E * 5 * sizeof(int32_t)));
    int32_t* h_lo = static_cast<int32_t*>(pin_edges.p);
    int32_t* h_hi = h_lo + E;
    int32_t* h_children = h_hi + E;          // 2E entries
    int32_t* h_sizes = h_children + 2 * E;
    HIP_TRY(hipMemcpyAsync(h_lo, mst_src, E * 4, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipMemcpyAsync(h_hi, mst_dst, E * 4, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    build_dendrogram(h_lo, h_hi, N, h_children, h_sizes);
    HIP_TRY(hipMemcpyAsync(children, h_children, E * 8, hipMemcpyHostToDevice, s));
    HIP_TRY(hipMemcpyAsync(sizes, h_sizes, E * 4, hipMemcpyHostToDevice, s));
    HIP_TRY(hipStreamSynchronize(s));
    const double t_end = now_ms();
    st.ms_dendrogram = (float)(t_end - t_sort);
    st.ms_total = (float)(t_end - t_begin);
    if (stats) *stats = st;
    return SLHC_OK;
}

}  // extern "C"
