/*
 * slhc.h - C ABI of the MI355X (gfx950) single-linkage clustering library.
 *
 * The library implements the data-parallel path of cuSLINK (Nolet et al., "cuSLINK:
 * Single-linkage Agglomerative Clustering on the GPU", ECML PKDD 2023):
 *   fused brute-force k-NN graph  ->  Boruvka minimum spanning forest over the k-NN lists  ->
 *   cross-component nearest-neighbour connection until the forest is the exact minimum spanning
 *   tree  ->  weight-sorted edges  ->  dendrogram in scipy linkage layout.
 *
 * Conventions for every entry point
 *   - Pointers marked DEVICE are device memory of the current HIP device, owned by the caller
 *     (for instance the data_ptr() of a torch tensor).  Pointers marked HOST are host memory.
 *     The library never frees or keeps a caller pointer after the call returns, and it never
 *     modifies an input.
 *   - X is row-major float32 [N, d].  Distances are squared Euclidean.  Values must be finite and
 *     small enough that a row's squared norm is finite in float32: slhc_slhc / slhc_slhc_opt and
 *     the SLHC_PRUNE form of slhc_knn_graph_opt detect a violation and return SLHC_NONFINITE.  The
 *     asynchronous entry points cannot return what only the device knows: there a row with a
 *     non-finite norm is never reported as anybody's neighbour, and the entries of its own result
 *     are unspecified except that every index written is -1 or a valid row.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - `workspace` is DEVICE scratch of at least the size the matching *_workspace_bytes call
 *     reports, 256-byte aligned; its contents on entry are ignored and on exit unspecified.
 *   - Every function returns an slhc_status.  No C++ exception crosses the boundary (a failed
 *     host allocation becomes SLHC_HOST_MEMORY).  On any status other than SLHC_OK the outputs are
 *     unspecified.  slhc_last_error() gives a thread-local detail string for the last failing call
 *     of the calling thread.
 *   - Device memory: the library allocates none; everything it needs is in `workspace`.  Host
 *     memory: the synchronous entry points (slhc_slhc*, slhc_csr_msf, and slhc_knn_graph_opt with
 *     SLHC_PRUNE) allocate pinned staging buffers and HIP events for the duration of the call
 *     (slhc_slhc: up to 28 bytes per row of pinned memory and 16 bytes per row of pageable memory for
 *     the host dendrogram pass) and free them before returning.
 *     The library keeps no mutable state between calls other than the thread-local error text
 *     (and the fixed scratch array of slhc_knn_graph_static, see there).
 *   - Calls that share a workspace must not overlap in time.  Calls on different streams with
 *     different workspaces and outputs are independent.
 */
#ifndef SLHC_H
#define SLHC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SLHC_ABI_VERSION 4

/* Largest k of the fused path: the selection keeps one list entry per lane of a 64-wide
 * wavefront.  (The paper's fused k-NN has the same limit, Sec. 2 and Sec. 3.1.1: k <= 64.) */
#define SLHC_MAX_K 64

typedef enum slhc_status {
    SLHC_OK = 0,
    SLHC_INVALID_ARG = 1,        /* null pointer, N < 2, d < 1, k < 1, k > N-1, malformed CSR input */
    SLHC_UNSUPPORTED = 2,        /* k > SLHC_MAX_K, or N*k / N*d beyond the 2^31-1 element indexing */
    SLHC_WORKSPACE_TOO_SMALL = 3,
    SLHC_HIP_ERROR = 4,          /* a HIP call failed; see slhc_last_error()                      */
    SLHC_NONFINITE = 5,          /* a row of X has a NaN, an infinity, or a squared norm that
                                    overflows float32 (found on the device by the norm kernel)    */
    SLHC_INTERNAL = 6,           /* a consistency check of the forest state failed, or the
                                    connection loop did not reach one component in
                                    ceil(log2 N) + 2 rounds (cannot happen for finite input)      */
    SLHC_HOST_MEMORY = 7         /* a host allocation failed                                      */
} slhc_status;

/* Counters and stage times of one slhc_slhc call (HOST struct, filled when not NULL). */
typedef struct slhc_stats {
    int32_t boruvka_rounds;          /* rounds of min-edge + relabel                              */
    int32_t connect_rounds;          /* rounds in which the cross-component 1-NN kernel ran        */
    int32_t components_after_knn;    /* components when the k-NN lists alone could add no edge     */
    int32_t order_pivots;            /* pivots of the row order (0 when not pruned)                */
    int64_t knn_filter_survivors;    /* pairs that passed the MFMA filter in the k-NN sweep        */
    int64_t connect_query_rows;      /* sum over connection rounds of queried rows                 */
    int64_t connect_filter_survivors;
    float ms_knn;                    /* norms + fused k-NN (host clock, includes the sync)         */
    float ms_boruvka;                /* all min-edge / commit / relabel kernels                    */
    float ms_connect;                /* all cross-component 1-NN sweeps                            */
    float ms_sort;                   /* edge sort                                                  */
    float ms_dendrogram;             /* device->host copy, host union-find, host->device copy      */
    float ms_total;
    float ms_norm_kernel;            /* HIP-event time of the half-norm kernel                     */
    float ms_knn_kernel;             /* HIP-event time of the fused k-NN sweep kernel alone        */
    float ms_connect_kernels;        /* HIP-event time summed over the cross-component 1-NN sweeps */
    float ms_order;                  /* HIP-event time of building the row order + tile balls     */
    int64_t knn_tile_steps;          /* (query panel, candidate tile) pairs the k-NN sweep multiplied;
                                        ceil(N/128)^2 when nothing is pruned (either sweep kernel)  */
    int64_t connect_tile_steps;      /* same, summed over the connection sweeps                    */
    int32_t pruned;                  /* 1 when tile pruning was active in this call                */
    int32_t order_padded_rows;       /* rows of the reordered copy incl. padding (0 when not pruned) */
    int32_t split_products;          /* 1 when the k-NN sweep formed its tile products from split bfloat16
                                        halves (see SLHC_FP32_FILTER), 0 when in float32              */
    int32_t reserved0;
} slhc_stats;

/* Option flags of the *_opt entry points. */
#define SLHC_PRUNE 1u   /* reorder rows spatially and skip (query panel, candidate tile) pairs whose
                           bounding balls prove that no pair can enter a list.  Results are identical
                           to the unpruned sweep; only available for d <= 128 and N >= 512 (ignored
                           otherwise).  Not in the paper, whose k-NN multiplies every tile.
                           Building the row order reads counters back, so a call with this flag
                           is synchronous and allocates pinned host staging while it runs.      */
#define SLHC_SPLIT_ROUNDS 2u   /* slhc_slhc_opt with SLHC_PRUNE only; a testing and tuning aid.  Every
                           pruned connection round of at least 256 query rows runs in two phases
                           (a sample of the row panels first, the rest under the thresholds that
                           leaves), which the library otherwise does only for rounds of >= 262144
                           rows under loose thresholds.  Same outputs.                          */
#define SLHC_SPLIT_SCANS 4u    /* slhc_slhc_opt with SLHC_PRUNE only; a testing and tuning aid.  Every
                           pruned connection sweep splits each query panel's scan of the candidate
                           tiles into 5 work items that exchange what they find, which the library
                           otherwise does (in 2 to 16 parts) only for launches with few panels and
                           long scans.  Same outputs.                                           */
#define SLHC_NO_TILE_TABLE 8u  /* with SLHC_PRUNE only; a testing aid.  The pruned sweeps compute the lower
                           bounds of every query panel against the candidate tiles themselves, as
                           they do for row orders of more than 32768 tiles, instead of reading them
                           from the table of all tile pairs.  Same outputs.                     */
#define SLHC_FP32_FILTER 16u   /* The sweeps accumulate their tile products in float32 (fp32 MFMA), as the
                           pruned sweeps always do below 64 features, instead of in split bfloat16 halves
                           (bf16 MFMA, 16 times the rate), which is the default of slhc_knn_graph* and
                           slhc_slhc* (these work on a copy of X with zero columns appended: whole chunks of
                           32 columns up to 128 features, a multiple of 4 beyond; a zero column changes no
                           bit of any distance).  Only the filter differs: every
                           pair that may enter a list is re-evaluated in float32 either way, so the
                           outputs are the same bit for bit.                                     */

#define SLHC_ONE_SHIFT 64u     /* with SLHC_PRUNE only; a testing and tuning aid.  The pruned k-NN sweep otherwise runs
                           as two launches where its products come from split bfloat16 halves (64 to 128
                           features): the candidate tiles of a row panel's own region (a run of tiles whose
                           centres stay close: a cluster) from a copy taken relative to a centre of that
                           region, which keeps the cluster's position out of the filter's slack, then the
                           other tiles from the copy relative to the column means.  With this flag: one launch,
                           all tiles from the latter copy.  Same outputs.                              */
#define SLHC_PANEL_ORDER 32u   /* A testing and tuning aid.  Every-tile sweeps of many query panels (from 4 panels
                           per workgroup slot on, d <= 128) otherwise hand out their work range by range:
                           the candidate tiles are cut into ranges of about 32 MiB, all workgroups sweep the
                           same range at a time (served by the memory-side cache instead of being fetched
                           from memory once per panel), and a panel's lists and thresholds travel from range to
                           range through the output arrays.  With this flag every workgroup sweeps all
                           candidates for one panel at a time, as the smaller launches do.  Same outputs.
                           (Going range by range, a work item waits for the item that wrote its panel's
                           lists one range earlier; the wait is bounded, and if it ever ran out the
                           synchronous entry points would return SLHC_INTERNAL.  slhc_knn_graph is
                           asynchronous and cannot; the condition has never been observed.)            */

int slhc_abi_version(void);
const char* slhc_strerror(int status);          /* static string, never NULL */
const char* slhc_last_error(void);              /* thread-local, never NULL  */

/*
 * k-NN graph (paper Sec. 3.1.1, Alg. "Fused k-NN" with its epilogues in Appendix A).
 *
 * For every row i the k rows j != i with the smallest (||x_i - x_j||^2, j), ascending.
 * The distance tile x_i . x_j is computed on fp32 MFMA and only used to discard pairs that
 * cannot enter a row's list; a pair that may enter is re-evaluated as sum_t (x_it - x_jt)^2
 * in fp32, so the reported value of (i,j) equals that of (j,i) bit for bit and duplicates are at
 * exactly 0.  A row is never its own neighbour (excluded by index, not by distance).
 * (How many pairs reach the re-evaluation depends on the rows' squared norms against their distances.
 * slhc_knn_graph, slhc_knn_graph_opt and slhc_slhc* multiply a copy of X taken relative to its column
 * means, so an offset shared by all rows costs nothing; slhc_knn_graph_static, slhc_cross_1nn and
 * slhc_fused_1nn multiply the rows as they are, and on rows whose common offset dwarfs their distances
 * they re-evaluate most pairs: same results, far slower.  Centre such data before calling them.)
 *
 *   X         DEVICE in   [N*d]
 *   nbr_idx   DEVICE out  [N*k] row-major int32
 *   nbr_dist  DEVICE out  [N*k] row-major float32
 * slhc_knn_graph (and _opt with flags = 0) is asynchronous: work is enqueued on `stream`; outputs
 * are complete when the stream reaches the end of that work; errors detected on the host are
 * reported immediately.  With SLHC_PRUNE the call is synchronous (see the flag).
 */
int slhc_knn_workspace_bytes(int64_t N, int32_t d, int32_t k, size_t* bytes /* HOST out */);
int slhc_knn_graph(const float* X, int64_t N, int32_t d, int32_t k,
                   int32_t* nbr_idx, float* nbr_dist,
                   void* workspace, size_t workspace_bytes, void* stream);
/* Same result; flags = 0 is slhc_knn_graph (every tile multiplied, as in the paper). */
int slhc_knn_graph_opt(const float* X, int64_t N, int32_t d, int32_t k,
                       int32_t* nbr_idx, float* nbr_dist,
                       void* workspace, size_t workspace_bytes, void* stream, uint32_t flags);

/*
 * slhc_knn_graph for callers that cannot allocate and have no workspace to pass: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels and the same
 * result as slhc_knn_graph, bit for bit; the scratch they need (a block of counters and one
 * float per row) is a fixed device array inside the library of 256 + 4 * SLHC_STATIC_MAX_ROWS
 * bytes, which every GPU the library runs on holds until the process ends.  The call allocates
 * and frees nothing, on the device or on the host (its first call on a device looks up the
 * array's address).  N > SLHC_STATIC_MAX_ROWS is rejected with SLHC_UNSUPPORTED.
 * All calls on one GPU share that array: two calls that overlap in time on one GPU (different
 * streams or threads) race; calls in order on one stream are safe.  Asynchronous on `stream`.
 * The counters are cleared by a kernel, not a memset node, so the call may be captured.
 */
#define SLHC_STATIC_MAX_ROWS 1048576
int slhc_knn_graph_static(const float* X, int64_t N, int32_t d, int32_t k,
                          int32_t* nbr_idx, float* nbr_dist, void* stream);

/*
 * Measurement aid for the roofline report of the distance tiles (paper Sec. 3.1.1, the tile contraction
 * of Alg. "Fused k-NN"): runs the MFMA instruction the sweep kernels use (v_mfma_f32_32x32x2_f32, four
 * independent accumulator blocks per wavefront, two workgroups of four wavefronts per compute unit) on
 * operands that stay in registers, for about 40 ms, and reports the rate it sustained.
 *
 *   tflops     HOST   out  10^12 floating-point operations per second
 *   workspace  DEVICE      at least 256 bytes
 * Synchronous.
 */
int slhc_probe_fp32_mfma(double* tflops, void* workspace, size_t workspace_bytes, void* stream);
/* The same for v_mfma_f32_32x32x16_bf16, the multiply of the sweeps that form their tile products from split
 * bfloat16 halves (SLHC_FP32_FILTER describes them); same arguments. */
int slhc_probe_bf16_mfma(double* tflops, void* workspace, size_t workspace_bytes, void* stream);
/*
 * Checking aid for the filter slack of those sweeps (paper Sec. 3.1.1: the tile contraction; how far its value may
 * be off decides which pairs must be re-evaluated): one v_mfma_f32_32x32x16_bf16 per trial on the caller's values,
 *   D[t] = C[t] + sum_{k<16} A[16 t + k] * B[16 t + k],
 * so that a test can compare the instruction with an exact sum.  A, B [16 * trials], C, D [trials]: DEVICE,
 * float32, A and B holding bfloat16-representable values (others are rounded to bfloat16 first).  Asynchronous
 * on `stream`; 0 <= trials <= 2^24.
 */
int slhc_probe_bf16_mfma_values(const float* A, const float* B, const float* C, float* D, int32_t trials, void* stream);

/*
 * Measurement aid like slhc_probe_fp32_mfma, for the panel loop of the sweeps (paper Sec. 3.1.1, the
 * `gemm_nt_loop` of Alg. "Fused k-NN"): the same multiplies with the loop's ingredients added one by one,
 * so that a run shows which of them costs MFMA rate.
 *   steps = 0  operands in registers (what slhc_probe_fp32_mfma runs)
 *           1  + one workgroup barrier per chunk of 64 multiplies, A operands read from LDS
 *           2  + the next chunk of a 128-row tile loaded from the workspace and stored to LDS
 *           3  + the filter: 16 compares and a ballot per accumulator block and tile
 *           4  as 2, the chunk loaded from global memory straight into LDS (no register staging)
 *           5  as 3, likewise
 *           6  as 2, the two wavefronts that share a SIMD run at different priorities
 *           7  as 3, likewise
 *   tflops     HOST   out
 *   workspace  DEVICE      at least 131 328 bytes, contents irrelevant but finite floats; steps >= 2
 *                          stream their tiles from it (the more, the less of the stream hits in L2)
 * Synchronous.
 */
int slhc_probe_panel_loop(int32_t steps, double* tflops, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Cross-component 1-NN (paper Sec. 3.1.2, Alg. "Fused 1-NN", used by Alg. "connect_graph").
 *
 * For each query row rows[q], q < m: the row j with colour[j] != colour[rows[q]] that minimises
 * (||x_rows[q] - x_j||^2, j).  out_idx[q] = -1 and out_dist[q] = +inf when every row has the
 * query's colour.  Same filter-then-re-evaluate arithmetic as slhc_knn_graph.
 *
 *   X        DEVICE in  [N*d]       colour   DEVICE in  [N] int32
 *   rows     DEVICE in  [m] int32   (each in [0, N); NULL means rows 0..m-1, then m <= N)
 *   out_idx  DEVICE out [m] int32   out_dist DEVICE out [m] float32
 * The row list lives on the device, so it is not validated on the host: an entry outside [0, N)
 * is not dereferenced and gets out_idx = -1, out_dist = +inf.
 * Asynchronous on `stream` like slhc_knn_graph.
 */
int slhc_cross_1nn_workspace_bytes(int64_t N, int32_t d, int64_t m, size_t* bytes /* HOST out */);
int slhc_cross_1nn(const float* X, int64_t N, int32_t d, const int32_t* colour,
                   const int32_t* rows, int64_t m, int32_t* out_idx, float* out_dist,
                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * Fused 1-NN between two matrices (paper Sec. 3.1.2, Alg. "Fused 1-NN"; the m x n shapes of the
 * paper's 1-NN benchmark, few queries against a large index).
 *
 * For each query row q < m: the index row j < n that minimises (||Q_q - Y_j||^2, j), and that
 * distance.  Same filter-then-re-evaluate arithmetic as slhc_knn_graph; nothing is excluded (a
 * query that also is an index row finds itself at distance 0).  With few query rows the index rows
 * are split over the workgroups and the partial minima are merged by a 64-bit atomic minimum over
 * (distance bits, index), so the result does not depend on the split.
 *
 *   Q        DEVICE in  [m*d]        Y         DEVICE in  [n*d]
 *   out_idx  DEVICE out [m] int32    out_dist  DEVICE out [m] float32
 * Asynchronous on `stream`.
 */
int slhc_fused_1nn_workspace_bytes(int64_t m, int64_t n, int32_t d, size_t* bytes /* HOST out */);
int slhc_fused_1nn(const float* Q, int64_t m, const float* Y, int64_t n, int32_t d,
                   int32_t* out_idx, float* out_dist,
                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * Single-linkage clustering (paper Alg. "cuSLINK Algorithm" without the final flat cut:
 * k-NN graph, Sec. 3.1.1; MST by Boruvka with colours, Sec. 3.2, Alg. "MST Algorithm";
 * connection of the forest, Sec. 3.1.2, Alg. "connect_graph"; sorted edges and dendrogram,
 * Sec. 3.3.1).
 *
 * The tree returned is the exact minimum spanning tree of the complete squared-L2 graph under
 * the strict edge order (weight, min endpoint, max endpoint), with weights evaluated as in
 * slhc_knn_graph.  A component adds its lightest known outgoing edge only once that edge is
 * proven lighter than every pair the k-NN lists do not cover; rows for which this cannot be
 * proven are sent to the cross-component 1-NN.
 *
 *   X         DEVICE in   [N*d]
 *   mst_src   DEVICE out  [N-1] int32   smaller endpoint
 *   mst_dst   DEVICE out  [N-1] int32   larger endpoint
 *   mst_w     DEVICE out  [N-1] float32 ascending by (w, src, dst)
 *   children  DEVICE out  [(N-1)*2] int32: merge i joins nodes children[2i] < children[2i+1]
 *                         into node N+i; ids below N are the input rows
 *   heights   DEVICE out  [N-1] float32 = mst_w (merge i has the weight of sorted edge i)
 *   sizes     DEVICE out  [N-1] int32 rows under node N+i
 *   stats     HOST   out  optional
 * Synchronous: returns after the outputs are complete (the dendrogram pass runs on the host, as
 * in the paper, so the call has to wait for the device anyway).  From 200 000 rows on that pass starts
 * host threads of its own, at most 16 and at most the number of hardware threads; SLHC_HOST_THREADS in
 * the environment sets another number (1: none).  The result does not depend on it.
 */
int slhc_workspace_bytes(int64_t N, int32_t d, int32_t k, size_t* bytes /* HOST out */);
int slhc_slhc(const float* X, int64_t N, int32_t d, int32_t k,
              int32_t* mst_src, int32_t* mst_dst, float* mst_w,
              int32_t* children, float* heights, int32_t* sizes,
              slhc_stats* stats, void* workspace, size_t workspace_bytes, void* stream);
/* slhc_slhc is slhc_slhc_opt with flags = SLHC_PRUNE from SLHC_AUTO_PRUNE_MIN_ROWS rows on and with flags = 0
 * below (building the row order costs more than it saves there; slhc_stats.pruned tells which ran);
 * flags = 0 multiplies every tile in the k-NN and connection sweeps (the paper's brute-force method).
 * Same outputs either way. */
#define SLHC_AUTO_PRUNE_MIN_ROWS 24576
int slhc_slhc_opt(const float* X, int64_t N, int32_t d, int32_t k,
                  int32_t* mst_src, int32_t* mst_dst, float* mst_w,
                  int32_t* children, float* heights, int32_t* sizes,
                  slhc_stats* stats, void* workspace, size_t workspace_bytes, void* stream,
                  uint32_t flags);

/*
 * Minimum spanning forest of a weighted undirected graph in CSR form (paper Sec. 3.2 "Spanning Trees",
 * Alg. "MST Algorithm", Sec. 3.2.2 and 3.2.3; the API of the paper's MST listing: CSR graph in, edge
 * list and colours out).
 *
 * Boruvka rounds with colours: every vertex finds its first outgoing edge in the strict order
 * (weight, min endpoint, max endpoint), every component keeps the first of those, components hook and
 * are relabelled, until a round adds no edge.  Under that order the forest is unique.  No weight
 * alteration is applied (ties and zero weights are handled by the order).
 *
 *   offsets   DEVICE in   [V+1] int32, offsets[0] = 0, offsets[V] = E, non-decreasing
 *   indices   DEVICE in   [E] int32 in [0, V)
 *   weights   DEVICE in   [E] float32, finite and >= 0 (SLHC_INVALID_ARG otherwise; the maximum
 *                         spanning tree by negated weights is not supported)
 *             Every undirected edge must be stored in both rows with the same weight; self loops and
 *             parallel edges are allowed.  An asymmetric graph can make the components hook in a cycle,
 *             which is reported as SLHC_INTERNAL.
 *   mst_src   DEVICE out  [V-1 capacity] int32, smaller endpoint     } the first *n_edges entries,
 *   mst_dst   DEVICE out  [V-1 capacity] int32, larger endpoint      } ascending by (w, src, dst)
 *   mst_w     DEVICE out  [V-1 capacity] float32                     }
 *   n_edges   HOST   out  V minus the number of connected components
 *   colours   DEVICE out  [V] int32: the same vertex id for all vertices of a connected component
 *   rounds    HOST   out  optional: Boruvka rounds used
 * Synchronous (the round loop reads a counter back every round, as the paper's host loop does).
 */
int slhc_csr_msf_workspace_bytes(int64_t V, int64_t E, size_t* bytes /* HOST out */);
int slhc_csr_msf(const int32_t* offsets, const int32_t* indices, const float* weights,
                 int64_t V, int64_t E, int32_t* mst_src, int32_t* mst_dst, float* mst_w,
                 int64_t* n_edges, int32_t* colours, int32_t* rounds,
                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * Flat clusters (paper Sec. 3.3.2, Alg. "extract_flattened_clusters" and Alg. "inherit_labels").
 *
 * Cuts the dendrogram after its first N - n_clusters merges.  The nodes that exist at that level
 * and are not merged further are the cluster roots; they are numbered 0 .. n_clusters-1 in
 * ascending order of node id (a row keeps its id, merge i is node N+i), and labels[v] is the number
 * of the root above row v.  With n_clusters = N every row is its own cluster (labels[v] = v).
 *
 *   children  DEVICE in   [(N-1)*2] int32, as written by slhc_slhc
 *   labels    DEVICE out  [N] int32
 * `children` must be a dendrogram in that layout (merge i joins two nodes with ids below N+i);
 * entries that are not are ignored, and the labels of the rows they would have joined are then
 * unspecified (never an out-of-range access).  Asynchronous on `stream`.
 */
int slhc_flat_clusters_workspace_bytes(int64_t N, size_t* bytes /* HOST out */);
int slhc_flat_clusters(const int32_t* children, int64_t N, int64_t n_clusters, int32_t* labels,
                       void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SLHC_H */
