// Launch interface of the Boruvka forest kernels and the edge sort (forest_kernels.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace slhc {

// Device state of the minimum-spanning-forest construction.  Components are named by the index
// of their root vertex ("colour", paper Sec. 3.2.3); per-component arrays are indexed by it.
struct ForestState {
    int N, k;
    const int32_t* nbr_idx;      // [N, k] ascending by (dist, idx)
    const float* nbr_dist;       // [N, k]
    int32_t* colour;             // [N]
    int32_t* ptr;                // [N] entries before ptr[v] are known to share v's colour
    int32_t* ext_idx;            // [N] last cross-component 1-NN answer of v (-1: none yet)
    float* ext_dist;             // [N]
    float* cand_w;               // [N] weight of v's lightest outgoing edge, or a lower bound
    int32_t* cand_u;             // [N] its other endpoint, or -1 when only the bound is known
    uint32_t* best_w;            // [N] per component: min weight bits over exact candidates
    unsigned long long* best_e;  // [N] per component: min (lo << 32 | hi) among those of best_w
    uint32_t* min_lb;            // [N] per component: min lower-bound bits over unknown vertices
    int32_t* hook;               // [N] per component: component it attaches to this round
    int32_t* qlist;              // [N] rows sent to the cross-component 1-NN
    int32_t* counters;           // [4]: 0 = queries this round, 1 = edges so far, 2 = hook chains not yet
                                 //      followed to their end (cleared by forest_round_reset),
                                 //      3 = site of the first failed index check (0 = none)
    int32_t* e_lo;               // [N-1] committed edges
    int32_t* e_hi;
    float* e_w;
};

hipError_t forest_init(const ForestState& f, hipStream_t s);
hipError_t forest_round_reset(const ForestState& f, hipStream_t s);
hipError_t forest_scan_lists(const ForestState& f, hipStream_t s);
hipError_t forest_classify(const ForestState& f, hipStream_t s);
// qrows[q] is the vertex query q was made for (f.qlist, or a reordered copy of it).  `thresholds`
// (or nullptr): the per-component thresholds the sweep ran under (SweepParams::comp_best); answers
// farther than their component's threshold are kept as lower bounds only.
hipError_t forest_apply_queries(const ForestState& f, const int32_t* qrows, const int32_t* q_idx,
                                const float* q_dist, int nq, const uint32_t* thresholds, hipStream_t s);
// Two-phase connection sweeps (n > 0): rows of `list` in every `stride`-th 128-row panel of the row
// order (inv[v] = position of row v) go to part_a, the others to part_b; counts[0], counts[1] (zeroed by
// the caller) receive the part sizes.  forest_still_needed keeps the rows of `list` that the test of
// forest_classify would still list after best_w has dropped; *count zeroed by the caller.
hipError_t forest_split_queries(const ForestState& f, const int32_t* list, int n, const int32_t* inv, int stride,
                                int32_t* part_a, int32_t* part_b, int32_t* counts, hipStream_t s);
hipError_t forest_still_needed(const ForestState& f, const int32_t* list, int n, int32_t* out, int32_t* count,
                               hipStream_t s);
hipError_t forest_select_edges(const ForestState& f, hipStream_t s);
// sizes[c] += 1 for every entry c of colour[0..n) inside [0, bins); sizes zeroed by the caller.  One atomic
// per colour and wavefront where neighbouring entries share their colour.
hipError_t forest_component_sizes(const int32_t* colour, int n, int bins, int32_t* sizes, hipStream_t s);
hipError_t forest_commit(const ForestState& f, hipStream_t s);
// Every component root follows the hooks up to `steps` components far and hooks itself there; with
// `flag`, counters[2] is set when some root has not reached the end of its chain.
hipError_t forest_jump(const ForestState& f, int steps, bool flag, hipStream_t s);
// colour[v] = hook[colour[v]]; with only_if_converged the kernel does nothing while counters[2] != 0.
hipError_t forest_relabel(const ForestState& f, bool only_if_converged, hipStream_t s);

// CSR input (offsets [V+1], indices [E], weights [E]).  forest_csr_check flags malformed arrays or
// weights that are negative / not finite in f.counters[3]; forest_csr_scan fills cand_w / cand_u with
// every vertex's first outgoing edge in the (w, lo, hi) order and folds the weights into best_w.
hipError_t forest_csr_check(const int32_t* offsets, const int32_t* indices, const float* weights, int V, int E,
                            int32_t* counters, hipStream_t s);
hipError_t forest_csr_scan(const int32_t* offsets, const int32_t* indices, const float* weights, int E,
                           const ForestState& f, hipStream_t s);

// Sort E edges ascending by (w, lo, hi).  keys/vals are scratch of E elements each; `temp` of
// edge_sort_temp_bytes(E).  Result in out_lo/out_hi/out_w.
size_t edge_sort_temp_bytes(int E);
hipError_t edge_sort(const int32_t* lo, const int32_t* hi, const float* w, int E,
                     unsigned long long* keys_a, unsigned long long* keys_b,
                     uint32_t* vals_a, uint32_t* vals_b, void* temp, size_t temp_bytes,
                     int32_t* out_lo, int32_t* out_hi, float* out_w, hipStream_t s);

// Components of the forest made of edges 0..R-1 of a tree's edge list (lo, hi < N): one pass hooks every
// edge's larger root under the smaller and flattens the labels; `first` initialises label[v] = v.  The
// caller clears *changed before a pass and repeats passes until one leaves it 0; label[v] is then the
// smallest vertex id of v's component.  prefix_forest_keys: key[e] = label[lo[e]], val[e] = e for e < R.
hipError_t prefix_forest_pass(const int32_t* lo, const int32_t* hi, int R, int N, int32_t* label, int32_t* changed,
                              bool first, hipStream_t s);
hipError_t prefix_forest_keys(const int32_t* lo, const int32_t* label, int R, int N, uint32_t* key, uint32_t* val,
                              hipStream_t s);

// glo[j] = lo[listed[j]], ghi[j] = hi[listed[j]] for j < R (-1 where listed[j] is not below R), and the way
// back: children[2 listed[j] ..] = cj[2 j ..], sizes[listed[j]] = sj[j].
hipError_t prefix_forest_gather(const int32_t* lo, const int32_t* hi, const uint32_t* listed, int R, int32_t* glo,
                                int32_t* ghi, hipStream_t s);
hipError_t prefix_forest_scatter(const uint32_t* listed, const int32_t* cj, const int32_t* sj, int R, int32_t* children,
                                 int32_t* sizes, hipStream_t s);

// Stable sort of n (key, value) pairs of 32-bit words by key (keys below 2^key_bits).
size_t pair_sort_temp_bytes(int n);
hipError_t pair_sort_u32(const uint32_t* keys_in, uint32_t* keys_out, const uint32_t* vals_in,
                         uint32_t* vals_out, int n, int key_bits, void* temp, size_t temp_bytes,
                         hipStream_t s);

}  // namespace slhc
