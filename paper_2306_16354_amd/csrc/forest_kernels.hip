// Boruvka minimum spanning forest over cached sorted neighbour lists, with colours instead of
// graph contraction (cuSLINK paper Sec. 3.2: Alg. "MST Algorithm", "Minimum incident edges",
// "Label Propagation"), plus the weight sort of Sec. 3.3.1.
//
// Differences from the paper's kernels, all deliberate:
//   * No weight alteration (Sec. 3.2.1).  Ties are broken by the strict order
//     (weight, min endpoint, max endpoint) on undirected edges, which also handles zero weights
//     and exact duplicates, where a random perturbation below the smallest weight gap cannot work.
//     A component's minimum is found in two atomic passes: 32-bit min over weight bits, then
//     64-bit min over (lo, hi) among the edges of that weight.
//   * The lists are the directed k-NN lists, already ascending, so "minimum edge per vertex" is
//     the first entry of another colour: one lane per entry, one ballot, no reduction tree.
//   * A vertex whose whole list shares its colour contributes a lower bound (its k-th distance,
//     or its last cross-component 1-NN distance) instead of an edge; the host commits a
//     component's edge only when it beats every such bound, and queries the rest.  This is what
//     makes the result the minimum spanning tree of the complete graph and not just of the
//     k-NN graph.
//   * Relabelling is pointer doubling over component roots, then one gather per vertex, instead
//     of iterated atomicMin colour exchange (Alg. "min_pair_colors" / "update_colors").
#include <hip/hip_runtime.h>
#include <cstring>
#include <rocprim/rocprim.hpp>
#include <stdint.h>
#include "forest_kernels.h"

namespace slhc {

constexpr uint32_t INF_BITS = 0x7f800000u;
constexpr int TB = 256;

static inline int blocks_for(long long n) { return (int)((n + TB - 1) / TB); }

// Every index that comes out of device memory is range-checked before it is used as an address.
// A failed check records its site in counters[3] (the host turns that into SLHC_INTERNAL) and the
// access is skipped, so corrupt state can never become an out-of-bounds access.
__device__ inline bool in_range(int i, int n) { return (unsigned int)i < (unsigned int)n; }
__device__ inline void report(const ForestState& f, int site) { atomicCAS(&f.counters[3], 0, site); }
// The first failed check of a state error also leaves what it saw in counters[16..23], for the host's message.
__device__ inline void report_with(const ForestState& f, int site, int a, int b, int c, int d, int e, int g)
{
    if (atomicCAS(&f.counters[3], 0, site) == 0) {
        f.counters[16] = site; f.counters[17] = a; f.counters[18] = b; f.counters[19] = c;
        f.counters[20] = d; f.counters[21] = e; f.counters[22] = g;
    }
}

// atomicMin that first looks: the per-component minima only decrease, so a value that does not beat
// what is already there never needs the atomic (a stale, larger value read here only costs an atomic).  In late rounds one component holds most vertices and
// unfiltered atomics on its single word serialise (measured 6 ms per round at N = 1M).
__device__ inline void min_into(uint32_t* slot, uint32_t v)
{
    if (v < *reinterpret_cast<volatile uint32_t*>(slot)) atomicMin(slot, v);
}
__device__ inline void min_into(unsigned long long* slot, unsigned long long v)
{
    if (v < *reinterpret_cast<volatile unsigned long long*>(slot)) atomicMin(slot, v);
}

// Minimum of `v` over the lanes that share a component, one atomic per component and wavefront.  In the
// late rounds most vertices belong to a few large components, and one atomic per vertex on those few
// words serialises (measured: 0.7 ms for one kernel at N = 1M).  The first two distinct colours of the
// wavefront are reduced across lanes; lanes of any further colour fall back to their own atomic, so a
// wavefront of 64 different colours (the first round) costs two short passes, not 64.
__device__ inline void wave_min_into(uint32_t* slots, int c, uint32_t v, bool active)
{
    const int lane = threadIdx.x & 63;
    unsigned long long todo = __ballot(active);
#pragma unroll 1
    for (int pass = 0; pass < 2 && todo; ++pass) {
        const int leader = __builtin_ctzll(todo);
        const int c0 = __shfl(c, leader);
        const bool mine = active && c == c0;
        uint32_t m = mine ? v : 0xffffffffu;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const uint32_t other = (uint32_t)__shfl_xor((int)m, o);
            m = other < m ? other : m;
        }
        if (lane == leader) min_into(&slots[c0], m);
        const unsigned long long served = __ballot(mine);
        todo &= ~served;
        active = active && !mine;
    }
    if (active) min_into(&slots[c], v);
}

// Slot of this thread among the threads of the grid that pass `mine`, behind *counter: one atomic per
// workgroup (per-vertex or per-wavefront atomics on the one counter word serialise: 15 600 of them took
// 0.18 ms at N = 1M).  Every thread of the workgroup must call it.
template <int THREADS>
__device__ inline int block_append(bool mine, int32_t* counter)
{
    __shared__ int wave_count[THREADS / 64];
    __shared__ int wave_base[THREADS / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned long long mask = __ballot(mine);
    if (lane == 0) wave_count[wave] = __popcll(mask);
    __syncthreads();
    if (threadIdx.x == 0) {
        int total = 0;
        for (int w = 0; w < THREADS / 64; ++w) { wave_base[w] = total; total += wave_count[w]; }
        const int base = total > 0 ? atomicAdd(counter, total) : 0;
        for (int w = 0; w < THREADS / 64; ++w) wave_base[w] += base;
    }
    __syncthreads();
    const int pre = __builtin_amdgcn_mbcnt_hi((unsigned int)(mask >> 32), __builtin_amdgcn_mbcnt_lo((unsigned int)mask, 0u));
    return mine ? wave_base[wave] + pre : -1;
}

__global__ void __launch_bounds__(TB) k_forest_init(ForestState f)
{
    const int v = blockIdx.x * TB + threadIdx.x;
    if (v < 4) f.counters[v] = 0;          // before the range test: N may be smaller than 4
    if (v >= f.N) return;
    f.colour[v] = v;
    f.ptr[v] = 0;
    f.ext_idx[v] = -1;
    f.ext_dist[v] = 0.f;
}

__global__ void __launch_bounds__(TB) k_round_reset(ForestState f)
{
    const int v = blockIdx.x * TB + threadIdx.x;
    if (v >= f.N) return;
    f.best_w[v] = INF_BITS;
    f.best_e[v] = ~0ull;
    f.min_lb[v] = INF_BITS;
    // (counters[2], the "hook chains unresolved" flag, is cleared by k_commit: the scan of the next round, and
    // with it this kernel, is enqueued behind the relabelling, before the host has read the flag)
    if (v == 0) f.counters[0] = 0;
}

// G lanes per vertex walk its list from ptr[v] on, G entries at a time, until an entry of another colour
// turns up: the lists are ascending, so that entry is the vertex's lightest listed outgoing edge.  Most
// vertices find it in their first step (in the first round entry 0 always is foreign), and ptr only moves
// forward over the rounds, so the colour gathers summed over all rounds stay near N * (k + G * rounds)
// instead of N * k * rounds with one lane per entry.
template <int G>
__global__ void __launch_bounds__(TB) k_scan_lists(ForestState f)
{
    // the scan for the next round is enqueued before the host knows that the tree is complete
    if (f.counters[1] >= f.N - 1) return;
    const int gid = (int)(((long long)blockIdx.x * TB + threadIdx.x) / G);
    const int j = threadIdx.x & (G - 1);
    const int lane = threadIdx.x & 63;
    const bool live = gid < f.N;
    const int v = live ? gid : 0;
    const int c = f.colour[v];
    int found = -1;
    for (int base = f.ptr[v];; base += G) {
        const bool more = live && base < f.k && found < 0;        // the same for the G lanes of a vertex
        if (!__any(more)) break;
        bool foreign = false;
        const int e = base + j;
        if (more && e < f.k) {
            const int u = f.nbr_idx[(size_t)v * f.k + e];
            if (in_range(u, f.N)) foreign = f.colour[u] != c;
            else report(f, 1);
        }
        unsigned long long mask = __ballot(foreign);
        mask = (mask >> (lane & ~(G - 1))) & ((1ull << G) - 1ull);
        if (more && mask) found = base + __builtin_ctzll(mask);
    }
    const bool head = live && j == 0;
    bool exact = false, bounded = false;
    uint32_t wbits = INF_BITS;
    if (head && !in_range(c, f.N)) report(f, 2);
    else if (head) {
        if (found >= 0) {
            const float w = f.nbr_dist[(size_t)v * f.k + found];
            f.ptr[v] = found;
            f.cand_w[v] = w;
            f.cand_u[v] = f.nbr_idx[(size_t)v * f.k + found];
            wbits = __float_as_uint(w);
            exact = true;
        } else {
            f.ptr[v] = f.k;
            const int eu = f.ext_idx[v];
            const float ed = f.ext_dist[v];
            if (eu >= f.N) report(f, 3);
            else if (eu >= 0 && f.colour[eu] != c) {      // cached answer still leads out of the component
                f.cand_w[v] = ed;
                f.cand_u[v] = eu;
                wbits = __float_as_uint(ed);
                exact = true;
            } else {
                // lower bounds on v's nearest foreign point: its k-th list distance, and whatever the last
                // cross-component query left in ext_dist (an exact answer that has since joined v's
                // component, or the component threshold a truncated search was run under; 0 when never queried)
                float lb = f.nbr_dist[(size_t)v * f.k + f.k - 1];
                if (ed > lb) lb = ed;
                f.cand_w[v] = lb;
                f.cand_u[v] = -1;
                wbits = __float_as_uint(lb);
                bounded = true;
            }
        }
    }
    wave_min_into(f.best_w, c, wbits, exact);
    wave_min_into(f.min_lb, c, wbits, bounded);
}

// Vertices that only know a lower bound and whose bound does not exceed their component's best
// exact weight must be queried (<=, so that weight ties are resolved by the edge order).
constexpr int TB_WIDE = 1024;
__global__ void __launch_bounds__(TB_WIDE) k_classify(ForestState f)
{
    const int v = blockIdx.x * TB_WIDE + threadIdx.x;
    bool need = false;
    if (f.counters[1] >= f.N - 1) return;                // tree complete (workgroup-uniform)
    if (v < f.N && f.cand_u[v] < 0) {
        const int c = f.colour[v];
        if (in_range(c, f.N)) need = __float_as_uint(f.cand_w[v]) <= f.best_w[c];
        else report(f, 4);
    }
    const int slot = block_append<TB_WIDE>(need, &f.counters[0]);
    if (need) {
        if (in_range(slot, f.N)) f.qlist[slot] = v;
        else report(f, 5);
    }
}

// `thresholds` (optional): the queries ran under their component's shared threshold, which started at the
// lightest outgoing edge the lists already knew and which the sweep lowered whenever one of the
// component's queries found a lighter one; thresholds[colour] is its value after the sweep, F.  A query's
// tiles were filtered under values that were never below F, so every candidate at most F away was
// examined: an answer at distance <= F is the query's exact nearest foreign row.  Any other query only
// learns that no foreign row is nearer than F: it keeps no candidate, and F becomes its lower bound for the
// following rounds (components only grow).  F = min(start value, lightest edge from a queried row of the
// component to a foreign row) does not depend on the order in which the panels ran.
__global__ void __launch_bounds__(TB) k_apply_queries(ForestState f, const int32_t* __restrict__ qrows,
                                                      const int32_t* __restrict__ q_idx,
                                                      const float* __restrict__ q_dist, int nq,
                                                      const uint32_t* __restrict__ thresholds)
{
    const int q = blockIdx.x * TB + threadIdx.x;
    bool found = false;
    int c = 0;
    float w = 0.f;
    if (q < nq) {
        const int v = qrows[q];
        const int u = q_idx[q];
        w = q_dist[q];
        if (!in_range(v, f.N) || u < -1 || u >= f.N || !in_range(f.colour[v], f.N)) report(f, 6);
        else {
            c = f.colour[v];
            // an answer inside the query's own component can only come from a broken sweep
            if (u >= 0 && f.colour[u] == c) report_with(f, 14, q, v, u, c, (int)__float_as_uint(w), nq);
            bool exact = true;
            if (thresholds) {
                const uint32_t fb = thresholds[c];
                if (!(u >= 0 && __float_as_uint(w) <= fb)) {
                    const float F = __uint_as_float(fb);
                    const float old = f.ext_dist[v];
                    f.ext_idx[v] = -1;
                    f.ext_dist[v] = F > old ? F : old;
                    f.cand_u[v] = -1;
                    f.cand_w[v] = F;
                    exact = false;
                }
            }
            if (exact) {
                f.ext_idx[v] = u;
                f.ext_dist[v] = w;
                f.cand_u[v] = u;
                f.cand_w[v] = w;
                found = u >= 0;
            }
        }
    }
    wave_min_into(f.best_w, c, __float_as_uint(w), found);
}

// slot of this lane among the lanes of `mask` behind *counter (one atomic per wavefront)
__device__ inline int wave_append(unsigned long long mask, bool mine, int32_t* counter)
{
    if (!mask) return -1;
    const int lane = threadIdx.x & 63;
    const int leader = __builtin_ctzll(mask);
    int base = 0;
    if (lane == leader) base = atomicAdd(counter, __popcll(mask));
    base = __shfl(base, leader);
    const int pre = __builtin_amdgcn_mbcnt_hi((unsigned int)(mask >> 32), __builtin_amdgcn_mbcnt_lo((unsigned int)mask, 0u));
    return mine ? base + pre : -1;
}

// Two-phase connection sweeps.  k_split_queries sends the listed rows whose 128-row panel in the row
// order is a sampled one (every `stride`-th panel) to part A and the others to part B.  After the
// sweep over part A has lowered best_w, k_still_needed keeps of part B only the rows whose bound still
// does not exceed their component's best exact weight (the test of k_classify again).
__global__ void __launch_bounds__(TB) k_split_queries(ForestState f, const int32_t* __restrict__ list, int n,
                                                      const int32_t* __restrict__ inv, int stride,
                                                      int32_t* __restrict__ part_a, int32_t* __restrict__ part_b,
                                                      int32_t* __restrict__ counts)
{
    const int q = blockIdx.x * TB + threadIdx.x;
    int v = -1;
    if (q < n) {
        v = list[q];
        if (!in_range(v, f.N)) { report(f, 10); v = -1; }
    }
    const bool sampled = v >= 0 && ((inv[v] >> 7) % stride) == 0;
    const bool other = v >= 0 && !sampled;
    const int slot_a = wave_append(__ballot(sampled), sampled, &counts[0]);
    const int slot_b = wave_append(__ballot(other), other, &counts[1]);
    if (sampled) { if (in_range(slot_a, f.N)) part_a[slot_a] = v; else report(f, 10); }
    if (other) { if (in_range(slot_b, f.N)) part_b[slot_b] = v; else report(f, 10); }
}

__global__ void __launch_bounds__(TB) k_still_needed(ForestState f, const int32_t* __restrict__ list, int n,
                                                     int32_t* __restrict__ out, int32_t* __restrict__ count)
{
    const int q = blockIdx.x * TB + threadIdx.x;
    bool keep = false;
    int v = -1;
    if (q < n) {
        v = list[q];
        if (!in_range(v, f.N) || !in_range(f.colour[v], f.N)) report(f, 11);
        else keep = __float_as_uint(f.cand_w[v]) <= f.best_w[f.colour[v]];
    }
    const int slot = wave_append(__ballot(keep), keep, count);
    if (keep) { if (in_range(slot, f.N)) out[slot] = v; else report(f, 11); }
}

__global__ void __launch_bounds__(TB) k_select_edges(ForestState f)
{
    const int v = blockIdx.x * TB + threadIdx.x;
    if (v >= f.N) return;
    const int u = f.cand_u[v];
    if (u < 0) return;
    const int c = f.colour[v];
    if (u >= f.N || !in_range(c, f.N)) { report(f, 7); return; }
    if (__float_as_uint(f.cand_w[v]) != f.best_w[c]) return;
    const unsigned int lo = (unsigned int)(v < u ? v : u), hi = (unsigned int)(v < u ? u : v);
    min_into(&f.best_e[c], ((unsigned long long)lo << 32) | hi);
}

// One thread per component root: append the component's edge (once per undirected edge) and
// record which component it attaches to.  Two components that chose the same edge keep the
// smaller root.
constexpr int COMMIT_ITEMS = 8;        // vertices per thread: one atomic on the edge counter per 8192 vertices
__global__ void __launch_bounds__(TB_WIDE) k_commit(ForestState f)
{
    __shared__ int wave_count[TB_WIDE / 64];
    __shared__ int wave_base[TB_WIDE / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (blockIdx.x == 0 && threadIdx.x == 0) f.counters[2] = 0;     // set again by k_jump if a hook chain stays unresolved
    int lo[COMMIT_ITEMS], hi[COMMIT_ITEMS];
    uint32_t wbits[COMMIT_ITEMS];
    unsigned int adds = 0;             // bit i: vertex i of this thread appends its component's edge
#pragma unroll
    for (int i = 0; i < COMMIT_ITEMS; ++i) {
        const long long vv = ((long long)blockIdx.x * COMMIT_ITEMS + i) * TB_WIDE + threadIdx.x;
        lo[i] = hi[i] = 0;
        wbits[i] = INF_BITS;
        if (vv >= f.N) continue;
        const int v = (int)vv;
        if (f.colour[v] != v) continue;
        const uint32_t wb = f.best_w[v];
        int hook = v;
        if (wb != INF_BITS) {
            const unsigned long long e = f.best_e[v];
            const int elo = (int)(e >> 32), ehi = (int)(e & 0xffffffffull);
            if (!in_range(elo, f.N) || !in_range(ehi, f.N)) report(f, 8);
            else {
                const int clo = f.colour[elo], chi = f.colour[ehi];
                const int other = (clo == v) ? chi : clo;
                if (!in_range(other, f.N) || other == v || (clo != v && chi != v))
                    report_with(f, 9, v, elo, ehi, clo, chi, (int)wb);
                else {
                    const bool mutual = (f.best_w[other] == wb) && (f.best_e[other] == e);
                    if (!mutual || v < other) { adds |= 1u << i; lo[i] = elo; hi[i] = ehi; wbits[i] = wb; }
                    hook = (mutual && v < other) ? v : other;
                }
            }
        }
        f.hook[v] = hook;
    }
    // exclusive prefix of the per-thread counts over the workgroup
    const int mine = __popc(adds);
    int incl = mine;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int up = __shfl_up(incl, o);
        if (lane >= o) incl += up;
    }
    if (lane == 63) wave_count[wave] = incl;
    __syncthreads();
    if (threadIdx.x == 0) {
        int total = 0;
        for (int w = 0; w < TB_WIDE / 64; ++w) { wave_base[w] = total; total += wave_count[w]; }
        const int base = total > 0 ? atomicAdd(&f.counters[1], total) : 0;
        for (int w = 0; w < TB_WIDE / 64; ++w) wave_base[w] += base;
    }
    __syncthreads();
    int slot = wave_base[wave] + incl - mine;
#pragma unroll
    for (int i = 0; i < COMMIT_ITEMS; ++i) {
        if (!(adds & (1u << i))) continue;
        if (slot < f.N - 1) {
            f.e_lo[slot] = lo[i];
            f.e_hi[slot] = hi[i];
            f.e_w[slot] = __uint_as_float(wbits[i]);
        }
        ++slot;
    }
}

// Every root follows the hooks up to `steps` components far and hooks itself to where it got; other
// roots do the same at the same time, which is harmless: whatever a hook is replaced by is an ancestor
// of what it held.  With `flag` a root that has not reached the end of its chain sets counters[2].
// Two launches of 32 steps resolve chains of up to 1024 hooks; the host loops only beyond that.
__global__ void __launch_bounds__(TB) k_jump(ForestState f, int steps, int flag)
{
    const int v = blockIdx.x * TB + threadIdx.x;
    if (v >= f.N || f.colour[v] != v) return;
    int h = f.hook[v];
    if (!in_range(h, f.N)) { report(f, 10); return; }
    bool at_root = false;
    for (int i = 0; i < steps; ++i) {
        const int hh = *reinterpret_cast<volatile int32_t*>(&f.hook[h]);
        if (!in_range(hh, f.N)) { report(f, 11); return; }
        if (hh == h) { at_root = true; break; }
        h = hh;
    }
    f.hook[v] = h;
    if (flag && !at_root) {
        const int hh = *reinterpret_cast<volatile int32_t*>(&f.hook[h]);
        if (hh != h) atomicOr(&f.counters[2], 1);
    }
}

// With `only_if_converged` the kernel does nothing while counters[2] says that some hook chain has not
// been followed to its end (the host then finishes the chains and launches it again).
__global__ void __launch_bounds__(TB) k_relabel(ForestState f, int only_if_converged)
{
    const int v = blockIdx.x * TB + threadIdx.x;
    if (v >= f.N) return;
    if (only_if_converged && f.counters[2] != 0) return;
    const int c = f.colour[v];
    if (!in_range(c, f.N)) { report(f, 12); return; }
    const int r = f.hook[c];
    if (!in_range(r, f.N)) { report(f, 13); return; }
    f.colour[v] = r;
}

// Rows per component: sizes[c] += 1 for every row of colour c (entries outside [0, bins) are skipped;
// sizes zeroed by the caller).  Meant for colours in a spatially coherent row order, where the lanes of a
// wavefront share one or two colours: those are counted with one atomic each.
__global__ void __launch_bounds__(TB) k_component_sizes(const int32_t* __restrict__ colour, int n, int bins,
                                                        int32_t* __restrict__ sizes)
{
    const int i = blockIdx.x * TB + threadIdx.x;
    const int lane = threadIdx.x & 63;
    const int c = i < n ? colour[i] : -1;
    bool active = (unsigned int)c < (unsigned int)bins;
    unsigned long long todo = __ballot(active);
#pragma unroll 1
    for (int pass = 0; pass < 4 && todo; ++pass) {
        const int leader = __builtin_ctzll(todo);
        const int c0 = __shfl(c, leader);
        const bool mine = active && c == c0;
        const unsigned long long served = __ballot(mine);
        if (lane == leader) atomicAdd(&sizes[c0], __popcll(served));
        todo &= ~served;
        active = active && !mine;
    }
    if (active) atomicAdd(&sizes[c], 1);
}

// ------------------------------------------------------------------------------- CSR graphs
// Sec. 3.2 takes the graph in CSR form.  Input check: offsets monotone from 0 to E, indices in
// range, weights finite and non-negative (the edge order compares weight bit patterns).  A failed
// check records its site in counters[3].
__global__ void __launch_bounds__(TB) k_csr_check(const int32_t* __restrict__ offsets,
                                                  const int32_t* __restrict__ indices,
                                                  const float* __restrict__ weights, int V, int E,
                                                  int32_t* __restrict__ counters)
{
    const long long i = (long long)blockIdx.x * TB + threadIdx.x;
    if (i < V) {
        const int o0 = offsets[i], o1 = offsets[i + 1];
        if (o0 < 0 || o1 < o0 || o1 > E) atomicCAS(&counters[3], 0, 20);
        if (i == 0 && o0 != 0) atomicCAS(&counters[3], 0, 21);
        if (i == V - 1 && o1 != E) atomicCAS(&counters[3], 0, 22);
    }
    if (i < E) {
        if (!in_range(indices[i], V)) atomicCAS(&counters[3], 0, 23);
        const float w = weights[i];
        if (!(w >= 0.f) || w == __builtin_inff()) atomicCAS(&counters[3], 0, 24);
    }
}

// Minimum outgoing edge of every vertex (Sec. 3.2.2 "Minimum Edge Per Vertex"): one thread scans
// the vertex's row for the edge to another colour that is first in the order (w, lo, hi).  The
// paper gives a warp to each vertex; road-like graphs have 2-3 edges per vertex, where a 64-wide
// wavefront per vertex would idle, so a thread per vertex is used (a row with thousands of edges
// is then scanned by one thread: correct, slow).
__global__ void __launch_bounds__(TB) k_csr_scan(const int32_t* __restrict__ offsets,
                                                 const int32_t* __restrict__ indices,
                                                 const float* __restrict__ weights, int E, ForestState f)
{
    const int v = blockIdx.x * TB + threadIdx.x;
    if (v >= f.N) return;
    // f.ptr[v] != 0: an earlier round found every neighbour of v in v's own component.  Components only
    // grow, so v never has an outgoing edge again; its cand_u stays -1 and its row is not read any more
    // (after a few rounds that is most vertices).
    if (f.ptr[v] != 0) return;
    const int c = f.colour[v];
    if (!in_range(c, f.N)) { report(f, 25); return; }
    int o0 = offsets[v], o1 = offsets[v + 1];
    o0 = o0 < 0 ? 0 : o0;
    o1 = o1 > E ? E : o1;
    uint32_t bw = INF_BITS;
    unsigned int blo = ~0u, bhi = ~0u;
    int bu = -1;
    for (int e = o0; e < o1; ++e) {
        const int u = indices[e];
        if (!in_range(u, f.N) || f.colour[u] == c) continue;      // also drops self loops
        const uint32_t wb = __float_as_uint(weights[e]);
        const unsigned int lo = (unsigned int)(v < u ? v : u), hi = (unsigned int)(v < u ? u : v);
        if (wb < bw || (wb == bw && (lo < blo || (lo == blo && hi < bhi)))) { bw = wb; blo = lo; bhi = hi; bu = u; }
    }
    f.cand_u[v] = bu;
    f.cand_w[v] = __uint_as_float(bw);
    if (bu >= 0) min_into(&f.best_w[c], bw);
    else f.ptr[v] = 1;
}

#define LAUNCH1(kern, n, s, ...)                                                       \
    do {                                                                               \
        hipLaunchKernelGGL(kern, dim3(blocks_for(n)), dim3(TB), 0, s, __VA_ARGS__);    \
        return hipGetLastError();                                                      \
    } while (0)

hipError_t forest_init(const ForestState& f, hipStream_t s) { LAUNCH1(k_forest_init, f.N, s, f); }
hipError_t forest_round_reset(const ForestState& f, hipStream_t s) { LAUNCH1(k_round_reset, f.N, s, f); }

hipError_t forest_scan_lists(const ForestState& f, hipStream_t s)
{
    if (f.k <= 2) LAUNCH1(k_scan_lists<2>, (long long)f.N * 2, s, f);
    LAUNCH1(k_scan_lists<4>, (long long)f.N * 4, s, f);
}

hipError_t forest_classify(const ForestState& f, hipStream_t s)
{
    hipLaunchKernelGGL(k_classify, dim3((f.N + TB_WIDE - 1) / TB_WIDE), dim3(TB_WIDE), 0, s, f);
    return hipGetLastError();
}

hipError_t forest_apply_queries(const ForestState& f, const int32_t* qrows, const int32_t* q_idx,
                                const float* q_dist, int nq, const uint32_t* thresholds, hipStream_t s)
{
    LAUNCH1(k_apply_queries, nq, s, f, qrows, q_idx, q_dist, nq, thresholds);
}

hipError_t forest_split_queries(const ForestState& f, const int32_t* list, int n, const int32_t* inv, int stride,
                                int32_t* part_a, int32_t* part_b, int32_t* counts, hipStream_t s)
{
    LAUNCH1(k_split_queries, n, s, f, list, n, inv, stride, part_a, part_b, counts);
}

hipError_t forest_still_needed(const ForestState& f, const int32_t* list, int n, int32_t* out, int32_t* count,
                               hipStream_t s)
{
    LAUNCH1(k_still_needed, n, s, f, list, n, out, count);
}

hipError_t forest_select_edges(const ForestState& f, hipStream_t s) { LAUNCH1(k_select_edges, f.N, s, f); }
hipError_t forest_component_sizes(const int32_t* colour, int n, int bins, int32_t* sizes, hipStream_t s)
{
    LAUNCH1(k_component_sizes, n, s, colour, n, bins, sizes);
}
hipError_t forest_commit(const ForestState& f, hipStream_t s)
{
    const int per_block = TB_WIDE * COMMIT_ITEMS;
    hipLaunchKernelGGL(k_commit, dim3((f.N + per_block - 1) / per_block), dim3(TB_WIDE), 0, s, f);
    return hipGetLastError();
}
hipError_t forest_jump(const ForestState& f, int steps, bool flag, hipStream_t s) { LAUNCH1(k_jump, f.N, s, f, steps, flag ? 1 : 0); }
hipError_t forest_relabel(const ForestState& f, bool only_if_converged, hipStream_t s) { LAUNCH1(k_relabel, f.N, s, f, only_if_converged ? 1 : 0); }

hipError_t forest_csr_check(const int32_t* offsets, const int32_t* indices, const float* weights, int V, int E,
                            int32_t* counters, hipStream_t s)
{
    LAUNCH1(k_csr_check, (V > E ? V : E), s, offsets, indices, weights, V, E, counters);
}

hipError_t forest_csr_scan(const int32_t* offsets, const int32_t* indices, const float* weights, int E,
                           const ForestState& f, hipStream_t s)
{
    LAUNCH1(k_csr_scan, f.N, s, offsets, indices, weights, E, f);
}

// ------------------------------------------------------------------------------- edge sort
__global__ void __launch_bounds__(TB) k_pack_edges(const int32_t* __restrict__ lo,
                                                   const int32_t* __restrict__ hi,
                                                   const float* __restrict__ w, int E,
                                                   unsigned long long* __restrict__ keys,
                                                   uint32_t* __restrict__ vals)
{
    const int i = blockIdx.x * TB + threadIdx.x;
    if (i >= E) return;
    keys[i] = ((unsigned long long)(unsigned int)lo[i] << 32) | (unsigned int)hi[i];
    vals[i] = __float_as_uint(w[i]);
}

__global__ void __launch_bounds__(TB) k_unpack_edges(const unsigned long long* __restrict__ ends,
                                                     const uint32_t* __restrict__ wbits, int E,
                                                     int32_t* __restrict__ lo, int32_t* __restrict__ hi,
                                                     float* __restrict__ w)
{
    const int i = blockIdx.x * TB + threadIdx.x;
    if (i >= E) return;
    lo[i] = (int32_t)(ends[i] >> 32);
    hi[i] = (int32_t)(ends[i] & 0xffffffffull);
    w[i] = __uint_as_float(wbits[i]);
}

// ---- components of the forest made of the first R edges of a weight-sorted tree (for the dendrogram) ----
// label[v] ends as the smallest vertex id of v's component.  Labels only ever decrease and label[x] <= x,
// so every chain of labels descends strictly and every walk below ends.
__global__ void __launch_bounds__(256) k_prefix_init(int32_t* __restrict__ label, int N)
{
    const int v = blockIdx.x * 256 + threadIdx.x;
    if (v < N) label[v] = v;
}

__device__ __forceinline__ int prefix_root(const int32_t* label, int v)
{
    for (;;) {
        const int up = __hip_atomic_load(label + v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (up == v) return v;
        v = up;
    }
}

// every edge hooks the larger of its two roots under the smaller one; *changed is set when any edge still
// joined two different roots (the hook may lose against a smaller one: the next pass sees to it)
__global__ void __launch_bounds__(256) k_prefix_hook(const int32_t* __restrict__ lo, const int32_t* __restrict__ hi,
                                                     int R, int N, int32_t* __restrict__ label,
                                                     int32_t* __restrict__ changed)
{
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= R) return;
    const int a = lo[e], b = hi[e];
    if ((unsigned int)a >= (unsigned int)N || (unsigned int)b >= (unsigned int)N) return;
    const int ra = prefix_root(label, a), rb = prefix_root(label, b);
    if (ra == rb) return;
    atomicMin(label + (ra > rb ? ra : rb), ra > rb ? rb : ra);
    *changed = 1;
}

__global__ void __launch_bounds__(256) k_prefix_flatten(int32_t* __restrict__ label, int N)
{
    const int v = blockIdx.x * 256 + threadIdx.x;
    if (v < N) label[v] = prefix_root(label, v);
}

// key[e] = label of edge e's component, val[e] = e
__global__ void __launch_bounds__(256) k_prefix_keys(const int32_t* __restrict__ lo, const int32_t* __restrict__ label,
                                                     int R, int N, uint32_t* __restrict__ key, uint32_t* __restrict__ val)
{
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= R) return;
    const int a = lo[e];
    key[e] = (unsigned int)a < (unsigned int)N ? (uint32_t)label[a] : 0u;
    val[e] = (uint32_t)e;
}

// end points of the grouped edges in list order
__global__ void __launch_bounds__(256) k_prefix_gather(const int32_t* __restrict__ lo, const int32_t* __restrict__ hi,
                                                       const uint32_t* __restrict__ listed, int R,
                                                       int32_t* __restrict__ glo, int32_t* __restrict__ ghi)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= R) return;
    const uint32_t e = listed[j];
    const bool ok = e < (uint32_t)R;
    glo[j] = ok ? lo[e] : -1;
    ghi[j] = ok ? hi[e] : -1;
}

// children / sizes computed in list order back to edge order
__global__ void __launch_bounds__(256) k_prefix_scatter(const uint32_t* __restrict__ listed, const int32_t* __restrict__ cj,
                                                        const int32_t* __restrict__ sj, int R,
                                                        int32_t* __restrict__ children, int32_t* __restrict__ sizes)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= R) return;
    const uint32_t e = listed[j];
    if (e >= (uint32_t)R) return;
    children[2 * (size_t)e] = cj[2 * (size_t)j];
    children[2 * (size_t)e + 1] = cj[2 * (size_t)j + 1];
    sizes[e] = sj[j];
}

hipError_t prefix_forest_gather(const int32_t* lo, const int32_t* hi, const uint32_t* listed, int R, int32_t* glo,
                                int32_t* ghi, hipStream_t s)
{
    hipLaunchKernelGGL(k_prefix_gather, dim3((R + 255) / 256), dim3(256), 0, s, lo, hi, listed, R, glo, ghi);
    return hipGetLastError();
}

hipError_t prefix_forest_scatter(const uint32_t* listed, const int32_t* cj, const int32_t* sj, int R, int32_t* children,
                                 int32_t* sizes, hipStream_t s)
{
    hipLaunchKernelGGL(k_prefix_scatter, dim3((R + 255) / 256), dim3(256), 0, s, listed, cj, sj, R, children, sizes);
    return hipGetLastError();
}

hipError_t prefix_forest_pass(const int32_t* lo, const int32_t* hi, int R, int N, int32_t* label, int32_t* changed,
                              bool first, hipStream_t s)
{
    if (first) hipLaunchKernelGGL(k_prefix_init, dim3((N + 255) / 256), dim3(256), 0, s, label, N);
    hipLaunchKernelGGL(k_prefix_hook, dim3((R + 255) / 256), dim3(256), 0, s, lo, hi, R, N, label, changed);
    hipLaunchKernelGGL(k_prefix_flatten, dim3((N + 255) / 256), dim3(256), 0, s, label, N);
    return hipGetLastError();
}

hipError_t prefix_forest_keys(const int32_t* lo, const int32_t* label, int R, int N, uint32_t* key, uint32_t* val,
                              hipStream_t s)
{
    hipLaunchKernelGGL(k_prefix_keys, dim3((R + 255) / 256), dim3(256), 0, s, lo, label, R, N, key, val);
    return hipGetLastError();
}

size_t edge_sort_temp_bytes(int E)
{
    size_t a = 0, b = 0;
    unsigned long long* k64 = nullptr;
    uint32_t* k32 = nullptr;
    (void)rocprim::radix_sort_pairs(nullptr, a, k64, k64, k32, k32, (size_t)E, 0, 64, (hipStream_t)0);
    (void)rocprim::radix_sort_pairs(nullptr, b, k32, k32, k64, k64, (size_t)E, 0, 32, (hipStream_t)0);
    return ((a > b ? a : b) + 255) & ~(size_t)255;
}

// Two stable least-significant-digit passes: by (lo, hi), then by the weight bits (non-negative
// floats order like their bit patterns).
hipError_t edge_sort(const int32_t* lo, const int32_t* hi, const float* w, int E,
                     unsigned long long* keys_a, unsigned long long* keys_b,
                     uint32_t* vals_a, uint32_t* vals_b, void* temp, size_t temp_bytes,
                     int32_t* out_lo, int32_t* out_hi, float* out_w, hipStream_t s)
{
    hipLaunchKernelGGL(k_pack_edges, dim3(blocks_for(E)), dim3(TB), 0, s, lo, hi, w, E, keys_a, vals_a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    size_t tb = temp_bytes;
    e = rocprim::radix_sort_pairs(temp, tb, keys_a, keys_b, vals_a, vals_b, (size_t)E, 0, 64, s);
    if (e != hipSuccess) return e;
    tb = temp_bytes;
    e = rocprim::radix_sort_pairs(temp, tb, vals_b, vals_a, keys_b, keys_a, (size_t)E, 0, 32, s);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_unpack_edges, dim3(blocks_for(E)), dim3(TB), 0, s, keys_a, vals_a, E, out_lo, out_hi, out_w);
    return hipGetLastError();
}

size_t pair_sort_temp_bytes(int n)
{
    size_t a = 0;
    uint32_t* k32 = nullptr;
    (void)rocprim::radix_sort_pairs(nullptr, a, k32, k32, k32, k32, (size_t)n, 0, 32, (hipStream_t)0);
    return (a + 255) & ~(size_t)255;
}

hipError_t pair_sort_u32(const uint32_t* keys_in, uint32_t* keys_out, const uint32_t* vals_in,
                         uint32_t* vals_out, int n, int key_bits, void* temp, size_t temp_bytes,
                         hipStream_t s)
{
    size_t tb = temp_bytes;
    if (key_bits < 1) key_bits = 1;
    if (key_bits > 32) key_bits = 32;
    return rocprim::radix_sort_pairs(temp, tb, keys_in, keys_out, vals_in, vals_out, (size_t)n, 0,
                                     (unsigned int)key_bits, s);
}

}  // namespace slhc
