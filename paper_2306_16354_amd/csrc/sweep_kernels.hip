// Fused distance + selection sweeps for gfx950 (MI355X).
//
// The two nearest-neighbour primitives of the cuSLINK paper share one tile/filter/select design:
//   - fused k-NN      (Sec. 3.1.1, Alg. "Fused k-NN"; epilogues of Appendix A)
//   - fused 1-NN restricted to points of another colour (Sec. 3.1.2, Alg. "Fused 1-NN")
// in two kernels: sweep_kernel streams query and candidate chunks through LDS (any d), and
// sweep_kernel_qreg keeps the query fragments in registers (d <= 128, d % 4 == 0) and can skip
// candidate tiles that provably hold nothing of use (tile pruning, not in the paper).
//
// Structure (our own design for 64-wide wavefronts, not the paper's CUDA tiling):
//   * a workgroup (4 wavefronts) owns a panel of 128 query rows and sweeps all N candidate rows
//     in tiles of 128; workgroups are persistent and all sweep the candidates in the same order,
//     but they drift out of step, so most of a panel's candidate stream misses the XCD's L2
//     (measured at 1M x 128: 10-17 % hits, 3.5-4.4 TB through the fabric per launch).  With
//     float32 products that stream runs at a fifth of the HBM peak behind the MFMA work; with
//     split bfloat16 products (below) the multiplies of a chunk are six times shorter than a
//     load takes, and the sweep waits for its loads.  Launches of many panels go range by range
//     (SweepParams::carry_ws): all workgroups sweep the same 32 MiB of candidates at a time, which
//     the memory-side cache then serves, and a panel's lists travel from range to range;
//   * the tile x_c . x_q is accumulated with v_mfma_f32_32x32x2_f32, or, with whole chunks of 32 columns,
//     from split bfloat16 halves as hi_c hi_q + hi_c lo_q + lo_c hi_q with
//     v_mfma_f32_32x32x16_bf16 (16 times the rate; the filter's slack covers the dropped terms, and
//     only the filter sees these products).  Candidates are the A
//     operand and queries the B operand, so a lane's 16 accumulators of a 32x32 block belong to
//     ONE query: the query's threshold is a per-lane scalar;
//   * the accumulator starts at -h_c with h = (1-c)/2 * ||x||^2, so after the K loop it holds
//     x_c.x_q - h_c and the filter "expanded distance <= threshold (+ rounding slack)" is the
//     single compare  acc >= h_q - threshold/2;
//   * pairs that pass are stream-compacted into a per-wavefront LDS queue (the paper's
//     compaction step, Sec. 3.1.1), re-evaluated exactly as sum_t (x_qt - x_ct)^2 by 8-lane
//     groups, and inserted into the query's sorted list in LDS (one list entry per lane).
//   Each wavefront owns its 32 queries outright (lists, thresholds, queue), so selection needs
//   no synchronisation between wavefronts and no mutex in global memory (the paper's
//   multi-block row epilogue, Appendix A, is not needed).
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "sweep_kernels.h"

namespace slhc {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

#ifndef SLHC_SPLIT_MIN_CHUNKS
#define SLHC_SPLIT_MIN_CHUNKS 1   // every-tile sweeps: split bfloat16 products from this many chunks of 32 columns on
#endif
#ifndef SLHC_SPLIT_MIN_CHUNKS_PRUNED
#define SLHC_SPLIT_MIN_CHUNKS_PRUNED 1   // pruned sweeps: likewise, when the caller passes the split copy (at 32 features it does so only for
                                         // data with a large common offset: there the wider filter costs more than the multiplies save)
#endif
#ifndef SLHC_STREAM_SPLIT_MIN_D
#define SLHC_STREAM_SPLIT_MIN_D 0   // the streaming kernel multiplies the split copy, where there is one, from this many features on
#endif
#ifndef SLHC_SEGMENT_HANDICAP
#define SLHC_SEGMENT_HANDICAP 1.18   // see sweep_segments_for
#endif
#ifndef SLHC_SCAN_AHEAD_1NN
#define SLHC_SCAN_AHEAD_1NN 4   // the same in the connection sweeps (8 and 16 measured: no gain at 2M x 32, 1-5 % slower at 1M x 128)
#endif
#ifndef SLHC_SCAN_AHEAD
#define SLHC_SCAN_AHEAD 4      // groups of 64 scan positions whose lower bounds a pruned sweep reads at once (see next_scan)
#endif
#ifndef SLHC_SPLIT_FRAGS
#define SLHC_SPLIT_FRAGS 2      // 2: the LDS reads of a whole chunk go ahead of its multiplies; 1: those of half a chunk
#endif

constexpr int WG_THREADS = 256;
constexpr int BM = 128;            // query rows per workgroup (32 per wavefront)
constexpr int BN = 128;            // candidate rows per tile
constexpr int KC = 32;             // feature columns staged per step
constexpr int LDK = KC + 4;        // LDS row stride in floats (pad: conflict-free b128 reads)
constexpr int QCAP = 1024;         // queue entries per wavefront (one 32x32 block can fill it)
constexpr unsigned long long LIST_SENTINEL = 0x7f8000007fffffffull;   // (+inf, INT_MAX)

__host__ __device__ inline size_t sweep_lds_bytes(int KL)
{
    return (size_t)(BM * LDK + BN * LDK + 2 * BN /*hc*/ + 2 * BN /*ccol*/ + BM /*bounds*/ + BM /*qid*/ +
                    BM /*hq*/ + 8 /*wmax*/ + 8 /*next panel*/) * 4 + (size_t)BM * KL * 8 + (size_t)4 * QCAP * 2;
}

// Rows are read through pointers in the global address space: the re-evaluation runs in functions that
// are real calls, where a plain pointer has lost its address space and every load would be a flat one.
typedef const __attribute__((address_space(1))) float* global_floats;
typedef const __attribute__((address_space(1))) int32_t* global_ints;

// Features t .. t+3 of a row as one vector; features at or beyond d read as 0.  The address is clamped rather
// than the load skipped, so that the loads of one round of group8_sqdist can all be in flight together.
template <bool VEC4>
__device__ inline v4f load_quad(global_floats row, int t, int d)
{
    v4f v;
    if (VEC4) {
        const bool live = t < d;
        const v4f w = *reinterpret_cast<const __attribute__((address_space(1))) v4f*>(row + (live ? t : 0));
        v = live ? w : v4f{0.f, 0.f, 0.f, 0.f};
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const bool live = t + e < d;
            const float w = row[live ? t + e : 0];
            v[e] = live ? w : 0.f;
        }
    }
    return v;
}

__device__ inline float quad_sqdist(v4f va, v4f vb, float s)
{
    float e;
    e = va[0] - vb[0]; s = __builtin_fmaf(e, e, s);
    e = va[1] - vb[1]; s = __builtin_fmaf(e, e, s);
    e = va[2] - vb[2]; s = __builtin_fmaf(e, e, s);
    e = va[3] - vb[3]; s = __builtin_fmaf(e, e, s);
    return s;
}

// sum_t (a_t - b_t)^2 over d features by a group of 8 adjacent lanes; every lane of the group returns
// the total.  The features are cut into 64-wide slabs; lane g adds features 4g..4g+3 of every slab
// into one accumulator and features 4(g+8)..4(g+8)+3 into a second one, in ascending t with fused
// multiply-adds; each set of eight partial sums goes through an xor butterfly (1, 2, 4) and the two
// totals are added last.  (a-b)^2 == (b-a)^2 exactly, so the result is symmetric in its arguments
// bit for bit, and every code path that re-evaluates a pair uses this one order of additions.
// (A feature beyond d contributes fma(0, 0, s) = s, so padding the last slab changes no bit.)
// Two slabs are read per round, eight vector loads in flight at once: one memory round trip per 128
// features.  Read one slab at a time, each waiting for its own data, a pair of 128-feature rows cost four
// round trips in a row, and the rare path of every sweep was mostly that wait.
template <bool VEC4>
__device__ inline float group8_sqdist(const float* __restrict__ a_, const float* __restrict__ b_,
                                      int d, int g, bool active)
{
    const global_floats a = (global_floats)a_;
    const global_floats b = (global_floats)b_;
    float s0 = 0.f, s1 = 0.f;
    if (active) {
        for (int base = 0; base < d; base += 128) {
            const int t0 = base + 4 * g;
            const v4f a00 = load_quad<VEC4>(a, t0, d), b00 = load_quad<VEC4>(b, t0, d);
            const v4f a10 = load_quad<VEC4>(a, t0 + 32, d), b10 = load_quad<VEC4>(b, t0 + 32, d);
            const v4f a01 = load_quad<VEC4>(a, t0 + 64, d), b01 = load_quad<VEC4>(b, t0 + 64, d);
            const v4f a11 = load_quad<VEC4>(a, t0 + 96, d), b11 = load_quad<VEC4>(b, t0 + 96, d);
            s0 = quad_sqdist(a00, b00, s0);
            s0 = quad_sqdist(a01, b01, s0);
            s1 = quad_sqdist(a10, b10, s1);
            s1 = quad_sqdist(a11, b11, s1);
        }
    }
    s0 += __shfl_xor(s0, 1);
    s0 += __shfl_xor(s0, 2);
    s0 += __shfl_xor(s0, 4);
    s1 += __shfl_xor(s1, 1);
    s1 += __shfl_xor(s1, 2);
    s1 += __shfl_xor(s1, 4);
    return s0 + s1;
}

// h_i = (1-c)/2 * ||x_i||^2 ; one 16-lane group per row.
// A row whose squared norm is not a finite float32 (NaN or infinity among its values, or overflow) sets
// *nonfinite (optional) to 1.
// `shift` (optional, [d], 16-byte aligned with VEC4): the norms are those of the rows fl(x - shift), the rows the
// split copy holds (see split_bf16_kernel); with `shift_tile` a matrix of shifts, one row of it per tile of 128 rows.
template <bool VEC4>
__global__ void __launch_bounds__(256) half_norm_kernel(const float* __restrict__ X, int N, int d,
                                                        float scale, float* __restrict__ hn,
                                                        unsigned int* __restrict__ nonfinite,
                                                        const float* __restrict__ shift_,
                                                        const int* __restrict__ shift_tile)
{
    const int lane16 = threadIdx.x & 15;
    const long long row = ((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 4;
    const bool active = row < N;
    float s = 0.f;
    if (active) {
        const float* x = X + (size_t)row * d;
        // (shift_tile: the rows of tile t = row / 128 take row shift_tile[t] of the matrix `shift`)
        const float* shift = (shift_ && shift_tile) ? shift_ + (size_t)shift_tile[row >> 7] * d : shift_;
        if (VEC4) {
            for (int t = 4 * lane16; t < d; t += 64) {
                v4f v = *reinterpret_cast<const v4f*>(x + t);
                if (shift) v -= *reinterpret_cast<const v4f*>(shift + t);
                s = __builtin_fmaf(v[0], v[0], s);
                s = __builtin_fmaf(v[1], v[1], s);
                s = __builtin_fmaf(v[2], v[2], s);
                s = __builtin_fmaf(v[3], v[3], s);
            }
        } else {
            for (int t0 = 4 * lane16; t0 < d; t0 += 64) {
                const int te = (t0 + 4 < d) ? t0 + 4 : d;
                for (int t = t0; t < te; ++t) {
                    const float v = shift ? x[t] - shift[t] : x[t];
                    s = __builtin_fmaf(v, v, s);
                }
            }
        }
    }
    s += __shfl_xor(s, 1);
    s += __shfl_xor(s, 2);
    s += __shfl_xor(s, 4);
    s += __shfl_xor(s, 8);
    if (active && lane16 == 0) {
        hn[row] = scale * s;
        if (nonfinite && !(s < __builtin_inff())) atomicOr(nonfinite, 1u);      // NaN fails the compare too
    }
}

// A value that is the same in all lanes, as the compiler can see it: queue lengths come back from real calls in
// vector registers, and a counter fed from them would live in a vector register (in practice in scratch memory,
// read and written once per visit of the rare path) instead of a scalar one.
__device__ inline int wave_uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

__device__ inline unsigned long long make_key(float dist, int idx)
{
    return ((unsigned long long)__float_as_uint(dist) << 32) | (unsigned int)idx;
}

// LDS layout of a sweep workgroup (dynamic shared memory).
template <int KL>
struct SweepLds {
    float* Qs; float* Cs; float* hcs; int* ccol; float* bounds; int* qid; float* hqs; float* wmax;
    unsigned long long* lists; unsigned short* queues;
    __device__ explicit SweepLds(unsigned char* base)
    {
        Qs = reinterpret_cast<float*>(base);
        Cs = Qs + BM * LDK;
        hcs = Cs + BN * LDK;                                  // two buffers of BN (tile parity)
        ccol = reinterpret_cast<int*>(hcs + 2 * BN);          // two buffers of BN
        bounds = reinterpret_cast<float*>(ccol + 2 * BN);
        qid = reinterpret_cast<int*>(bounds + BM);
        hqs = reinterpret_cast<float*>(qid + BM);
        wmax = hqs + BM;                                      // [2 parities][4 wavefronts], then 8 spare words
        lists = reinterpret_cast<unsigned long long*>(wmax + 16);
        queues = reinterpret_cast<unsigned short*>(lists + BM * KL);
    }
};

extern __shared__ __align__(16) unsigned char sweep_smem[];

// Rare path of the tile epilogue, in two real calls so that its registers do not weigh on the
// multiply loop.
//
// compact_block: stream-compacts the pairs of one 32x32 block that pass the filter into the
// wavefront's queue (entry = query lane << 8 | candidate row within the tile).  `t` holds the
// block's accumulators, `tag` the lane's query row (k-NN self-join: to skip itself; -1 when nothing
// is to be skipped) or the lane's query colour (cross-colour 1-NN: to skip its own component).
// Returns the new queue length, or -1 (nothing written) when the block might not fit: the caller then
// resolves the queue and calls again with an empty one.
template <int KL, bool MASKED>
__device__ __attribute__((noinline)) int compact_block(v16f t, int b, float bound, int tag, int col0,
                                                       int colbuf, int N, int qcount)
{
    const SweepLds<KL> L(sweep_smem);
    const int* ccol = L.ccol + colbuf * BN;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int l32 = lane & 31;
    const int lhalf = lane >> 5;
    unsigned short* myq = L.queues + wave * QCAP;
    const bool real_query = L.qid[wave * 32 + l32] >= 0;    // padding rows of the last panel
    // A wavefront instruction costs four cycles of the SIMD whatever it does, and this routine runs for every
    // flagged block, so it is written for instruction count.  First one compare per accumulator row, whose
    // ballots also bound the number of entries (if the bound fits the queue, nothing below can overflow; if it
    // does not, the caller resolves the queue and calls again with an empty one, which always fits).  Then
    // only the rows that hold a passing accumulator pay for the full test and the write.
    unsigned long long rough[16];
    int upper = 0;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        rough[r] = __ballot(t[r] >= bound);
        upper += __popcll(rough[r]);
    }
    if (qcount + upper > QCAP) return -1;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        if (rough[r] == 0ull) continue;
        const int cl = b * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3);
        const int cg = col0 + cl;
        // candidates past the end or padding rows carry h = +inf, i.e. an accumulator of -inf
        bool pred = real_query && (t[r] >= bound) && (t[r] > -__builtin_inff()) && (cg < N);
        if (MASKED) pred = pred && (ccol[cl] != tag);
        else pred = pred && (cg != tag);
        const unsigned long long mask = __ballot(pred);
        const int pre = __builtin_amdgcn_mbcnt_hi((unsigned int)(mask >> 32),
                          __builtin_amdgcn_mbcnt_lo((unsigned int)mask, 0u));
        if (pred) myq[qcount + pre] = (unsigned short)((l32 << 8) | cl);
        qcount += __popcll(mask);
    }
    return qcount;
}

// group8_list_insert: the eight 8-lane groups of a wavefront each hold one re-evaluated pair (`key`, and the
// query lane `ql` it belongs to, the same in all lanes of a group; `want`: the pair beat its query's k-th
// entry when it was tested).  All eight keys go into their queries' sorted lists in one round: a group's
// lane g holds entries g*E .. g*E+E-1 of the list (E = KL/8), counts how many of them precede the key, the
// counts of the group give the key's position (E ballots, no reduction tree), every lane rebuilds its E
// entries (the one before its first comes from the lane below through a DPP row shift) and writes them back;
// the last entry drops out.  Two keys of one query cannot share a round: the higher group waits for the
// next one, so a round costs one LDS read and one write per lane whatever the number of lists.  On change
// the query's filter bound is refreshed from the new k-th entry: bound = h_q - worst/2.
// (One lane per list entry and 64/KL lists per round, as this routine did before, needs four rounds for
// eight keys at k = 32; the rounds, not the re-evaluation, were most of the rare path.)
__device__ inline unsigned long long dpp_from_lane_below(unsigned long long v)
{
    const int lo = __builtin_amdgcn_update_dpp(0, (int)(unsigned int)v, 0x111, 0xf, 0xf, false);          // row_shr:1
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(unsigned int)(v >> 32), 0x111, 0xf, 0xf, false);
    return ((unsigned long long)(unsigned int)hi << 32) | (unsigned int)lo;
}

template <int KL>
__device__ inline void group8_list_insert(bool want, unsigned long long key, int ql, unsigned long long* mylists,
                                          int k, const float* hqs, float* bounds, int lane)
{
    static_assert(KL % 8 == 0, "one list is spread over the eight lanes of a group");
    constexpr int E = KL / 8;
    const int grp = lane >> 3, g8 = lane & 7;
    unsigned long long pending = __ballot(want && g8 == 0);              // bit 8*grp: group grp still has its key
    while (pending) {
        // lane g of every group compares the group's query with group g's
        const int other_q = __shfl(ql, g8 * 8);
        const bool clash = g8 < grp && ((pending >> (g8 * 8)) & 1ull) && other_q == ql;
        const unsigned long long clashes = __ballot(clash);
        const bool go = ((pending >> (grp * 8)) & 1ull) && (((clashes >> (grp * 8)) & 0xffull) == 0ull);
        unsigned long long* lst = mylists + (size_t)ql * KL + g8 * E;
        unsigned long long old[E];
        int cnt = 0;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            old[e] = go ? lst[e] : ~0ull;
            cnt += (g8 * E + e < k && old[e] < key) ? 1 : 0;
        }
        // the list ascends, so the entries that precede the key are a prefix: its length is the key's position
        int pos = 0;
#pragma unroll
        for (int c = 1; c <= E; ++c) {
            const unsigned long long m = __ballot(go && cnt >= c);
            pos += __popcll((m >> (grp * 8)) & 0xffull);
        }
        const bool ins = go && pos < k;                                   // the key still beats the k-th entry
        const unsigned long long below = dpp_from_lane_below(old[E - 1]);
        unsigned long long now[E];
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const int i = g8 * E + e;
            const unsigned long long moved = e == 0 ? below : old[e > 0 ? e - 1 : 0];
            now[e] = (i < pos || i >= k) ? old[e] : (i == pos ? key : moved);
            if (ins && i == k - 1) bounds[ql] = hqs[ql] - 0.5f * __uint_as_float((unsigned int)(now[e] >> 32));
        }
        if (ins && g8 * E + E > pos && g8 * E < k) {
#pragma unroll
            for (int e = 0; e < E; ++e) lst[e] = now[e];
        }
        pending &= ~__ballot(go && g8 == 0);
    }
}

// resolve_queue: re-evaluates every queued pair exactly (eight pairs per pass, 8 lanes each),
// drops those that do not beat their query's current k-th entry, inserts the rest into the query
// lists and refreshes the bounds.
template <int KL, bool VEC4>
__device__ __attribute__((noinline)) void resolve_queue(int qcount, int col0, const float* __restrict__ Xq,
                                                        const float* __restrict__ Xc,
                                                        const int32_t* __restrict__ c_id, int d, int k)
{
    const SweepLds<KL> L(sweep_smem);
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const unsigned short* myq = L.queues + wave * QCAP;
    unsigned long long* mylists = L.lists + (size_t)wave * 32 * KL;
    __builtin_amdgcn_wave_barrier();
    const int grp = lane >> 3, g8 = lane & 7;
    for (int s = 0; s < qcount; s += 8) {
        const int e = s + grp;
        const bool valid = e < qcount;
        const unsigned int ent = valid ? myq[e] : 0u;
        const int ql = (int)(ent >> 8);
        const int cg = col0 + (int)(ent & 255u);
        const int qrow = L.qid[wave * 32 + ql];
        const float* xa = Xq + (size_t)(valid ? qrow : 0) * d;
        const float* xb = Xc + (size_t)(valid ? cg : 0) * d;
        const int cid = (c_id && valid) ? ((global_ints)c_id)[cg] : cg;   // id that orders ties and is reported
#ifdef SLHC_STUDY_DOUBLE_EVAL
        const float dist = fmaxf(group8_sqdist<VEC4>(xa, xb, d, g8, valid), group8_sqdist<VEC4>(xb, xa, d, g8, valid));
#else
        const float dist = group8_sqdist<VEC4>(xa, xb, d, g8, valid);
#endif
        const unsigned long long key = make_key(dist, cid);
        // a stale k-th entry is only larger than the current one, so this test never drops a
        // pair that belongs in the list; group8_list_insert tests again
        if constexpr (KL == 1) {
            // k = 1: a list is one key, so the eight group leaders update their queries at once
            // (64-bit LDS minimum; two pairs of one query in the same pass are ordered by it) and
            // then refresh the bounds from what the lists hold, as group8_list_insert would
            if (valid && g8 == 0) atomicMin(&mylists[ql], key);
            __builtin_amdgcn_wave_barrier();
            if (valid && g8 == 0)
                L.bounds[wave * 32 + ql] = L.hqs[wave * 32 + ql] - 0.5f * __uint_as_float((unsigned int)(mylists[ql] >> 32));
            continue;
        }
        if constexpr (KL > 1) {
            const bool want = valid && key < mylists[(size_t)ql * KL + k - 1];
            group8_list_insert<KL>(want, key, ql, mylists, k, L.hqs + wave * 32, L.bounds + wave * 32, lane);
        }
    }
    __builtin_amdgcn_wave_barrier();
}

// Seeding of 1-NN sweeps.  In the first tile of a panel no query has a threshold yet, so all of its
// 128 x 32 pairs per wavefront would pass the filter and be re-evaluated one after the other, which
// costs as much as dozens of later tiles when a panel only multiplies a few hundred of them (row
// order, pruned connection sweeps).  The accumulators already rank the candidates: every lane takes
// the admissible candidate with the largest accumulator among the 64 it holds (seed_block, one call
// per block), those 64 pairs per wavefront are evaluated exactly and recorded (seed_resolve), and the
// tile then goes through the filter with the thresholds they leave.  The seeds are ordinary exact
// candidates, so the result of the sweep does not depend on them.
struct SeedPick { float v; int cl; };
constexpr int SEED_AGAIN_LANES = 8;     // later tiles of a pruned 1-NN sweep are seeded too from this many passing lanes on

template <int KL, bool MASKED>
__device__ __attribute__((noinline)) SeedPick seed_block(v16f t, int b, SeedPick cur, int tag, int col0,
                                                         int colbuf, int N)
{
    const SweepLds<KL> L(sweep_smem);
    const int* ccol = L.ccol + colbuf * BN;
    const int lhalf = (threadIdx.x & 63) >> 5;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int cl = b * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3);
        const int cg = col0 + cl;
        bool ok = cg < N;
        if (MASKED) ok = ok && (ccol[cl] != tag);
        else ok = ok && (cg != tag);
        if (ok && t[r] > cur.v) { cur.v = t[r]; cur.cl = cl; }
    }
    return cur;
}

template <int KL, bool VEC4>
__device__ __attribute__((noinline)) void seed_resolve(SeedPick pick, int col0, const float* __restrict__ Xq,
                                                       const float* __restrict__ Xc,
                                                       const int32_t* __restrict__ c_id, int d, int k)
{
    const SweepLds<KL> L(sweep_smem);
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int l32 = lane & 31;
    unsigned short* myq = L.queues + wave * QCAP;
    const bool has = pick.cl >= 0 && L.qid[wave * 32 + l32] >= 0;
    const unsigned long long mask = __ballot(has);
    if (mask == 0ull) return;
    const int pre = __builtin_amdgcn_mbcnt_hi((unsigned int)(mask >> 32),
                      __builtin_amdgcn_mbcnt_lo((unsigned int)mask, 0u));
    if (has) myq[pre] = (unsigned short)((l32 << 8) | pick.cl);
    resolve_queue<KL, VEC4>(__popcll(mask), col0, Xq, Xc, c_id, d, k);
}

// Seeding of pruned k-NN sweeps (k > 1).  The same problem as above, but a list has to be full before
// its query has a threshold, so the first tile must deliver at least k candidates per query, and
// should not deliver many more.  Each of the two lanes that hold a query's 128 accumulators finds, by
// bisection with counting (seed_range, seed_count: one call per block and step), a value that at least
// k/2 + 1 of its 64 accumulators reach; the smaller of the two values is the provisional bound of the
// query, the pairs that reach it go through the batched path (which fills the list and sets the
// threshold), and their accumulators are then set to -inf so that the ordinary epilogue of the tile,
// which runs next under the real threshold, only sees the others.
struct SeedRange { float lo, hi; };

__device__ __attribute__((noinline)) SeedRange seed_range(v16f t, SeedRange cur)
{
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        if (t[r] > -__builtin_inff()) {
            cur.lo = fminf(cur.lo, t[r]);
            cur.hi = fmaxf(cur.hi, t[r]);
        }
    }
    return cur;
}

__device__ __attribute__((noinline)) int seed_count(v16f t, float x)
{
    int n = 0;
#pragma unroll
    for (int r = 0; r < 16; ++r) n += (t[r] >= x) ? 1 : 0;
    return n;
}

// Deferred form of the rare path, for the sweeps that multiply every tile.  After the first tiles of
// a panel a step leaves one or two surviving pairs per wavefront, and resolving them at once costs a
// full dependent chain (queue, two row loads from L2, reduction, insert) in every step.  Here a step
// only compacts a small number of survivors into a queue that lives across steps (its length sits in
// LDS, one word per wavefront); the queue is resolved when it holds DEFER_MIN pairs, eight pairs per
// pass, and at the end of the panel.  Thresholds are then a few steps stale, which is safe: a stale
// threshold is larger and only lets more pairs through.  Entries are 32-bit (query lane << 27 |
// candidate row) so that they outlive the step they were found in (candidate sets of 2^27 rows and
// more are not deferred); the queue shares the LDS bytes of the 16-bit queue that compact_block and
// resolve_queue use for blocks with many survivors, so that path resolves the deferred pairs first.
constexpr int QCAP_WIDE = QCAP / 2;
constexpr int DEFER_MIN = 8;           // measured best at N = 1M, d = 128, k = 32 (4, 16, 32, 64 are slower)
constexpr int DEFER_BLOCK_MAX = 32;
constexpr int DEFER_ROW_BITS = 27;

template <int KL>
__device__ inline int* deferred_count(const SweepLds<KL>& L, int wave)
{
    return reinterpret_cast<int*>(L.wmax + 12) + wave;
}

// Resolves the first `qcount` entries of the deferred queue and empties it.
template <int KL, bool VEC4>
__device__ __attribute__((noinline)) void resolve_deferred(int qcount, const float* __restrict__ Xq,
                                                           const float* __restrict__ Xc,
                                                           const int32_t* __restrict__ c_id, int d, int k)
{
    const SweepLds<KL> L(sweep_smem);
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const unsigned int* myq = reinterpret_cast<const unsigned int*>(L.queues + wave * QCAP);
    unsigned long long* mylists = L.lists + (size_t)wave * 32 * KL;
    __builtin_amdgcn_wave_barrier();
    const int grp = lane >> 3, g8 = lane & 7;
    for (int s = 0; s < qcount; s += 8) {
        const int e = s + grp;
        const bool valid = e < qcount;
        const unsigned int ent = valid ? myq[e] : 0u;
        const int ql = (int)(ent >> DEFER_ROW_BITS);
        const int cg = (int)(ent & ((1u << DEFER_ROW_BITS) - 1u));
        const int qrow = L.qid[wave * 32 + ql];
        const float* xa = Xq + (size_t)(valid ? qrow : 0) * d;
        const float* xb = Xc + (size_t)(valid ? cg : 0) * d;
        const int cid = (c_id && valid) ? ((global_ints)c_id)[cg] : cg;
        const float dist = group8_sqdist<VEC4>(xa, xb, d, g8, valid);
        const unsigned long long key = make_key(dist, cid);
        if constexpr (KL == 1) {
            if (valid && g8 == 0) atomicMin(&mylists[ql], key);
            __builtin_amdgcn_wave_barrier();
            if (valid && g8 == 0)
                L.bounds[wave * 32 + ql] = L.hqs[wave * 32 + ql] - 0.5f * __uint_as_float((unsigned int)(mylists[ql] >> 32));
            continue;
        }
        if constexpr (KL > 1) {
            const bool want = valid && key < mylists[(size_t)ql * KL + k - 1];
            group8_list_insert<KL>(want, key, ql, mylists, k, L.hqs + wave * 32, L.bounds + wave * 32, lane);
        }
    }
    __builtin_amdgcn_wave_barrier();
    if (lane == 0) *deferred_count(L, wave) = 0;
    __builtin_amdgcn_wave_barrier();
}

// Appends the passing pairs of one 32x32 block to the deferred queue and returns its new length,
// or -1 when the block has more than DEFER_BLOCK_MAX of them, the queue is full or a candidate row does
// not fit an entry (what was written then lies beyond the queue's length and is ignored).  A flagged
// block holds one or two such pairs in one or two of its 16 accumulator rows, so a row is first tested
// with a single compare and a wavefront-uniform branch; rows beyond N need no test of their own here:
// the pair test includes cg < N.
template <int KL, bool MASKED>
__device__ __attribute__((noinline)) int defer_block(v16f t, int b, float bound, int tag, int col0, int colbuf, int N)
{
    const SweepLds<KL> L(sweep_smem);
    const int* ccol = L.ccol + colbuf * BN;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int l32 = lane & 31;
    const int lhalf = lane >> 5;
    unsigned int* myq = reinterpret_cast<unsigned int*>(L.queues + wave * QCAP);
    int* cnt = deferred_count(L, wave);
    const int qcount0 = *cnt;
    const bool real_query = L.qid[wave * 32 + l32] >= 0;
    if (N > (1 << DEFER_ROW_BITS)) return -1;
    const int limit = (qcount0 + DEFER_BLOCK_MAX < QCAP_WIDE) ? qcount0 + DEFER_BLOCK_MAX : QCAP_WIDE;
    int qcount = qcount0;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        if (__ballot(t[r] >= bound) == 0ull) continue;
        const int cl = b * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3);
        const int cg = col0 + cl;
        bool pred = real_query && (t[r] >= bound) && (t[r] > -__builtin_inff()) && (cg < N);
        if (MASKED) pred = pred && (ccol[cl] != tag);
        else pred = pred && (cg != tag);
        const unsigned long long mask = __ballot(pred);
        if (mask == 0ull) continue;
        const int more = __popcll(mask);
        if (qcount + more > limit) return -1;
        const int pre = __builtin_amdgcn_mbcnt_hi((unsigned int)(mask >> 32),
                          __builtin_amdgcn_mbcnt_lo((unsigned int)mask, 0u));
        if (pred) myq[qcount + pre] = ((unsigned int)l32 << DEFER_ROW_BITS) | (unsigned int)cg;
        qcount += more;
    }
    if (qcount != qcount0) {
        __builtin_amdgcn_wave_barrier();
        if (lane == 0) *cnt = qcount;
        __builtin_amdgcn_wave_barrier();
    }
    return qcount;
}

// Tile epilogue after the hot filter flagged blocks `flagged` of this wavefront: all blocks go
// through one queue, so the exact re-evaluation runs once per tile step.  Expands at its call site
// with static block indices (a dynamic index into the accumulators would spill them).
#define FINE_MARK(i) do { } while (0)      // redefined for study builds where the phase timers exist
#ifdef SLHC_STUDY_DOUBLE_COMPACT
#define STUDY_AGAIN(...) __VA_ARGS__
#else
#define STUDY_AGAIN(...) do { } while (0)
#endif
#define SLHC_SELECT_TILE(KL_, MASKED_, VEC4_)                                                               \
    do {                                                                                                    \
        int qn_ = 0;                                                                                        \
        FINE_MARK(6);                                                                                       \
        _Pragma("unroll") for (int b_ = 0; b_ < 4; ++b_) {                                                  \
            if (flagged & (1u << b_)) {                                                                     \
                int r_ = wave_uniform(compact_block<KL_, MASKED_>(acc[b_], b_, bound, my_tag, col0, colbuf_, N, qn_)); \
                STUDY_AGAIN(r_ = compact_block<KL_, MASKED_>(acc[b_], b_, bound, my_tag, col0, colbuf_, N, qn_)); \
                if (r_ < 0) {                                                                               \
                    survivors += (unsigned int)qn_;                                                         \
                    resolve_queue<KL_, VEC4_>(qn_, col0, Xq, Xc, p.c_id, d, k);                             \
                    bound = bounds[my_q_local];                                                             \
                    r_ = wave_uniform(compact_block<KL_, MASKED_>(acc[b_], b_, bound, my_tag, col0, colbuf_, N, 0)); \
                }                                                                                           \
                qn_ = r_;                                                                                   \
            }                                                                                               \
        }                                                                                                   \
        FINE_MARK(0);                                                                                       \
        if (qn_ > 0) {                                                                                      \
            survivors += (unsigned int)qn_;                                                                 \
            resolve_queue<KL_, VEC4_>(qn_, col0, Xq, Xc, p.c_id, d, k);                                     \
            bound = bounds[my_q_local];                                                                     \
        }                                                                                                   \
        FINE_MARK(2);                                                                                       \
    } while (0)

template <int KL, bool MASKED, bool VEC4, bool SPLIT = false>
__global__ void __launch_bounds__(WG_THREADS, 2) sweep_kernel(SweepParams p)
{
    static_assert(!SPLIT || VEC4, "the split copy is read in 16-byte pieces");
    const SweepLds<KL> L(sweep_smem);
    float* Qs = L.Qs; float* Cs = L.Cs; float* hcs = L.hcs; int* ccol = L.ccol;
    float* bounds = L.bounds; int* qid = L.qid; float* hqs = L.hqs;
    unsigned long long* lists = L.lists;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int l32 = lane & 31;
    const int lhalf = lane >> 5;
    const int N = p.NC, d = p.d, k = p.k;          // N: candidate rows
    const float* __restrict__ Xq = p.Xq;
    const float* __restrict__ Xc = p.Xc;
    const float* __restrict__ hq = SPLIT ? p.hq_split : p.hq;          // the norms that go with the rows multiplied
    const float* __restrict__ hc = SPLIT ? p.hc_split : p.hc;
    const int nq = MASKED ? p.m : p.NQ;
    const int npanels = (nq + BM - 1) / BM;
    const int ntiles = (N + BN - 1) / BN;
    const int nchunks = (d + KC - 1) / KC;
    const int ld_row = tid >> 3;          // 0..31 (+32 i)
    const int ld_col = (tid & 7) * 4;     // 0..28
    unsigned long long* mylists = lists + (size_t)wave * 32 * KL;
    unsigned long long survivors = 0;
    unsigned long long tiles_done = 0;
    // SPLIT: the chunks are staged from the split bfloat16 copies (see SweepParams::Xq_split), whose rows hold
    // whole chunks (stride nchunks * 32 words, zeros past column d), and multiplied on the bf16 MFMA; the exact
    // re-evaluation of the pairs that pass reads Xq / Xc as always.
    const float* __restrict__ Xq_ld = SPLIT ? p.Xq_split : Xq;
    const float* __restrict__ Xc_ld = SPLIT ? p.Xc_split : Xc;
    const int d_ld = SPLIT ? nchunks * KC : d;

    // Work item = (query panel, segment of the candidate tiles).  With one segment a workgroup
    // sweeps all candidates for its panel; with few query rows the candidates are split so that
    // the whole chip works, and the partial results meet in p.out_key (see SweepParams).
    const int nseg = p.segments > 1 ? p.segments : 1;
    const int nitems = npanels * nseg;
    for (int item = blockIdx.x; item < nitems; item += gridDim.x) {
        const int panel = item % npanels;
        const int seg = item / npanels;
        const int t_begin = (int)((long long)seg * ntiles / nseg);
        const int t_end = (int)((long long)(seg + 1) * ntiles / nseg);
        __syncthreads();          // previous panel fully written out before its state is reused
        if (tid < BM) {
            const int qi = panel * BM + tid;
            int row = -1;
            if (qi < nq) row = (MASKED && p.rows) ? p.rows[qi] : qi;
            if ((unsigned int)row >= (unsigned int)p.NQ) row = -1;   // never index Xq with a bad row
            if (!MASKED && p.q_out_row && row >= 0 && p.q_out_row[row] < 0) row = -1;   // padding row
            qid[tid] = row;
            hqs[tid] = row >= 0 ? hq[row] : 0.f;
            bounds[tid] = row >= 0 ? -__builtin_inff() : __builtin_inff();
        }
        for (int i = tid; i < BM * KL; i += WG_THREADS) lists[i] = LIST_SENTINEL;
        __syncthreads();

        // Element offsets of the rows this thread stages.  Rows past the end are clamped to a
        // valid row: such queries carry a +inf bound and such candidates a +inf h, so whatever
        // is multiplied for them can never pass the filter.
        unsigned int qoff[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = qid[ld_row + 32 * i];
            qoff[i] = (unsigned int)(r >= 0 ? r : 0) * (unsigned int)d_ld;
        }
        const int my_q_local = wave * 32 + l32;
        const int my_qrow = qid[my_q_local];
        int my_qcol = -1;
        if (MASKED) my_qcol = my_qrow >= 0 ? p.qcolour[my_qrow] : -1;
        float bound = bounds[my_q_local];

        v4f qreg[4], creg[4];
        float hreg = 0.f;
        int colreg = 0;
        // VEC4: a chunk is loaded from a wavefront-uniform base (the chunk's first column) plus per-lane element
        // offsets that change once per panel (queries) and once per tile (candidates, rows clamped to N - 1), so
        // a chunk costs little address arithmetic.  Only the last chunk can reach past column d: there the dead
        // lanes take the chunk's first quad instead and their values are zeroed when they are staged.
        const bool last_has_dead = !SPLIT && d < nchunks * KC;
        const bool dead_lane = (nchunks - 1) * KC + ld_col >= d;           // in the last chunk
        unsigned int qlo[4], clo[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) { qlo[i] = qoff[i] + (unsigned int)ld_col; clo[i] = 0u; }
        auto gload = [&](int tile, int chunk) {
            const int col = chunk * KC + ld_col;
            const int crow0 = tile * BN + ld_row;
            if (VEC4) {
                if (chunk == 0) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        int crow = crow0 + 32 * i;
                        crow = crow < N ? crow : N - 1;
                        clo[i] = (unsigned int)crow * (unsigned int)d_ld + (unsigned int)ld_col;
                    }
                }
                const float* qb = Xq_ld + chunk * KC;
                const float* cb = Xc_ld + chunk * KC;
                if (chunk == nchunks - 1 && last_has_dead) {
                    const unsigned int back = dead_lane ? (unsigned int)ld_col : 0u;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        qreg[i] = *reinterpret_cast<const v4f*>(qb + (qlo[i] - back));
                        creg[i] = *reinterpret_cast<const v4f*>(cb + (clo[i] - back));
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        qreg[i] = *reinterpret_cast<const v4f*>(qb + qlo[i]);
                        creg[i] = *reinterpret_cast<const v4f*>(cb + clo[i]);
                    }
                }
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    int crow = crow0 + 32 * i;
                    crow = crow < N ? crow : N - 1;
                    v4f q, c;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const bool live = col + e < d;
                        const unsigned int ce = live ? (unsigned int)(col + e) : 0u;
                        q[e] = Xq[qoff[i] + ce];
                        c[e] = Xc[(unsigned int)crow * (unsigned int)d + ce];
                    }
                    qreg[i] = q;
                    creg[i] = c;
                }
            }
            if (chunk == 0 && tid < BN) {
                const int crow = tile * BN + tid;
                const int cr = crow < N ? crow : N - 1;
                hreg = hc[cr];
                if (MASKED) colreg = p.ccolour[cr];
            }
        };

        v16f acc[4];
        if (t_begin < t_end) gload(t_begin, 0);
        tiles_done += (unsigned long long)(t_end - t_begin);
        for (int tile = t_begin; tile < t_end; ++tile) {
            const int col0 = tile * BN;
            for (int chunk = 0; chunk < nchunks; ++chunk) {
                __syncthreads();                       // everyone is done reading the staged step
                // values staged past the last feature column were loaded from a valid address and are zeroed
                // here, at the point of use, so the loads stay in flight until now; only the last chunk has any
                if (!VEC4 || (chunk == nchunks - 1 && last_has_dead)) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        v4f q = qreg[i], c = creg[i];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const bool live = chunk * KC + ld_col + (VEC4 ? 0 : e) < d;
                            q[e] = live ? q[e] : 0.f;
                            c[e] = live ? c[e] : 0.f;
                        }
                        *reinterpret_cast<v4f*>(Qs + (ld_row + 32 * i) * LDK + ld_col) = q;
                        *reinterpret_cast<v4f*>(Cs + (ld_row + 32 * i) * LDK + ld_col) = c;
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        *reinterpret_cast<v4f*>(Qs + (ld_row + 32 * i) * LDK + ld_col) = qreg[i];
                        *reinterpret_cast<v4f*>(Cs + (ld_row + 32 * i) * LDK + ld_col) = creg[i];
                    }
                }
                if (chunk == 0 && tid < BN) {
                    const bool in_range = tile * BN + tid < N;
                    hcs[tid] = in_range ? -hreg : -__builtin_inff();     // negated here: the accumulators start from it as it is
                    if (MASKED) ccol[tid] = in_range ? colreg : -1;
                }
                __syncthreads();
                // prefetch the next step into registers while this one is multiplied
                {
                    int nt = tile, nc = chunk + 1;
                    if (nc == nchunks) { nc = 0; nt = tile + 1; }
                    if (nt < t_end) gload(nt, nc);
                }
                if (chunk == 0) {
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
#pragma unroll
                        for (int g = 0; g < 4; ++g) {
                            const v4f h = *reinterpret_cast<const v4f*>(hcs + b * 32 + 8 * g + 4 * lhalf);
                            acc[b][4 * g + 0] = h[0];
                            acc[b][4 * g + 1] = h[1];
                            acc[b][4 * g + 2] = h[2];
                            acc[b][4 * g + 3] = h[3];
                        }
                    }
                }
                if (SPLIT) {
                    // x_c . x_q ~ hi_c hi_q + hi_c lo_q + lo_c hi_q, 16 columns per instruction (see sweep_kernel_qreg)
#pragma unroll
                    for (int s2 = 0; s2 < 2; ++s2) {
                        v8bf ch[4], cl[4];
#pragma unroll
                        for (int b = 0; b < 4; ++b)
                            ch[b] = __builtin_bit_cast(v8bf, *reinterpret_cast<const v4f*>(Cs + (b * 32 + l32) * LDK + 4 * (2 * s2 + lhalf)));
#pragma unroll
                        for (int b = 0; b < 4; ++b)
                            cl[b] = __builtin_bit_cast(v8bf, *reinterpret_cast<const v4f*>(Cs + (b * 32 + l32) * LDK + 4 * (2 * s2 + lhalf) + 16));
                        const v8bf qh = __builtin_bit_cast(v8bf, *reinterpret_cast<const v4f*>(Qs + my_q_local * LDK + 4 * (2 * s2 + lhalf)));
                        const v8bf ql = __builtin_bit_cast(v8bf, *reinterpret_cast<const v4f*>(Qs + my_q_local * LDK + 4 * (2 * s2 + lhalf) + 16));
                        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                        for (int b = 0; b < 4; ++b) acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ch[b], qh, acc[b], 0, 0, 0);
#pragma unroll
                        for (int b = 0; b < 4; ++b) acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ch[b], ql, acc[b], 0, 0, 0);
#pragma unroll
                        for (int b = 0; b < 4; ++b) acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cl[b], qh, acc[b], 0, 0, 0);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                } else
#pragma unroll
                for (int kk = 0; kk < KC / 8; ++kk) {
                    const v4f qf = *reinterpret_cast<const v4f*>(Qs + my_q_local * LDK + kk * 8 + 4 * lhalf);
                    v4f cf[4];
#pragma unroll
                    for (int b = 0; b < 4; ++b)
                        cf[b] = *reinterpret_cast<const v4f*>(Cs + (b * 32 + l32) * LDK + kk * 8 + 4 * lhalf);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
#pragma unroll
                        for (int b = 0; b < 4; ++b)
                            acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(cf[b][e], qf[e], acc[b], 0, 0, 0);
                    }
                }
            }

            // ---- first tile of a 1-NN work item: seed the thresholds (see seed_block) ----
            if (k == 1 && tile == t_begin) {
                const int seed_tag = MASKED ? my_qcol : (p.exclude_self ? my_qrow : -1);
                SeedPick pick{-__builtin_inff(), -1};
                pick = seed_block<KL, MASKED>(acc[0], 0, pick, seed_tag, col0, 0, N);
                pick = seed_block<KL, MASKED>(acc[1], 1, pick, seed_tag, col0, 0, N);
                pick = seed_block<KL, MASKED>(acc[2], 2, pick, seed_tag, col0, 0, N);
                pick = seed_block<KL, MASKED>(acc[3], 3, pick, seed_tag, col0, 0, N);
                seed_resolve<KL, VEC4>(pick, col0, Xq, Xc, p.c_id, d, k);
                bound = bounds[my_q_local];
            }
            // ---- tile epilogue: filter (hot), then compact / re-evaluate / select (rare) ----
            unsigned int flagged = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                bool any = false;
                if (MASKED) {
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int4 cc = *reinterpret_cast<const int4*>(ccol + b * 32 + 8 * g + 4 * lhalf);
                        any |= (acc[b][4 * g + 0] >= bound) & (cc.x != my_qcol);
                        any |= (acc[b][4 * g + 1] >= bound) & (cc.y != my_qcol);
                        any |= (acc[b][4 * g + 2] >= bound) & (cc.z != my_qcol);
                        any |= (acc[b][4 * g + 3] >= bound) & (cc.w != my_qcol);
                    }
                } else {
#pragma unroll
                    for (int r = 0; r < 16; ++r) any |= (acc[b][r] >= bound);
                }
                if (__any(any)) flagged |= 1u << b;
            }
            if (__builtin_expect(flagged != 0, 0)) {
                const int my_tag = MASKED ? my_qcol : (p.exclude_self ? my_qrow : -1);
                const int colbuf_ = 0;
                SLHC_SELECT_TILE(KL, MASKED, VEC4);
            }
        }

        // ---- panel epilogue: lists are already ascending; write them out ----
        __builtin_amdgcn_wave_barrier();
        for (int ql = 0; ql < 32; ++ql) {
            const int row = qid[wave * 32 + ql];
            if (row < 0) {
                // a listed row outside [0, NQ): never dereferenced, answered with "nothing found"
                // (with p.out_key the slot keeps the sentinel it was filled with, which unpacks to the same)
                const int qi = panel * BM + wave * 32 + ql;
                if (MASKED && !p.out_key && lane == 0 && qi < nq) {
                    p.out_idx[qi] = -1;
                    p.out_dist[qi] = __builtin_inff();
                }
                continue;
            }
            if (lane < k) {
                const unsigned long long key = mylists[(size_t)ql * KL + lane];
                const float dist = __uint_as_float((unsigned int)(key >> 32));
                int idx = (int)(unsigned int)(key & 0xffffffffull);
                if (key == LIST_SENTINEL) idx = -1;
                const size_t o = MASKED ? (size_t)(panel * BM + wave * 32 + ql)
                                        : (size_t)(p.q_out_row ? p.q_out_row[row] : row) * k + lane;
                if (p.out_key) {
                    if (key != LIST_SENTINEL) atomicMin(p.out_key + o, key);
                } else {
                    p.out_idx[o] = idx;
                    p.out_dist[o] = dist;
                }
            }
        }
    }
    if (p.survivors && lane == 0 && survivors) atomicAdd(p.survivors, survivors);
    if (p.tiles_done && tid == 0 && tiles_done) atomicAdd(p.tiles_done, tiles_done);
}

// Variant for d <= 128 (d a multiple of 4): the query fragments of the MFMA B operand stay in
// registers for the whole sweep (DCH chunks of 32 columns -> 16*DCH registers per lane), so the
// query panel is read from memory once per panel instead of once per candidate tile, and LDS only
// stages candidates.  Candidate chunks are double-buffered in LDS (the buffer the streaming
// variant uses for queries is the second candidate buffer), which leaves ONE barrier per chunk:
// a wavefront can only overwrite buffer s&1 at step s+2 after every wavefront has passed the
// barrier of step s+1, i.e. has finished multiplying step s.  The per-tile candidate half norms
// and colours are double-buffered by step parity for the same reason.
//
// Tile pruning (when p.tile_c is given; not in the paper, which multiplies every tile): at the
// start of a panel the workgroup computes the bounding ball of its query rows and, for every
// candidate tile, a lower bound on any query-candidate distance of the pair of balls,
//     lb = max(0, |c_Q - c_T| - r_Q - r_T)^2     (rounded towards zero),
// into its slice of gap_ws.  A tile whose bound exceeds the largest current threshold of the
// panel's queries cannot change any list and is neither loaded nor multiplied.  Thresholds only
// shrink, so testing against an older maximum is safe; the maximum is exchanged between the four
// wavefronts through LDS slots that alternate with the step parity, which makes the skip decision
// identical in all wavefronts (they have to agree on the barrier sequence).
// Study builds (-DSLHC_PHASE_TIMERS): thread 0 of every workgroup accumulates shader-clock cycles per
// phase of the panel loop into p.phase_cycles[0..7].  Not compiled into the product library.
#ifdef SLHC_PHASE_TIMERS
#define PHASE_MARK(i)                                              \
    do {                                                           \
        const unsigned long long now_ = clock64();                 \
        ph[i] += now_ - ph_t;                                      \
        ph_t = now_;                                               \
    } while (0)
#else
#define PHASE_MARK(i) do { } while (0)
#endif
// study builds: compaction goes to phase slot 0 and the queue's resolution to slot 2 (both otherwise tiny)
#if defined(SLHC_PHASE_TIMERS) && defined(SLHC_PHASE_TIMERS_FINE)
#undef FINE_MARK
#define FINE_MARK(i) PHASE_MARK(i)
#endif

template <int KL, bool MASKED, int DCH, bool PRUNE, bool SPLIT = false>
__global__ void __launch_bounds__(WG_THREADS, 2) sweep_kernel_qreg(SweepParams p)
{
    const SweepLds<KL> L(sweep_smem);
    float* bounds = L.bounds; int* qid = L.qid; float* hqs = L.hqs;
    unsigned long long* lists = L.lists;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int l32 = lane & 31;
    const int lhalf = lane >> 5;
    const int N = p.NC, d = p.d, k = p.k;          // N: candidate rows
    const float* __restrict__ Xq = p.Xq;
    const float* __restrict__ Xc = p.Xc;
    const float* __restrict__ hq = SPLIT ? p.hq_split : p.hq;          // the norms that go with the rows multiplied
    const float* __restrict__ hc = SPLIT ? p.hc_split : p.hc;
    // cross 1-NN with a slot map: panel p holds the query rows among rows 128p .. 128p+127
    const bool aligned = PRUNE && MASKED && p.qslot != nullptr;
    const int nq = (MASKED && !aligned) ? p.m : p.NQ;
    const int npanels = (nq + BM - 1) / BM;
    const int ntiles = (N + BN - 1) / BN;
    const int ld_row = tid >> 3;          // 0..31 (+32 i)
    const int ld_col = (tid & 7) * 4;     // 0..28
    constexpr bool prune = PRUNE;         // p.tile_c, p.tile_r and p.gap_ws are given
    float* __restrict__ gap_own = prune ? p.gap_ws + (size_t)blockIdx.x * ntiles : nullptr;
    unsigned long long* mylists = lists + (size_t)wave * 32 * KL;
    unsigned long long survivors = 0;
    unsigned long long tiles_done = 0;
#ifdef SLHC_PHASE_TIMERS
    unsigned long long ph[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    unsigned long long ph_t = clock64();
#endif

    int* next_panel = reinterpret_cast<int*>(L.wmax + 8);      // LDS word after the wmax slots
    unsigned int* panel_thr_bits = reinterpret_cast<unsigned int*>(L.wmax + 9);   // see the panel prologue
    // Pruned cross 1-NN sweeps with a slot map may split every panel's scan into p.segments work items (item =
    // panel * segments + part): part s takes every segments-th position of the panel's scan order, starting at
    // position s, so each part begins among the near tiles; the parts keep separate thresholds and meet in
    // p.out_key by a 64-bit atomic minimum, which is the (distance, index) order of the lists.  A few panels
    // whose queries admit thousands of tiles otherwise outlast the rest of a launch several times over.
    // The pairs that pass the filter are either resolved step by step, all flagged blocks through one queue
    // (pruned sweeps, whose near tiles leave dozens per step; split-product sweeps, whose wider slack lets two to
    // three times as many through: 1M x 128 4.5 per wavefront and step, 1003 -> 901 ms against queueing), or queued
    // across steps and resolved eight at a time (every-tile sweeps with float32 products: one or two per step).
    constexpr bool BATCHED = PRUNE || SPLIT;
    constexpr bool CAN_SPLIT = PRUNE && MASKED && KL == 1;
    // k-NN sweeps of few panels (k > 1, every tile): part s of a panel takes the s-th range of the candidate
    // tiles and writes lists of its own; see SweepParams::part_idx.
    constexpr bool CAN_RANGE = !PRUNE && !MASKED && KL > 1;
    const int nparts = (CAN_SPLIT && aligned && p.segments > 1 && p.out_key != nullptr) ? p.segments
                     : (CAN_RANGE && p.segments > 1 && p.part_idx != nullptr && p.part_dist != nullptr) ? p.segments : 1;
    const bool listed_panels = PRUNE && MASKED && aligned && p.panel_list != nullptr;
    // Every-tile sweeps of many panels, range by range (p.carry_ranges, set by the launcher): the candidate tiles
    // are cut into ranges of 32 MiB and the work items (range, panel) are handed out in that order, so
    // that all workgroups in flight sweep the same range and its tiles are served by the memory-side cache instead
    // of being fetched from memory once per panel.  A panel's lists travel from range to range through the
    // output arrays: item (r, panel) starts from what item (r - 1, panel) wrote, thresholds included, so no
    // list is filled twice.  Item (r - 1, panel) was handed out a whole round of panels earlier and has long
    // finished; carry_ws[2 + panel] counts the ranges written, and an item waits for its predecessor there (the
    // workgroup that took the predecessor is running and waits only for still earlier items, so every wait
    // ends; it is bounded all the same, and a wait that runs out is reported in carry_fault).
    constexpr bool CAN_CARRY = !PRUNE;
    constexpr bool REGIONS = PRUNE && !MASKED;          // p.region_mode applies
    const int ncarry = (CAN_CARRY && p.carry_ranges > 1 && p.carry_ws != nullptr) ? p.carry_ranges : 1;
    const int nitems = ncarry > 1 ? npanels * ncarry : (listed_panels ? p.panel_list_n : npanels) * nparts;
    unsigned int* hand_out = ncarry > 1 ? p.carry_ws : (PRUNE ? p.panel_counter : nullptr);
    for (int item = blockIdx.x;; item += gridDim.x) {
        __syncthreads();          // previous panel fully written out before its state is reused
        if (hand_out) {
            // work items are handed out one by one: with pruning their cost differs by orders of
            // magnitude.  The counter only grows, so every workgroup reaches nitems and leaves.
            if (tid == 0) *next_panel = (int)atomicAdd(hand_out, 1u);
            __syncthreads();
            item = *next_panel;
        }
        if (item >= nitems) break;
        const int crange = ncarry > 1 ? item / npanels : 0;
        const int panel_at = ncarry > 1 ? item - crange * npanels : (nparts > 1 ? item / nparts : item);
        const int part = (ncarry == 1 && nparts > 1) ? item - panel_at * nparts : 0;
        const int panel = listed_panels ? p.panel_list[panel_at] : panel_at;
        if ((unsigned int)panel >= (unsigned int)npanels) continue;          // never trust a list entry as an index
#ifdef SLHC_STUDY_PANEL_STEPS
        const long long study_t0 = clock64();
#endif
        if (tid < BM) {
            const int qi = panel * BM + tid;
            int row = -1;
            if (qi < nq) row = (MASKED && !aligned && p.rows) ? p.rows[qi] : qi;
            if ((unsigned int)row >= (unsigned int)p.NQ) row = -1;   // never index Xq with a bad row
            if (!MASKED && p.q_out_row && row >= 0 && p.q_out_row[row] < 0) row = -1;   // padding row
            if (aligned && row >= 0 && p.qslot[row] < 0) row = -1;                      // not queried
            qid[tid] = row;
            hqs[tid] = row >= 0 ? hq[row] : 0.f;
            bounds[tid] = row >= 0 ? -__builtin_inff() : __builtin_inff();
        }
        for (int i = tid; i < BM * KL; i += WG_THREADS) lists[i] = LIST_SENTINEL;
        if (CAN_SPLIT && nparts > 1 && tid < BM && qid[tid] >= 0) {
            // what the other parts of this panel have found for this query so far: an exact candidate like any
            // other (the list of a 1-NN sweep is the one entry lists[tid])
            const unsigned long long found = __hip_atomic_load(p.out_key + p.qslot[qid[tid]], __ATOMIC_RELAXED,
                                                               __HIP_MEMORY_SCOPE_AGENT);
            if (found != LIST_SENTINEL) {
                lists[tid] = found;
                bounds[tid] = hqs[tid] - 0.5f * __uint_as_float((unsigned int)(found >> 32));
            }
        }
        if (tid < 8) { if (PRUNE) L.wmax[tid] = __builtin_inff(); else reinterpret_cast<int*>(L.wmax)[tid] = 0; }
        if (tid < 4) *deferred_count(L, tid) = 0;
        __syncthreads();
        // a listed row outside [0, NQ) is never dereferenced and is answered with "nothing found"
        if (MASKED && !aligned && tid < BM && qid[tid] < 0 && panel * BM + tid < nq) {
            p.out_idx[panel * BM + tid] = -1;
            p.out_dist[panel * BM + tid] = __builtin_inff();
        }
        // a panel without a single query has nothing to do (every wavefront reads the same qid)
        if (!__any(qid[lane] >= 0 || qid[lane + 64] >= 0)) continue;
        // Pruned k-NN sweeps in two launches (p.region_mode, see SweepParams): the second starts from the lists the
        // first wrote, like an item of a later range
        const bool lists_in = (CAN_CARRY && crange > 0) || (REGIONS && p.region_mode == 2 && p.tile_region != nullptr && panel < ntiles);
        if (lists_in) {
            // the lists item (crange - 1, panel) left in the output arrays, and the thresholds they imply
            if (CAN_CARRY && tid == 0) {
                int spins = 0;
                while (__hip_atomic_load(p.carry_ws + 2 + panel, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) < (unsigned int)crange) {
                    __builtin_amdgcn_s_sleep(16);
                    if (++spins > (1 << 22)) { if (p.carry_fault) atomicOr(p.carry_fault, 2u); break; }
                }
            }
            __syncthreads();
            // (thread 0's acquire has invalidated this CU's L1; the lists are read past it all the same)
            for (int i = tid; i < BM * KL; i += WG_THREADS) {
                const int ql = i / KL, j = i - ql * KL;
                const int row = qid[ql];
                if (row >= 0 && j < k) {
                    const size_t o = MASKED ? (size_t)(panel * BM + ql)
                                            : (size_t)(p.q_out_row ? p.q_out_row[row] : row) * k + j;
                    const int idx = (int)__hip_atomic_load(reinterpret_cast<const unsigned int*>(p.out_idx) + o, __ATOMIC_RELAXED,
                                                           __HIP_MEMORY_SCOPE_AGENT);
                    const unsigned int dbits = __hip_atomic_load(reinterpret_cast<const unsigned int*>(p.out_dist) + o,
                                                                 __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if (idx >= 0) lists[i] = ((unsigned long long)dbits << 32) | (unsigned int)idx;
                }
            }
            __syncthreads();
            if (tid < BM && qid[tid] >= 0) {
                const unsigned long long worst = lists[(size_t)tid * KL + k - 1];
                if (worst != LIST_SENTINEL) bounds[tid] = hqs[tid] - 0.5f * __uint_as_float((unsigned int)(worst >> 32));
            }
            __syncthreads();
        }
        PHASE_MARK(0);

        int panel_colour = -2;       // the colour all queries of the panel share (-2: they differ / unknown)
        // lower bounds of this panel against every candidate tile: its row of the table of all tile pairs when
        // the panel's rows lie in candidate tile `panel`, else computed here from a ball of the panel's own
        const bool table_row = prune && p.tile_gap != nullptr && panel < ntiles &&
                               (MASKED ? aligned : (p.own_tile_first != 0));
        const float* __restrict__ gap = table_row ? p.tile_gap + (size_t)panel * ntiles : gap_own;
        if (prune) {
            // ---- bounding ball of the panel's query rows (L.Cs is free here: d <= 128 floats)
            float* qc = L.Cs;                       // centre
            unsigned int* rq_bits = reinterpret_cast<unsigned int*>(L.Cs + 256);
            int* col_lo = reinterpret_cast<int*>(L.Cs + 257);
            int* col_hi = reinterpret_cast<int*>(L.Cs + 258);
            if (tid == 0) { *rq_bits = 0u; *col_lo = 0x7fffffff; *col_hi = -0x7fffffff - 1; }
            if (!table_row) {
                // partial column sums by groups of rows (fixed assignment and order: the centre is
                // the same in every run), then one thread per column adds the partial sums
                float* part = L.Cs + 512;           // [groups][d]
                const int ncol4 = d >> 2;
                const int groups = WG_THREADS / ncol4;
                const int c4 = tid % ncol4, grp = tid / ncol4;
                if (grp < groups) {
                    v4f sum = {0.f, 0.f, 0.f, 0.f};
                    for (int r = grp; r < BM; r += groups) {
                        const int row = qid[r];
                        if (row >= 0) sum += *reinterpret_cast<const v4f*>(Xq + (size_t)row * d + 4 * c4);
                    }
                    *reinterpret_cast<v4f*>(part + grp * d + 4 * c4) = sum;
                }
                __syncthreads();
                if (tid < d) {
                    int cnt = 0;
                    for (int r = 0; r < BM; ++r) cnt += qid[r] >= 0 ? 1 : 0;
                    float sum = 0.f;
                    for (int gq = 0; gq < groups; ++gq) sum += part[gq * d + tid];
                    qc[tid] = cnt > 0 ? sum / (float)cnt : 0.f;
                }
            }
            __syncthreads();
            if (tid < BM && qid[tid] >= 0) {
                if (!table_row) {
                    const float* x = Xq + (size_t)qid[tid] * d;
                    float s2 = 0.f;
                    for (int t = 0; t < d; ++t) { const float e = x[t] - qc[t]; s2 = __builtin_fmaf(e, e, s2); }
                    atomicMax(rq_bits, __float_as_uint(__builtin_sqrtf(s2)));
                }
                if (MASKED && p.tile_colour) {
                    const int c = p.qcolour[qid[tid]];
                    atomicMin(col_lo, c);
                    atomicMax(col_hi, c);
                }
            }
            __syncthreads();
            const float rq = __uint_as_float(*rq_bits);
            // the colour all queries of the panel share (-2: they differ, or no colour summary)
            panel_colour = (MASKED && p.tile_colour && *col_lo == *col_hi) ? *col_lo : -2;
            // The component's shared threshold is read ONCE per panel, by one thread, and handed to the others
            // through LDS (published by the barrier below): other workgroups lower the word while this one
            // starts, and four wavefronts that each read it for themselves can get four different values,
            // which then make them skip different tiles.
            if (MASKED && tid == 0 && p.comp_best != nullptr && panel_colour >= 0 && panel_colour < p.comp_count)
                *panel_thr_bits = __hip_atomic_load(p.comp_best + panel_colour, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            for (int t = tid; t < (table_row ? 0 : ntiles); t += WG_THREADS) {
                const float* c = p.tile_c + (size_t)t * d;
                float s2 = 0.f;
                for (int j = 0; j < d; j += 4) {
                    const v4f cv = *reinterpret_cast<const v4f*>(c + j);
                    const v4f qv = *reinterpret_cast<const v4f*>(qc + j);
                    float e;
                    e = cv[0] - qv[0]; s2 = __builtin_fmaf(e, e, s2);
                    e = cv[1] - qv[1]; s2 = __builtin_fmaf(e, e, s2);
                    e = cv[2] - qv[2]; s2 = __builtin_fmaf(e, e, s2);
                    e = cv[3] - qv[3]; s2 = __builtin_fmaf(e, e, s2);
                }
                // rounding: the centre distance may be 2e-5 too large, the radii 2e-5 too small
                const float rt = p.tile_r[t];
                const float g = __builtin_sqrtf(s2) * (1.f - 2e-5f) - (rq + rt) * (1.f + 2e-5f);
                float lb = g > 0.f ? g * g * (1.f - 1e-5f) : 0.f;
                // NaN marks a tile that is never needed: no valid row, or (cross 1-NN) every row of
                // it has the colour all queries of this panel have
                if (rt < 0.f) lb = __builtin_nanf("");
                if (MASKED && p.tile_colour && p.tile_colour[t] == panel_colour) lb = __builtin_nanf("");
                gap_own[t] = lb;
            }
            __syncthreads();
        }
        // (a row of the table knows nothing of colours: tiles in the colour of all the panel's queries are
        // sorted out where the bounds are read)
        const bool own_colour_test = MASKED && table_row && p.tile_colour != nullptr && panel_colour >= 0;
        // p.region_mode 1: only the candidate tiles of the panel's own region are of use; 2: only the others
        const int region_mode = (REGIONS && p.tile_region != nullptr && panel < ntiles) ? p.region_mode : 0;
        const int my_region = region_mode ? p.tile_region[panel] : 0;
        auto gap_of = [&](int t) -> float {
            float g = gap[t];
            if (own_colour_test && p.tile_colour[t] == panel_colour) g = __builtin_nanf("");
            if (REGIONS && region_mode && ((p.tile_region[t] == my_region) != (region_mode == 1))) g = __builtin_nanf("");
            return g;
        };
        PHASE_MARK(1);

        const int my_q_local = wave * 32 + l32;
        const int my_qrow = qid[my_q_local];
        int my_qcol = -1;
        if (MASKED) my_qcol = my_qrow >= 0 ? p.qcolour[my_qrow] : -1;
        float bound = bounds[my_q_local];
        // largest threshold among this wavefront's queries (no query: nothing can enter a list)
        float wave_thr_max = __any(my_qrow >= 0) ? __builtin_inff() : 0.f;
        // Shared component threshold (cross 1-NN with p.comp_best, all queries of one colour): only
        // the lightest edge leaving the component matters, so a candidate farther than the lightest
        // outgoing edge already known for this component is of no use to any of its queries.
        // comp_best[colour] holds that weight (bits of a non-negative float); it is folded into the
        // filter bound and into the tile-skipping threshold.  The sweep only reads it.  (Lowering it
        // from inside the sweep whenever a query finds a nearer row was tried and dropped: it made
        // rare runs end with an inconsistent forest state, and the read-only form is deterministic.)
        const bool shared_thr = PRUNE && MASKED && p.comp_best != nullptr && panel_colour >= 0 &&
                                panel_colour < p.comp_count;
        float thr_c = __builtin_inff();
        if (shared_thr) thr_c = __uint_as_float(*panel_thr_bits);       // the same value in all four wavefronts
        // With p.comp_best_lower the threshold also falls while the sweep runs: a wavefront whose query
        // finds a foreign row at distance w with lower_factor * w < thr_c lowers the component's word to
        // that (atomic minimum over the bits of non-negative floats), and every wavefront re-reads the
        // word every step or every few steps, a whole period ahead of its use so that the read never
        // waits.  The word never rises, so at any moment every candidate at most as far as the word's
        // FINAL value has passed (or will pass) the filter: the caller classifies the answers against
        // the final value (see SweepParams).
        // A wavefront's copy of the threshold (thr_c) differs from its neighbours' while it falls, and the
        // four wavefronts must take the same tile-skipping decision (they share the barrier sequence and
        // each stages a quarter of every tile): the decision therefore only uses the one value that was
        // read for the whole workgroup at the start of the panel (thr_c0, handed out through LDS) and
        // what each wavefront has published in the LDS slots; a wavefront's own copy only tightens its
        // own filter.
        const bool lowering = shared_thr && p.comp_best_lower != nullptr &&
                              (p.comp_size == nullptr || p.comp_size[panel_colour] >= p.comp_lower_min_size);
        const float thr_c0 = thr_c;
        unsigned int fresh_bits = __float_as_uint(thr_c);

        // query fragments: lane (l32, lhalf) holds columns kk*8 + 4*lhalf .. +3 of its query row
        // (SPLIT: per chunk of 32 columns and per 16-column step s, the 8 hi values of columns 16 s + 8 lhalf ..
        // in qf[4 chunk + s] and the 8 lo values in qf[4 chunk + 2 + s]; a chunk of the split copy holds its 32 hi
        // values in the first 16 words and its 32 lo values in the last 16)
        v4f qf[DCH * 4];
        {
            const unsigned int qo = (unsigned int)(my_qrow >= 0 ? my_qrow : 0) * (unsigned int)d;
#pragma unroll
            for (int kk = 0; kk < DCH * 4; ++kk) {
                if (SPLIT) {
                    const int word = (kk >> 2) * KC + ((kk & 2) ? 16 : 0) + 4 * (2 * (kk & 1) + lhalf);
                    qf[kk] = *reinterpret_cast<const v4f*>(p.Xq_split + (qo + (unsigned int)word));
                } else {
                    const int col = kk * 8 + 4 * lhalf;
                    const bool live = col < d;
                    const v4f v = *reinterpret_cast<const v4f*>(Xq + (qo + (live ? (unsigned int)col : 0u)));
                    qf[kk] = live ? v : v4f{0.f, 0.f, 0.f, 0.f};
                }
            }
        }

        // Order in which the candidate tiles are visited.  Every-tile sweeps: 0, 1, 2, ...  Pruned
        // sweeps start at the tile the panel's own rows sit in (a self-join in the same row order
        // visits that tile before the scan starts) and move outwards on both sides in turn: c+1, c-1,
        // c+2, c-2, ... and on along the longer side once the shorter one is used up.  In a spatially
        // coherent order the nearest rows sit in the neighbouring tiles on either side, so the
        // thresholds tighten early and the gap test skips more of what follows.
        // `scan` indices count positions in that order; every lane of every wavefront evaluates
        // next_scan on the same data, so its result is workgroup-uniform.
        // (the second launch of a sweep by regions has no use for the panel's own tile; its scan still starts there)
        const bool rows_in_own_tile = PRUNE && !MASKED && p.own_tile_first && panel < ntiles;
        const int own_tile = (rows_in_own_tile && !(REGIONS && region_mode == 2)) ? panel : -1;
        int centre = 0;
        if (own_tile >= 0) centre = own_tile;
        else if (rows_in_own_tile) centre = panel;
        else if (aligned) centre = panel < ntiles ? panel : 0;
        else if (prune && MASKED && qid[0] >= 0) centre = qid[0] / BN;
        if (centre >= ntiles) centre = ntiles - 1;
        const int with_centre = own_tile >= 0 ? 0 : 1;        // the scan itself begins at the centre tile
        int nscan_all = own_tile >= 0 ? ntiles - 1 : ntiles;
        if (REGIONS && region_mode == 1 && p.tile_first != nullptr && p.tile_last != nullptr) {
            // the tiles of the panel's own region are a run around it, and the scan moves outwards from the centre:
            // it ends where the run does (a panel of a small cluster otherwise reads its whole row of lower bounds
            // to find nothing)
            const int left = panel - p.tile_first[panel], right = p.tile_last[panel] - panel;
            const int reach = left > right ? left : right;
            const int to_r = ntiles - 1 - centre, to_l = centre;
            const int within = (reach < to_l ? reach : to_l) + (reach < to_r ? reach : to_r) + (own_tile >= 0 ? 0 : 1);
            if (reach >= 0 && within < nscan_all) nscan_all = within;
        }
        // positions of this work item: part, part + nparts, ... of the panel's scan order
        const bool ranged = (CAN_RANGE && nparts > 1) || (CAN_CARRY && ncarry > 1);
        const int range_at = ncarry > 1 ? crange : part, range_count = ncarry > 1 ? ncarry : nparts;
        const int range_begin = ranged ? (int)((long long)range_at * ntiles / range_count) : 0;
        const int range_end = ranged ? (int)((long long)(range_at + 1) * ntiles / range_count) : ntiles;
        const int nscan = ranged ? range_end - range_begin
                        : nparts > 1 ? (nscan_all > part ? (nscan_all - part + nparts - 1) / nparts : 0) : nscan_all;
        const int side_r = ntiles - 1 - centre, side_l = centre;
        const int side_min = side_r < side_l ? side_r : side_l;
        auto scan_tile = [&](int i) -> int {                   // 0 <= i < nscan
            if (!prune) return i + range_begin;
            if (nparts > 1) i = i * nparts + part;
            if (with_centre) { if (i == 0) return centre; --i; }
            if (i < 2 * side_min) { const int j = (i >> 1) + 1; return (i & 1) ? centre - j : centre + j; }
            const int r = i - 2 * side_min;
            return side_r > side_l ? centre + side_min + 1 + r : centre - side_min - 1 - r;
        };
        auto tile_of = [&](int i) -> int { return i >= nscan ? ntiles : scan_tile(i); };
        // (SCAN_AHEAD groups of 64 positions are read at once: one group at a time the scan is a chain of dependent
        // loads, a microsecond each, and a panel that multiplies two tiles of 20 000 spends its time there)
        constexpr int SCAN_AHEAD = MASKED ? SLHC_SCAN_AHEAD_1NN : SLHC_SCAN_AHEAD;
        auto next_scan = [&](int i, float thr_max) -> int {
            if (!prune) return i;
            while (i < nscan) {
                // (all the votes are taken before the first is looked at: a vote cannot move into a branch, so
                // the loads behind it cannot either)
                float g[SCAN_AHEAD];
#pragma unroll
                for (int u = 0; u < SCAN_AHEAD; ++u) {
                    const int ii = i + 64 * u + lane;
                    g[u] = ii < nscan ? gap_of(scan_tile(ii)) : __builtin_nanf("");
                }
                unsigned long long mask[SCAN_AHEAD];
#pragma unroll
                for (int u = 0; u < SCAN_AHEAD; ++u) mask[u] = __ballot(g[u] <= thr_max);          // false for NaN
#pragma unroll
                for (int u = 0; u < SCAN_AHEAD; ++u)
                    if (mask[u]) return i + 64 * u + __builtin_ctzll(mask[u]);
                i += 64 * SCAN_AHEAD;
            }
            return nscan;
        };

        v4f creg[4];
        float hreg = 0.f;
        int colreg = 0;
        // A chunk is loaded from a wavefront-uniform base (tile, chunk) plus four per-lane offsets, one per staged
        // row, that stay the same from tile to tile: a chunk costs no address arithmetic in the vector unit.
        // Only a tile that reaches past row N has other offsets (its rows are clamped to N - 1): they are
        // rewritten when such a tile comes and when the next full one follows.  Only the last chunk can reach
        // past column d: lanes that would take the first quad of that chunk instead (finite values of the same
        // row, multiplied by query fragments that are zero).
        unsigned int row_off[4];
        bool row_off_clamped;
        auto set_row_off = [&](int tile) {
            const int last = N - 1 - tile * BN;                 // last valid row of the tile, >= 0
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int r = ld_row + 32 * i;
                row_off[i] = (unsigned int)(r < last ? r : last) * (unsigned int)d + (unsigned int)ld_col;
            }
        };
        set_row_off(0);
        row_off_clamped = BN > N;
        const unsigned int dead_adj = (DCH - 1) * KC + ld_col < d ? 0u : (unsigned int)ld_col;
        auto gload = [&](int tile, int chunk) {
            const bool clamped = (tile + 1) * BN > N;
            if (clamped != row_off_clamped) { set_row_off(tile); row_off_clamped = clamped; }
            const float* base = (SPLIT ? p.Xc_split : Xc) + ((size_t)tile * BN * (size_t)d + (size_t)(chunk * KC));
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const unsigned int off = (chunk == DCH - 1 && d < DCH * KC) ? row_off[i] - dead_adj : row_off[i];
                creg[i] = *reinterpret_cast<const v4f*>(base + off);
            }
            if (chunk == 0 && tid < BN) {
                const int crow = tile * BN + tid;
                const int cr = crow < N ? crow : N - 1;
                hreg = hc[cr];
                if (MASKED) colreg = p.ccolour[cr];
            }
        };

        // largest threshold of this wavefront's 32 queries, from their bounds: thr = 2 (h_q - bound)
        auto refresh_wave_thr = [&]() {
            float t = (my_qrow >= 0) ? 2.f * (hqs[my_q_local] - bound) : 0.f;
            t = fmaxf(t, __shfl_xor(t, 1));
            t = fmaxf(t, __shfl_xor(t, 2));
            t = fmaxf(t, __shfl_xor(t, 4));
            t = fmaxf(t, __shfl_xor(t, 8));
            t = fmaxf(t, __shfl_xor(t, 16));
            // 2 (h_q - bound) reproduces the threshold up to a few ulps of h_q; widen it
            wave_thr_max = t + 4.f * 1.1920929e-07f * fmaxf(fabsf(hqs[my_q_local]), t);
            wave_thr_max = fmaxf(wave_thr_max, __shfl_xor(wave_thr_max, 1));
            wave_thr_max = fmaxf(wave_thr_max, __shfl_xor(wave_thr_max, 2));
            wave_thr_max = fmaxf(wave_thr_max, __shfl_xor(wave_thr_max, 4));
            wave_thr_max = fmaxf(wave_thr_max, __shfl_xor(wave_thr_max, 8));
            wave_thr_max = fmaxf(wave_thr_max, __shfl_xor(wave_thr_max, 16));
        };
        // a launch that starts from lists already written: their thresholds decide from the first tile on
        float first_thr = __builtin_inff();
        if (REGIONS && lists_in) {
            refresh_wave_thr();
            if (lane == 0) { L.wmax[wave] = wave_thr_max; L.wmax[4 + wave] = wave_thr_max; }
            __syncthreads();
            first_thr = fmaxf(fmaxf(L.wmax[0], L.wmax[1]), fmaxf(L.wmax[2], L.wmax[3]));
        }
        // ... and when even the nearest tile outside the panel's region lies beyond them (its lower bound, taken from
        // the table's row), the launch has nothing to add to this panel: no scan
        const bool nothing_outside = REGIONS && lists_in && table_row && p.region_other_min != nullptr &&
                                     p.region_other_min[panel] > first_thr;

        v16f acc[4];
        int scan_from = 0;                 // scan indices below this one are done or skipped
        int tile = own_tile;
        if (own_tile < 0) {
            const int first = nothing_outside ? nscan : next_scan(0, first_thr);
            tile = tile_of(first);
            scan_from = first + 1;
        }
        float ahead_gap = __builtin_nanf("");          // lower bound of scan position scan_from + lane (NaN: none)
        if (prune) ahead_gap = scan_from + lane < nscan ? gap_of(scan_tile(scan_from + lane)) : __builtin_nanf("");
 if (tile < ntiles) gload(tile, 0);
        PHASE_MARK(2);
        // split scans: this query's slot in p.out_key, the entry last published there, the word last read
        int part_slot = 0;
        unsigned long long part_published = LIST_SENTINEL, part_seen = LIST_SENTINEL;
        if (CAN_SPLIT && nparts > 1) {
            if (my_qrow >= 0) { part_slot = p.qslot[my_qrow]; part_published = mylists[l32]; }
            if (prune) refresh_wave_thr();       // the thresholds adopted at set-up
        }
        int step = 0;                      // multiplied tiles of this panel (buffer parity)
        while (tile < ntiles) {
            const int col0 = tile * BN;
            const int tpar = step & 1;
            float* hcs = L.hcs + tpar * BN;
            int* ccol = L.ccol + tpar * BN;
            int tile_after = ntiles;
#pragma unroll
            for (int chunk = 0; chunk < DCH; ++chunk) {
                // candidate buffer of this step: steps alternate between the two LDS buffers
                float* Cb = (((DCH & 1) ? (step + chunk) : chunk) & 1) ? L.Qs : L.Cs;
                // columns past d are staged as they were loaded (finite values of column 0): the query fragments
                // are zero there, so they add nothing
#pragma unroll
                for (int i = 0; i < 4; ++i) *reinterpret_cast<v4f*>(Cb + (ld_row + 32 * i) * LDK + ld_col) = creg[i];
                if (chunk == 0 && tid < BN) {
                    const bool in_range = col0 + tid < N;
                    hcs[tid] = in_range ? -hreg : -__builtin_inff();     // negated here: the accumulators start from it as it is
                    if (MASKED) ccol[tid] = in_range ? colreg : -1;
                }
                __syncthreads();
                // The loads of the next step are issued here, ahead of this step's multiplies, and
                // must stay here: left to itself the scheduler sinks them towards their use at
                // the end of the multiply block, which exposes their latency (measured: 6 % of
                // the whole sweep).
                if (chunk + 1 < DCH) {
                    gload(tile, chunk + 1);
                    __builtin_amdgcn_sched_barrier(0);
                } else {
                    PHASE_MARK(3);
                    // thresholds published in the epilogue of the previous step (other parity)
                    const float* wm = L.wmax + (tpar ^ 1) * 4;
                    float thr_max = prune ? fmaxf(fmaxf(wm[0], wm[1]), fmaxf(wm[2], wm[3])) : 0.f;
                    // a read takes about as long as 64 multiplies: with fewer per step (d < 128) it is issued
                    // every few steps only, and always consumed a whole period later
                    constexpr int REFRESH = DCH >= 4 ? 1 : 8 / DCH;
                    if (lowering && (step % REFRESH) == 0) {
                        // what the previous read brought, then the next read
                        thr_c = fminf(thr_c, __uint_as_float(fresh_bits));
                        fresh_bits = __hip_atomic_load(p.comp_best_lower + panel_colour, __ATOMIC_RELAXED,
                                                       __HIP_MEMORY_SCOPE_AGENT);
                    }
                    if (shared_thr) thr_max = fminf(thr_max, thr_c0);
                    // the lower bounds of the next 64 scan positions were read a step ago (ahead_gap): when
                    // one of them is admissible, as it nearly always is, the choice costs no memory wait
                    int nxt;
                    if (prune) {
                        const unsigned long long ok = __ballot(scan_from + lane < nscan && ahead_gap <= thr_max);
                        nxt = ok ? scan_from + __builtin_ctzll(ok) : next_scan(scan_from + 64, thr_max);
                    } else {
                        nxt = next_scan(scan_from, thr_max);
                    }
                    scan_from = nxt + 1;
                    tile_after = tile_of(nxt);
                    if (tile_after < ntiles) gload(tile_after, 0);
                    if (prune) ahead_gap = scan_from + lane < nscan ? gap_of(scan_tile(scan_from + lane)) : __builtin_nanf("");
                    __builtin_amdgcn_sched_barrier(0);
                    PHASE_MARK(4);
                }
                if (chunk == 0) {
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
#pragma unroll
                        for (int g = 0; g < 4; ++g) {
                            const v4f h = *reinterpret_cast<const v4f*>(hcs + b * 32 + 8 * g + 4 * lhalf);
                            acc[b][4 * g + 0] = h[0];
                            acc[b][4 * g + 1] = h[1];
                            acc[b][4 * g + 2] = h[2];
                            acc[b][4 * g + 3] = h[3];
                        }
                    }
                }
                if (SPLIT) {
                    // x_c . x_q ~ hi_c hi_q + hi_c lo_q + lo_c hi_q, 16 columns per instruction.
                    // All LDS reads of a group of multiplies are issued before the first of them, into registers of
                    // their own, and a scheduling fence keeps them there: left to itself the scheduler saves
                    // registers by reading each fragment just before the multiply that needs it, which exposes
                    // one LDS round trip per multiply or two (the sweep then runs at the speed of the LDS latency,
                    // not of either pipe).
#if SLHC_SPLIT_FRAGS == 2
                    v8bf ch[2][4], cl[2][4];
#pragma unroll
                    for (int s2 = 0; s2 < 2; ++s2) {
#pragma unroll
                        for (int b = 0; b < 4; ++b)
                            ch[s2][b] = __builtin_bit_cast(v8bf, *reinterpret_cast<const v4f*>(Cb + (b * 32 + l32) * LDK + 4 * (2 * s2 + lhalf)));
#pragma unroll
                        for (int b = 0; b < 4; ++b)
                            cl[s2][b] = __builtin_bit_cast(v8bf, *reinterpret_cast<const v4f*>(Cb + (b * 32 + l32) * LDK + 4 * (2 * s2 + lhalf) + 16));
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int s2 = 0; s2 < 2; ++s2) {
                        const v8bf qh = __builtin_bit_cast(v8bf, qf[chunk * 4 + s2]);
                        const v8bf ql = __builtin_bit_cast(v8bf, qf[chunk * 4 + 2 + s2]);
#pragma unroll
                        for (int b = 0; b < 4; ++b) acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ch[s2][b], qh, acc[b], 0, 0, 0);
#pragma unroll
                        for (int b = 0; b < 4; ++b) acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ch[s2][b], ql, acc[b], 0, 0, 0);
#pragma unroll
                        for (int b = 0; b < 4; ++b) acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cl[s2][b], qh, acc[b], 0, 0, 0);
                    }
#else
#pragma unroll
                    for (int s2 = 0; s2 < 2; ++s2) {
                        v8bf ch[4], cl[4];
#pragma unroll
                        for (int b = 0; b < 4; ++b)
                            ch[b] = __builtin_bit_cast(v8bf, *reinterpret_cast<const v4f*>(Cb + (b * 32 + l32) * LDK + 4 * (2 * s2 + lhalf)));
#pragma unroll
                        for (int b = 0; b < 4; ++b)
                            cl[b] = __builtin_bit_cast(v8bf, *reinterpret_cast<const v4f*>(Cb + (b * 32 + l32) * LDK + 4 * (2 * s2 + lhalf) + 16));
                        __builtin_amdgcn_sched_barrier(0);
                        const v8bf qh = __builtin_bit_cast(v8bf, qf[chunk * 4 + s2]);
                        const v8bf ql = __builtin_bit_cast(v8bf, qf[chunk * 4 + 2 + s2]);
#pragma unroll
                        for (int b = 0; b < 4; ++b) acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ch[b], qh, acc[b], 0, 0, 0);
#pragma unroll
                        for (int b = 0; b < 4; ++b) acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ch[b], ql, acc[b], 0, 0, 0);
#pragma unroll
                        for (int b = 0; b < 4; ++b) acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cl[b], qh, acc[b], 0, 0, 0);
                        __builtin_amdgcn_sched_barrier(0);
                    }
#endif
                } else {
#pragma unroll
                for (int kk = 0; kk < KC / 8; ++kk) {
                    v4f cf[4];
#pragma unroll
                    for (int b = 0; b < 4; ++b)
                        cf[b] = *reinterpret_cast<const v4f*>(Cb + (b * 32 + l32) * LDK + kk * 8 + 4 * lhalf);
                    const v4f q = qf[chunk * 4 + kk];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
#pragma unroll
                        for (int b = 0; b < 4; ++b)
                            acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(cf[b][e], q[e], acc[b], 0, 0, 0);
                    }
                }
                }
                // Nothing that consumes the loads issued at the top of this chunk may move up into its
                // multiplies: the chunks are unrolled, and the scheduler otherwise hoists the select that
                // prepares the next chunk's LDS stores to just behind the first multiply, where it has
                // to wait out the whole memory latency with 63 multiplies still to issue.
#ifndef SLHC_STUDY_NO_CHUNK_FENCE
                __builtin_amdgcn_sched_barrier(0);
#endif
            }

            // ---- first tile of a 1-NN panel: seed the thresholds (see seed_block) ----
            if (k == 1 && step == 0 && !lists_in) {
                const int seed_tag = MASKED ? my_qcol : (p.exclude_self ? my_qrow : -1);
                SeedPick pick{-__builtin_inff(), -1};
                pick = seed_block<KL, MASKED>(acc[0], 0, pick, seed_tag, col0, tpar, N);
                pick = seed_block<KL, MASKED>(acc[1], 1, pick, seed_tag, col0, tpar, N);
                pick = seed_block<KL, MASKED>(acc[2], 2, pick, seed_tag, col0, tpar, N);
                pick = seed_block<KL, MASKED>(acc[3], 3, pick, seed_tag, col0, tpar, N);
                seed_resolve<KL, true>(pick, col0, Xq, Xc, p.c_id, d, k);
                bound = bounds[my_q_local];
                if (prune) refresh_wave_thr();     // the tile may leave no survivor to do it below
            }
            // ---- tile epilogue: filter (hot), then compact / re-evaluate / select (rare) ----
            PHASE_MARK(3);
            const float own_bound = bound;
            if (shared_thr) bound = fmaxf(bound, hqs[my_q_local] - 0.5f * thr_c);
            unsigned int flagged = 0;
            int hits = 0;                  // pruned sweeps: lanes that hold a passing pair, over the four blocks
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                // Every-tile sweeps: one fused test (a tile of random rows nearly always holds near rows of
                // the query's own component, so a distance-only pre-test would rarely save the colour
                // test).  Pruned sweeps skip the tiles of the panel's own colour, and what is left is
                // mostly far: distances first, colours only in a block where some accumulator passes.
                bool any = false;
                if (MASKED && !PRUNE) {
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int4 cc = *reinterpret_cast<const int4*>(ccol + b * 32 + 8 * g + 4 * lhalf);
                        any |= (acc[b][4 * g + 0] >= bound) & (cc.x != my_qcol);
                        any |= (acc[b][4 * g + 1] >= bound) & (cc.y != my_qcol);
                        any |= (acc[b][4 * g + 2] >= bound) & (cc.z != my_qcol);
                        any |= (acc[b][4 * g + 3] >= bound) & (cc.w != my_qcol);
                    }
                } else {
#pragma unroll
                    for (int r = 0; r < 16; ++r) any |= (acc[b][r] >= bound);
                    if (MASKED && __any(any)) {
                        any = false;
#pragma unroll
                        for (int g = 0; g < 4; ++g) {
                            const int4 cc = *reinterpret_cast<const int4*>(ccol + b * 32 + 8 * g + 4 * lhalf);
                            any |= (acc[b][4 * g + 0] >= bound) & (cc.x != my_qcol);
                            any |= (acc[b][4 * g + 1] >= bound) & (cc.y != my_qcol);
                            any |= (acc[b][4 * g + 2] >= bound) & (cc.z != my_qcol);
                            any |= (acc[b][4 * g + 3] >= bound) & (cc.w != my_qcol);
                        }
                    }
                }
                const unsigned long long hit = __ballot(any);
                if (hit) flagged |= 1u << b;
                if (PRUNE) hits += __popcll(hit);
            }
            PHASE_MARK(5);
            if (__builtin_expect(flagged != 0, 0)) {
                // the rare path is a chain of short dependent steps: let it issue ahead of the
                // multiplies of the other workgroup's wavefront on this SIMD (measured: 0.8 %)
                __builtin_amdgcn_s_setprio(1);
                const int my_tag = MASKED ? my_qcol : (p.exclude_self ? my_qrow : -1);
                if (BATCHED) {
                    // First tile of a k-NN panel (k > 1): fill the lists from its best candidates (see
                    // seed_range).  Later tiles were tried too and gain nothing: what passes there are
                    // mostly real list updates.
                    if (!MASKED && k > 1 && step == 0 && !lists_in) {
                        SeedRange range{__builtin_inff(), -__builtin_inff()};
                        range = seed_range(acc[0], range);
                        range = seed_range(acc[1], range);
                        range = seed_range(acc[2], range);
                        range = seed_range(acc[3], range);
                        const int want = (k >> 1) + 1;
                        for (int it = 0; it < 12; ++it) {
                            const float mid = 0.5f * (range.lo + range.hi);
                            const int reach = seed_count(acc[0], mid) + seed_count(acc[1], mid) +
                                              seed_count(acc[2], mid) + seed_count(acc[3], mid);
                            if (reach >= want) range.lo = mid; else range.hi = mid;
                        }
                        float provisional = range.lo;                       // +inf when the lane has no candidate
                        provisional = fminf(provisional, __shfl_xor(provisional, 32));
                        {
                            // every pair that reaches the provisional bound, whatever the lists hold meanwhile
                            // (the bound is not refreshed between blocks: the masking below relies on it)
                            const int seed_tag = p.exclude_self ? my_qrow : -1;
                            const float reach_bound = fmaxf(bound, provisional);
                            int queued = 0;
#pragma unroll
                            for (int b = 0; b < 4; ++b) {
                                int r = wave_uniform(compact_block<KL, MASKED>(acc[b], b, reach_bound, seed_tag, col0, tpar, N, queued));
                                if (r < 0) {                                 // queue full: resolve, then this block alone
                                    survivors += (unsigned int)queued;
                                    resolve_queue<KL, true>(queued, col0, Xq, Xc, p.c_id, d, k);
                                    r = wave_uniform(compact_block<KL, MASKED>(acc[b], b, reach_bound, seed_tag, col0, tpar, N, 0));
                                }
                                queued = r;
                            }
                            if (queued > 0) {
                                survivors += (unsigned int)queued;
                                resolve_queue<KL, true>(queued, col0, Xq, Xc, p.c_id, d, k);
                            }
                            bound = bounds[my_q_local];
                        }
#pragma unroll
                        for (int b = 0; b < 4; ++b) {
#pragma unroll
                            for (int r = 0; r < 16; ++r)
                                acc[b][r] = (acc[b][r] >= provisional) ? -__builtin_inff() : acc[b][r];
                        }
                        refresh_wave_thr();
                    }
                    // A pruned 1-NN sweep only multiplies near tiles, where a query can have dozens of
                    // candidates below its threshold at once: evaluate the most promising one per lane
                    // first (as in the first tile), so that the compaction below runs under the
                    // threshold it leaves and only the close contenders are re-evaluated.
                    if (k == 1 && step > 0 && hits >= SEED_AGAIN_LANES) {
                        SeedPick pick{-__builtin_inff(), -1};
                        pick = seed_block<KL, MASKED>(acc[0], 0, pick, my_tag, col0, tpar, N);
                        pick = seed_block<KL, MASKED>(acc[1], 1, pick, my_tag, col0, tpar, N);
                        pick = seed_block<KL, MASKED>(acc[2], 2, pick, my_tag, col0, tpar, N);
                        pick = seed_block<KL, MASKED>(acc[3], 3, pick, my_tag, col0, tpar, N);
                        if (!(pick.v >= bound)) pick.cl = -1;
                        seed_resolve<KL, true>(pick, col0, Xq, Xc, p.c_id, d, k);
                        bound = bounds[my_q_local];
                        if (shared_thr) bound = fmaxf(bound, hqs[my_q_local] - 0.5f * thr_c);
                    }
                    const int colbuf_ = tpar;
                    SLHC_SELECT_TILE(KL, MASKED, true);
                    if (shared_thr) bound = bounds[my_q_local];         // this query's own bound again
                    if constexpr (KL == 1 && MASKED) {
                        if (lowering) {
                            // the lightest exact edge any query of this wavefront holds now
                            unsigned int best = my_qrow >= 0 ? (unsigned int)(mylists[l32] >> 32) : 0x7f800000u;
#pragma unroll
                            for (int o = 16; o > 0; o >>= 1) {
                                const unsigned int other = (unsigned int)__shfl_xor((int)best, o);
                                best = other < best ? other : best;
                            }
                            // the word is lowered to `lower_factor` times that edge, not to the edge itself (see SweepParams)
                            const float target = p.comp_lower_factor * __uint_as_float(best);
                            if (target < thr_c) {
                                if (lane == 0) atomicMin(p.comp_best_lower + panel_colour, __float_as_uint(target));
                                thr_c = target;
                            }
                        }
                    }
                } else {
                    // few survivors: queue them for a later batch.  Blocks with many (the first tiles
                    // of a panel) are resolved at once afterwards, behind what already waits; their
                    // calls sit apart so that the common sequence keeps the accumulators in registers.
                    unsigned int heavy = 0;
                    if ((flagged & 1u) && defer_block<KL, MASKED>(acc[0], 0, bound, my_tag, col0, tpar, N) < 0) heavy |= 1u;
                    if ((flagged & 2u) && defer_block<KL, MASKED>(acc[1], 1, bound, my_tag, col0, tpar, N) < 0) heavy |= 2u;
                    if ((flagged & 4u) && defer_block<KL, MASKED>(acc[2], 2, bound, my_tag, col0, tpar, N) < 0) heavy |= 4u;
                    if ((flagged & 8u) && defer_block<KL, MASKED>(acc[3], 3, bound, my_tag, col0, tpar, N) < 0) heavy |= 8u;
                    PHASE_MARK(1);
                    int waiting_ = wave_uniform(*deferred_count(L, wave));
                    if (__builtin_expect(heavy != 0, 0)) {
                        if (waiting_ > 0) { survivors += (unsigned int)waiting_; resolve_deferred<KL, true>(waiting_, Xq, Xc, p.c_id, d, k); }
                        waiting_ = 0;
                        const unsigned int all_flagged = flagged;
                        flagged = heavy;
                        const int colbuf_ = tpar;
                        SLHC_SELECT_TILE(KL, MASKED, true);
                        flagged = all_flagged;
                    }
                    (void)waiting_;
                    bound = bounds[my_q_local];
                }
                __builtin_amdgcn_s_setprio(0);
                if (prune) refresh_wave_thr();
            }
            if (!BATCHED) {
                // Deferred pairs are resolved by all four wavefronts in the same step: a wavefront in the
                // rare path keeps the other three waiting at the next barrier, so four queues that fill
                // and resolve at different steps stall the workgroup four times as often as queues
                // that resolve together.  Every wavefront publishes its queue length at the end of a step
                // (slots alternate with the step parity, like the threshold slots of the pruned sweeps,
                // which these sweeps do not use); in the next step all of them read the same four
                // lengths and resolve what they hold as soon as one queue has reached DEFER_MIN.
                const int4 lens = *reinterpret_cast<const int4*>(reinterpret_cast<const int*>(L.wmax) + (tpar ^ 1) * 4);
                const int longest = max(max(lens.x, lens.y), max(lens.z, lens.w));
                int waiting_ = wave_uniform(*deferred_count(L, wave));
                if (__builtin_expect(longest >= DEFER_MIN, 0) && waiting_ > 0) {
                    __builtin_amdgcn_s_setprio(1);
                    survivors += (unsigned int)waiting_;
                    resolve_deferred<KL, true>(waiting_, Xq, Xc, p.c_id, d, k);
                    bound = bounds[my_q_local];
                    waiting_ = 0;
                    __builtin_amdgcn_s_setprio(0);
                }
                if (lane == 0) reinterpret_cast<int*>(L.wmax)[tpar * 4 + wave] = waiting_;
            }
            if (shared_thr && flagged == 0) bound = own_bound;
            if (CAN_SPLIT && nparts > 1) {
                // Exchange with the other parts of the panel through p.out_key: publish this query's entry when
                // it has improved, adopt the word read a step ago when it is better (its read has had a whole
                // step to arrive), and read it again for the next step.
                bool adopted = false;
                if (lhalf == 0 && my_qrow >= 0) {
                    const unsigned long long mine = mylists[l32];
                    if (mine < part_published) { atomicMin(p.out_key + part_slot, mine); part_published = mine; }
                    if (part_seen < mine) {
                        mylists[l32] = part_seen;
                        bounds[my_q_local] = hqs[my_q_local] - 0.5f * __uint_as_float((unsigned int)(part_seen >> 32));
                        part_published = part_seen;
                        adopted = true;
                    }
                    part_seen = __hip_atomic_load(p.out_key + part_slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                if (__any(adopted)) {
                    __builtin_amdgcn_wave_barrier();
                    bound = bounds[my_q_local];
                    if (prune) refresh_wave_thr();
                }
            }
            PHASE_MARK(6);
            // (with a falling component threshold: no query of this wavefront can use a candidate beyond it)
            if (prune && lane == 0) L.wmax[tpar * 4 + wave] = lowering ? fminf(wave_thr_max, thr_c) : wave_thr_max;
            ++tiles_done;
            ++step;
            tile = tile_after;
        }

#ifdef SLHC_STUDY_PANEL_STEPS
        if (p.panel_steps && tid == 0) { atomicAdd(p.panel_steps + panel, step); atomicMax(p.panel_steps + npanels + panel, (int)((clock64() - study_t0) >> 10)); }
#endif
        // ---- panel epilogue: lists are already ascending; write them out ----
        if (!BATCHED) {
            const int waiting_ = wave_uniform(*deferred_count(L, wave));
            if (waiting_ > 0) { survivors += (unsigned int)waiting_; resolve_deferred<KL, true>(waiting_, Xq, Xc, p.c_id, d, k); }
        }
        __builtin_amdgcn_wave_barrier();
        for (int ql = 0; ql < 32; ++ql) {
            const int row = qid[wave * 32 + ql];
            if (row < 0) continue;
            if (lane < k) {
                const unsigned long long key = mylists[(size_t)ql * KL + lane];
                const float dist = __uint_as_float((unsigned int)(key >> 32));
                int idx = (int)(unsigned int)(key & 0xffffffffull);
                if (key == LIST_SENTINEL) idx = -1;
                const size_t o = MASKED ? (size_t)(aligned ? p.qslot[row] : panel * BM + wave * 32 + ql)
                                        : (size_t)(p.q_out_row ? p.q_out_row[row] : row) * k + lane;
                if (CAN_SPLIT && nparts > 1) {
                    if (key != LIST_SENTINEL) atomicMin(p.out_key + o, key);      // the parts of a panel meet here
                } else if (CAN_RANGE && nparts > 1) {
                    const size_t po = ((size_t)part * (size_t)p.NQ + (size_t)row) * k + lane;
                    p.part_idx[po] = idx;
                    p.part_dist[po] = dist;
                } else {
                    p.out_idx[o] = idx;
                    p.out_dist[o] = dist;
                }
            }
        }
        if (CAN_CARRY && ncarry > 1) {
            // the lists of this range are written: let item (crange + 1, panel) start from them.  Every thread
            // waits for its own stores to be acknowledged (workgroup-scope release), the barrier collects that, and
            // one thread alone makes them visible to the other XCDs and raises the word (an agent-scope release
            // in every thread would have each of them write back the L2).
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            __syncthreads();
            if (tid == 0) __hip_atomic_store(p.carry_ws + 2 + panel, (unsigned int)(crange + 1), __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        }
        PHASE_MARK(7);
    }
#ifdef SLHC_PHASE_TIMERS
    if (p.phase_cycles && tid == 0)
        for (int i = 0; i < 8; ++i) atomicAdd(p.phase_cycles + i, ph[i]);
#endif
    if (p.survivors && lane == 0 && survivors) atomicAdd(p.survivors, survivors);
    if (p.tiles_done && tid == 0 && tiles_done) atomicAdd(p.tiles_done, tiles_done);
}

// ------------------------------------------------------------------------------- launchers
// Compute units of the current device (asked on every call: the answer belongs to the device
// that is current now, and the runtime answers from its own cache).
static hipError_t device_cus(int* cus)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    int v = 0;
    e = hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return e;
    *cus = v > 0 ? v : 1;
    return hipSuccess;
}

// Register-only fp32 MFMA loop: every wavefront chains v_mfma_f32_32x32x2_f32 on four independent
// accumulator blocks (the instruction and the accumulator count of the sweep kernels) with operands that
// never leave registers.  What it sustains is the rate the chip holds at its clocks under this load: the
// practical ceiling of the distance tiles, next to the published peak.
__global__ void __launch_bounds__(WG_THREADS, 2) mfma_probe_kernel(int iters, float seed, float* __restrict__ sink)
{
    v16f acc[4];
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[b][r] = 0.f;
    float a = seed + (float)(threadIdx.x & 7) * 1e-3f, c = seed * 0.5f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
#pragma unroll
            for (int b = 0; b < 4; ++b) acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, c, acc[b], 0, 0, 0);
        }
    }
    float total = 0.f;
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) total += acc[b][r];
    if (total == 123456.789f) sink[0] = total;          // keeps the chain alive; practically never taken
}

// The same for the multiply of the split-product sweeps, v_mfma_f32_32x32x16_bf16.
__global__ void __launch_bounds__(WG_THREADS, 2) mfma_bf16_probe_kernel(int iters, float seed, float* __restrict__ sink)
{
    v16f acc[4];
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[b][r] = 0.f;
    v8bf a, c;
#pragma unroll
    for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(seed + (float)((threadIdx.x + e) & 7) * 0.125f); c[e] = (__bf16)(seed * 0.5f); }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
#pragma unroll
            for (int b = 0; b < 4; ++b) acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, c, acc[b], 0, 0, 0);
        }
    }
    float total = 0.f;
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) total += acc[b][r];
    if (total == 123456.789f) sink[0] = total;
}

// One v_mfma_f32_32x32x16_bf16 per trial on caller-given values: D[t] = C[t] + sum_k A[t][k] B[t][k], k < 16, the
// values rounded to bfloat16 first (pass bfloat16-representable ones).  For checking the rounding behaviour that
// split_slack_coefficient relies on against an exact sum computed elsewhere.
__global__ void __launch_bounds__(64) mfma_bf16_values_kernel(const float* __restrict__ A, const float* __restrict__ B,
                                                              const float* __restrict__ C, float* __restrict__ D, int trials)
{
    const int t = blockIdx.x, lane = threadIdx.x;
    if (t >= trials) return;
    v8bf a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        a[e] = (__bf16)A[(size_t)t * 16 + 8 * (lane >> 5) + e];
        b[e] = (__bf16)B[(size_t)t * 16 + 8 * (lane >> 5) + e];
    }
    v16f acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = C[t];
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
    if (lane == 0) D[t] = acc[0];
}

hipError_t launch_mfma_bf16_values(const float* A, const float* B, const float* C, float* D, int trials, hipStream_t stream)
{
    if (trials < 1) return hipSuccess;
    hipLaunchKernelGGL(mfma_bf16_values_kernel, dim3(trials), dim3(64), 0, stream, A, B, C, D, trials);
    return hipGetLastError();
}

hipError_t launch_mfma_bf16_probe(int iters, float* sink, hipStream_t stream, double* flop)
{
    int cus = 0;
    hipError_t e = device_cus(&cus);
    if (e != hipSuccess) return e;
    const int grid = 2 * cus;
    hipLaunchKernelGGL(mfma_bf16_probe_kernel, dim3(grid), dim3(WG_THREADS), 0, stream, iters, 1.0f, sink);
    *flop = (double)grid * (WG_THREADS / 64) * (double)iters * 16.0 * (2.0 * 32 * 32 * 16);
    return hipGetLastError();
}

hipError_t launch_mfma_probe(int iters, float* sink, hipStream_t stream, double* flop)
{
    int cus = 0;
    hipError_t e = device_cus(&cus);
    if (e != hipSuccess) return e;
    const int grid = 2 * cus;
    hipLaunchKernelGGL(mfma_probe_kernel, dim3(grid), dim3(WG_THREADS), 0, stream, iters, 1.0f, sink);
    *flop = (double)grid * (WG_THREADS / 64) * (double)iters * 16.0 * (2.0 * 32 * 32 * 2);
    return hipGetLastError();
}

// The same multiplies with the ingredients of the sweep's panel loop added one by one (a measurement aid:
// which ingredient costs MFMA rate).  STEPS: 1 = a workgroup barrier per chunk of 64 multiplies and the A
// operands read from LDS (16 ds_read_b128 per chunk); 2 = also the next chunk of a 128-row candidate tile
// loaded from `stream` (rows of 128 floats, `rows` a power of two) into registers and stored to LDS, double
// buffered as in the sweep; 3 = also 16 compares and a ballot per accumulator block after every fourth
// chunk.  Nothing it computes means anything.
template <int STEPS, bool DIRECT, bool ASYM = false, bool BF16 = false>
__global__ void __launch_bounds__(WG_THREADS, 2) loop_probe_kernel(int iters, const float* __restrict__ stream,
                                                                   int rows, float* __restrict__ sink)
{
    // ASYM: the two wavefronts that share a SIMD (one of each resident workgroup) run at different priorities,
    // chosen by the parity of the wavefront's slot number on its SIMD (HW_ID bits 3:0)
    if (ASYM) {
        if (__builtin_amdgcn_s_getreg((3 << 11) | (0 << 6) | 4) & 1) __builtin_amdgcn_s_setprio(2);
    }
    // DIRECT: the candidate chunk goes from global memory straight into LDS (global_load_lds_dwordx4: lane l of a
    // wavefront fills the 16 bytes at base + 16 l), rows of 32 floats without padding, the 16-byte quads of row r
    // stored at position quad ^ (r & 7) so that the operand reads of 8 consecutive rows fall into different banks.
    constexpr int LDR = DIRECT ? KC : LDK;
    extern __shared__ __align__(16) unsigned char probe_smem[];
    float* buf0 = reinterpret_cast<float*>(probe_smem);
    float* buf1 = buf0 + BN * LDR;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, lhalf = lane >> 5;
    const int ld_row = DIRECT ? wave * 32 + (lane >> 3) : tid >> 3;
    const int ld_step = DIRECT ? 8 : 32;
    const int ld_col = DIRECT ? ((lane & 7) ^ (lane >> 3)) * 4 : (tid & 7) * 4;
    for (int i = tid; i < 2 * BN * LDR; i += WG_THREADS) buf0[i] = 1e-3f * (float)(i & 15);
    __syncthreads();
    v16f acc[4];
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[b][r] = 0.f;
    v4f q[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) q[kk] = v4f{1.f + lane * 1e-3f, 0.5f, 0.25f, 0.125f};
    v4f creg[4];
    unsigned int row = ((unsigned int)blockIdx.x * BN + ld_row) & (unsigned int)(rows - 1);
    unsigned int flagged = 0;
    const float bound = 1e30f;
    auto stage = [&](float* dst, int col) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float* src = stream + (size_t)((row + ld_step * i) & (rows - 1)) * 128 + col;
            if (DIRECT)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src),
                                                 (__attribute__((address_space(3))) void*)(dst + (wave * 32 + 8 * i) * LDR),
                                                 16, 0, 0);
            else
                creg[i] = *reinterpret_cast<const v4f*>(src);
        }
    };
    if (STEPS >= 2) stage(buf0, ld_col);
    for (int it = 0; it < iters; ++it) {
        float* Cb = (it & 1) ? buf1 : buf0;
        if (STEPS >= 2 && !DIRECT) {
#pragma unroll
            for (int i = 0; i < 4; ++i) *reinterpret_cast<v4f*>(Cb + (ld_row + 32 * i) * LDR + ld_col) = creg[i];
        }
        if (STEPS >= 2 && DIRECT) __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0): this wavefront's part of the chunk is in LDS
        __syncthreads();
        if (STEPS >= 2) {
            row = (row + BN) & (unsigned int)(rows - 1);
            stage((it & 1) ? buf0 : buf1, ((it + 1) & 3) * KC + ld_col);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (BF16) {
            // the multiplies of the split-product sweeps: 16 LDS reads (hi and lo fragments), 24 bf16 multiplies
            v8bf ch[2][4], cl[2][4];
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    ch[s2][b] = __builtin_bit_cast(v8bf, *reinterpret_cast<const v4f*>(Cb + (b * 32 + l32) * LDR + 4 * (2 * s2 + lhalf)));
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    cl[s2][b] = __builtin_bit_cast(v8bf, *reinterpret_cast<const v4f*>(Cb + (b * 32 + l32) * LDR + 4 * (2 * s2 + lhalf) + 16));
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                const v8bf qh = __builtin_bit_cast(v8bf, q[s2]), ql = __builtin_bit_cast(v8bf, q[2 + s2]);
#pragma unroll
                for (int b = 0; b < 4; ++b) acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ch[s2][b], qh, acc[b], 0, 0, 0);
#pragma unroll
                for (int b = 0; b < 4; ++b) acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ch[s2][b], ql, acc[b], 0, 0, 0);
#pragma unroll
                for (int b = 0; b < 4; ++b) acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cl[s2][b], qh, acc[b], 0, 0, 0);
            }
        } else
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            v4f cf[4];
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int quad = kk * 2 + lhalf;
                cf[b] = *reinterpret_cast<const v4f*>(Cb + (b * 32 + l32) * LDR + (DIRECT ? (quad ^ (l32 & 7)) * 4 : quad * 4));
            }
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int b = 0; b < 4; ++b) acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(cf[b][e], q[kk][e], acc[b], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (STEPS >= 3 && (it & 3) == 3) {
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                bool any = false;
#pragma unroll
                for (int r = 0; r < 16; ++r) any |= acc[b][r] >= bound;
                if (__any(any)) flagged |= 1u << b;
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[b][r] = -1.0f;
            }
        }
    }
    if (STEPS >= 2 && DIRECT) __builtin_amdgcn_s_waitcnt(0x0f70);
    float total = (float)flagged;
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) total += acc[b][r];
    if (total == 123456.789f) sink[0] = total;
}

hipError_t launch_loop_probe(int steps, int iters, const float* stream_rows, int rows, float* sink, hipStream_t stream,
                             double* flop)
{
    if (steps <= 0) return launch_mfma_probe(iters * 4, sink, stream, flop);     // 16 multiplies per iteration there
    if (steps == 8) return launch_mfma_bf16_probe(iters * 2, sink, stream, flop);
    int cus = 0;
    hipError_t e = device_cus(&cus);
    if (e != hipSuccess) return e;
    const int grid = 2 * cus;
    const size_t lds = 80000;              // the two chunk buffers need 36 864 B; this size admits two workgroups per CU, like the sweep
    auto run = [&](auto kernel) -> hipError_t {
        hipError_t e2 = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e2 != hipSuccess) return e2;
        hipLaunchKernelGGL(kernel, dim3(grid), dim3(WG_THREADS), lds, stream, iters, stream_rows, rows, sink);
        return hipGetLastError();
    };
    if (steps >= 9) {          // 9..11: steps 1..3 with the 24 bf16 multiplies of a split-product chunk
        *flop = (double)grid * (WG_THREADS / 64) * (double)iters * 24.0 * (2.0 * 32 * 32 * 16);
        if (steps == 9) return run(&loop_probe_kernel<1, false, false, true>);
        if (steps == 10) return run(&loop_probe_kernel<2, false, false, true>);
        return run(&loop_probe_kernel<3, false, false, true>);
    }
    *flop = (double)grid * (WG_THREADS / 64) * (double)iters * 64.0 * (2.0 * 32 * 32 * 2);
    if (steps == 1) return run(&loop_probe_kernel<1, false>);
    if (steps == 2) return run(&loop_probe_kernel<2, false>);
    if (steps == 3) return run(&loop_probe_kernel<3, false>);
    if (steps == 4) return run(&loop_probe_kernel<2, true>);      // 2 and 3 with the chunk loaded straight into LDS
    if (steps == 5) return run(&loop_probe_kernel<3, true>);
    if (steps == 6) return run(&loop_probe_kernel<2, false, true>);   // 2 and 3 with unequal wavefront priorities
    return run(&loop_probe_kernel<3, false, true>);
}

float filter_slack_coefficient(int d)
{
    // The accumulator is a chain of d+1 round-to-nearest fused multiply-adds whose partial sums
    // are bounded by ||x_q||^2 + ||x_c||^2, so it is off by at most (d+1) 2^-24 (n_q + n_c);
    // the filter has c (n_q + n_c)/2 of slack.  c = (d+8) 2^-23 covers that chain plus the
    // roundings of the norms, of h and of the bound.
    return (float)(d + 8) * 1.1920928955078125e-07f;
}

float split_slack_coefficient(int d)
{
    // x = hi + lo + r with |r| <= 2^-16 |x| (two roundings to 8 significant bits).  The accumulated sum
    // hi_c hi_q + hi_c lo_q + lo_c hi_q leaves out lo_c lo_q and the r terms: at most 3 * 2^-16 |x_c x_q| per
    // column, i.e. 3 * 2^-16 (n_q + n_c) / 2 per pair.  Its products are exact in float32 and there are 3 d of
    // them to accumulate, counted like the d of filter_slack_coefficient.
    // The split copy holds the rows fl(x - shift) (split_bf16_kernel).  A translation changes no distance, but its
    // rounding moves each of the two rows by at most 2^-24 of its length, i.e. the squared distance by at most
    // 2^-23 (|u| + |v|)^2 <= 2^-22 (n_q + n_c): two more units, and two to spare.
    return 3.0f * 1.52587890625e-05f + (float)(3 * d + 12) * 1.1920928955078125e-07f;
}

// one thread per 8 columns: hi = bf16(x), lo = bf16(x - hi), both rounded to nearest even.  A row of the split
// copy holds whole chunks of 32 columns (stride = d rounded up to a multiple of 32 words); columns past d are 0.
// `shift` (optional, [d]): the copy holds fl(x - shift) instead of x.  The sweeps' products only feed the filter, a
// distance does not change when both rows are translated, and the filter's slack is a fraction of the rows' squared
// norms: with the column means taken off, a common offset of the data no longer counts towards it.
__global__ void __launch_bounds__(256) split_bf16_kernel(const float* __restrict__ X, long long octets, int d, int stride,
                                                         float* __restrict__ Xsplit, const float* __restrict__ shift_,
                                                         const int* __restrict__ shift_tile)
{
    const long long o = (long long)blockIdx.x * 256 + threadIdx.x;
    if (o >= octets) return;
    const int per_row = stride >> 3;
    const long long row = o / per_row;
    const int oct = (int)(o - row * per_row);              // columns 8 oct .. 8 oct + 7
    const int chunk = oct >> 2, piece = oct & 3;
    const float* src = X + row * d + 8 * oct;
    v4f a = {0.f, 0.f, 0.f, 0.f}, b = {0.f, 0.f, 0.f, 0.f};
    if (8 * oct + 4 <= d) a = *reinterpret_cast<const v4f*>(src);          // d is a multiple of 4
    if (8 * oct + 8 <= d) b = *reinterpret_cast<const v4f*>(src + 4);
    if (shift_) {
        const float* shift = shift_tile ? shift_ + (size_t)shift_tile[row >> 7] * d : shift_;
        if (8 * oct + 4 <= d) a -= *reinterpret_cast<const v4f*>(shift + 8 * oct);
        if (8 * oct + 8 <= d) b -= *reinterpret_cast<const v4f*>(shift + 8 * oct + 4);
    }
    v8bf hi, lo;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float x = e < 4 ? a[e] : b[e - 4];
        const __bf16 h = (__bf16)x;
        hi[e] = h;
        lo[e] = (__bf16)(x - (float)h);
    }
    float* dst = Xsplit + row * stride + chunk * KC;       // chunk: 16 words of hi, 16 words of lo
    *reinterpret_cast<v4f*>(dst + 4 * piece) = __builtin_bit_cast(v4f, hi);
    *reinterpret_cast<v4f*>(dst + 16 + 4 * piece) = __builtin_bit_cast(v4f, lo);
}

int split_row_stride(int d) { return (d + KC - 1) / KC * KC; }

hipError_t launch_split_bf16(const float* X, int N, int d, float* Xsplit, hipStream_t stream, const float* shift,
                             const int* shift_tile)
{
    if (d % 4 != 0 || ((reinterpret_cast<uintptr_t>(X) | reinterpret_cast<uintptr_t>(Xsplit) | reinterpret_cast<uintptr_t>(shift)) & 15) != 0)
        return hipErrorInvalidValue;
    const int stride = split_row_stride(d);
    const long long octets = (long long)N * (stride >> 3);
    hipLaunchKernelGGL(split_bf16_kernel, dim3((unsigned int)((octets + 255) / 256)), dim3(256), 0, stream, X, octets, d, stride, Xsplit, shift, shift_tile);
    return hipGetLastError();
}

hipError_t launch_half_norms(const float* X, int N, int d, float* hn, hipStream_t stream, unsigned int* nonfinite,
                             bool split_slack, const float* shift, const int* shift_tile)
{
    const float scale = 0.5f * (1.0f - (split_slack ? split_slack_coefficient(d) : filter_slack_coefficient(d)));
    const long long threads = (long long)N * 16;
    const int blocks = (int)((threads + 255) / 256);
    const bool vec4 = (d % 4 == 0) && (((reinterpret_cast<uintptr_t>(X) | reinterpret_cast<uintptr_t>(shift)) & 15) == 0);
    if (vec4) hipLaunchKernelGGL(half_norm_kernel<true>, dim3(blocks), dim3(256), 0, stream, X, N, d, scale, hn, nonfinite, shift, shift_tile);
    else hipLaunchKernelGGL(half_norm_kernel<false>, dim3(blocks), dim3(256), 0, stream, X, N, d, scale, hn, nonfinite, shift, shift_tile);
    return hipGetLastError();
}

// A central value of every column, from a sample of at most MEAN_SAMPLE evenly spaced rows: the sample is cut into
// MEAN_PARTS runs, each run gives a mean, and the column's value is the median of those means (a plain mean follows
// a single far outlier, and a shift that follows it inflates every other row's norm).  Fixed order of additions: the
// same vector in every run.  Any vector serves as a shift: values that are not finite are left out, and a result
// that is not finite or beyond 2^50 is replaced by 0, so that taking it off a finite row overflows no sooner than
// the row's own norm does.
constexpr int MEAN_SAMPLE = 16384, MEAN_PARTS = 64;
__global__ void __launch_bounds__(256) column_sums_kernel(const float* __restrict__ X, int N, int d, int samples,
                                                          float* __restrict__ partial)
{
    const int c = blockIdx.y * 256 + threadIdx.x;
    if (c >= d) return;
    const int part = blockIdx.x;
    const int i0 = (int)((long long)part * samples / MEAN_PARTS), i1 = (int)((long long)(part + 1) * samples / MEAN_PARTS);
    float sum = 0.f;
    for (int i = i0; i < i1; i += 8) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {          // eight loads in flight; the additions keep their order
            const int iu = i + u < i1 ? i + u : i1 - 1;
            v[u] = X[((long long)iu * N / samples) * d + c];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (i + u < i1 && fabsf(v[u]) < __builtin_inff()) sum += v[u];          // false for NaN as well
    }
    partial[(size_t)part * d + c] = i1 > i0 ? sum / (float)(i1 - i0) : __builtin_nanf("");       // NaN: an empty run
}
// one wavefront per column: lane p holds the mean of run p and finds its rank among the valid ones by comparing with
// all 64 (ties broken by run number); the two middle ranks give the median
__global__ void __launch_bounds__(256) column_means_kernel(const float* __restrict__ partial, int d,
                                                           float* __restrict__ mean)
{
    static_assert(MEAN_PARTS == 64, "one lane per run");
    const int lane = threadIdx.x & 63;
    const int c = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int cc = c < d ? c : d - 1;                    // whole wavefronts stay in step; the surplus ones store nothing
    const float x = partial[(size_t)lane * d + cc];
    const bool valid = fabsf(x) < __builtin_inff();      // not an empty run, not a mean that overflowed
    const int n = __popcll(__ballot(valid));
    int rank = 0;
    for (int q = 0; q < 64; ++q) {
        const float y = __shfl(x, q);
        const bool yvalid = __shfl((int)valid, q) != 0;
        if (yvalid && (y < x || (y == x && q < lane))) ++rank;
    }
    float pick = 0.f;
    if (valid && n > 0) {
        if (rank == ((n - 1) >> 1)) pick += 0.5f * x;
        if (rank == (n >> 1)) pick += 0.5f * x;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) pick += __shfl_xor(pick, o);          // two non-zero terms at most: exact order is immaterial
    if (lane == 0 && c < d) mean[c] = fabsf(pick) <= 1.125899906842624e15f ? pick : 0.f;       // 2^50; false for NaN
}
size_t column_means_scratch_floats(int d) { return (size_t)MEAN_PARTS * (size_t)d; }
hipError_t launch_column_means(const float* X, int N, int d, float* scratch, float* mean, hipStream_t stream)
{
    if (N < 1 || d < 1) return hipErrorInvalidValue;
    const int samples = N < MEAN_SAMPLE ? N : MEAN_SAMPLE;
    const unsigned int cblocks = (unsigned int)((d + 255) / 256);
    hipLaunchKernelGGL(column_sums_kernel, dim3(MEAN_PARTS, cblocks), dim3(256), 0, stream, X, N, d, samples, scratch);
    hipLaunchKernelGGL(column_means_kernel, dim3((unsigned int)((d + 3) / 4)), dim3(256), 0, stream, scratch, d, mean);
    return hipGetLastError();
}

template <typename K>
static hipError_t launch_with_lds(K kernel, int grid, size_t lds, const SweepParams& p, hipStream_t stream)
{
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(WG_THREADS), lds, stream, p);
    return hipGetLastError();
}

__global__ void __launch_bounds__(256) zero_words_kernel(unsigned int* __restrict__ w, long long n)
{
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i < n) w[i] = 0u;
}

#ifndef SLHC_CARRY_RANGE_BYTES
#define SLHC_CARRY_RANGE_BYTES (32 << 20)
#endif
#ifndef SLHC_CARRY_MIN_ROUNDS
#define SLHC_CARRY_MIN_ROUNDS 4
#endif
// candidate bytes per range of a sweep that goes range by range: a small share of the 256 MiB memory-side cache, so
// that the range the workgroups are in and the one the first of them move on to both stay there.  (Ranges of 2 MiB,
// half of an XCD's L2, cut the fabric traffic five times but pay more per work item than they save: measured.)
constexpr long long CARRY_RANGE_BYTES = SLHC_CARRY_RANGE_BYTES;
// ... and only with at least this many panels per workgroup slot: a panel's item in range r + 1 is handed out
// that many rounds of items after its item in range r, which therefore has finished by then
constexpr int CARRY_MIN_ROUNDS = SLHC_CARRY_MIN_ROUNDS;

template <int KL, bool MASKED>
static hipError_t launch_sweep_t(const SweepParams& p_in, hipStream_t stream)
{
    SweepParams p = p_in;
    p.carry_ranges = 0;
    int cus = 0;
    hipError_t e = device_cus(&cus);
    if (e != hipSuccess) return e;
    const bool aligned = MASKED && p.qslot != nullptr;
    const int nq = (MASKED && !aligned) ? p.m : p.NQ;
    const int npanels = (nq + BM - 1) / BM;
    if (npanels < 1) return hipSuccess;
    const size_t lds = sweep_lds_bytes(KL);
    const int per_cu = lds * 2 <= 160 * 1024 ? 2 : 1;
    // candidate segments: the streaming kernel (no pruning); parts of a pruned scan: cross 1-NN with a slot map
    const bool ranges = !MASKED && p.k > 1 && p.segments > 1 && p.part_idx && p.part_dist && !p.tile_c;     // k-NN in candidate ranges
    if (p.segments > 1 && !ranges && (!p.out_key || p.k != 1 || (p.tile_c && !(MASKED && p.qslot)))) return hipErrorInvalidValue;
    const bool listed = MASKED && aligned && p.tile_c && p.panel_list;
    if (listed && p.panel_list_n < 1) return hipSuccess;
    const long long nitems = (long long)(listed ? p.panel_list_n : npanels) * (p.segments > 1 ? p.segments : 1);
    int grid = cus * per_cu;
    if (grid > nitems) grid = (int)nitems;
    const bool vec4 = (p.d % 4 == 0) && (((reinterpret_cast<uintptr_t>(p.Xq) | reinterpret_cast<uintptr_t>(p.Xc)) & 15) == 0);
    if (vec4 && p.d <= 4 * KC && (p.segments <= 1 || p.tile_c || ranges)) {
        // up to 128 features: query fragments live in registers
        const int dch = (p.d + KC - 1) / KC;
        if (p.tile_c) {
            if (!p.tile_r || !p.gap_ws) return hipErrorInvalidValue;
            if (p.Xq_split && p.Xc_split && p.hq_split && p.hc_split && p.d % KC == 0 && dch >= SLHC_SPLIT_MIN_CHUNKS_PRUNED &&
                (((reinterpret_cast<uintptr_t>(p.Xq_split) | reinterpret_cast<uintptr_t>(p.Xc_split)) & 15) == 0)) {
#if SLHC_SPLIT_MIN_CHUNKS_PRUNED < 2
                if (dch == 1) return launch_with_lds(&sweep_kernel_qreg<KL, MASKED, 1, true, true>, grid, lds, p, stream);
#endif
                if (dch == 2) return launch_with_lds(&sweep_kernel_qreg<KL, MASKED, 2, true, true>, grid, lds, p, stream);
                if (dch == 3) return launch_with_lds(&sweep_kernel_qreg<KL, MASKED, 3, true, true>, grid, lds, p, stream);
                return launch_with_lds(&sweep_kernel_qreg<KL, MASKED, 4, true, true>, grid, lds, p, stream);
            }
            if (dch == 1) return launch_with_lds(&sweep_kernel_qreg<KL, MASKED, 1, true>, grid, lds, p, stream);
            if (dch == 2) return launch_with_lds(&sweep_kernel_qreg<KL, MASKED, 2, true>, grid, lds, p, stream);
            if (dch == 3) return launch_with_lds(&sweep_kernel_qreg<KL, MASKED, 3, true>, grid, lds, p, stream);
            return launch_with_lds(&sweep_kernel_qreg<KL, MASKED, 4, true>, grid, lds, p, stream);
        }
        if (p.qslot || p.tile_colour || p.panel_counter || p.own_tile_first) return hipErrorInvalidValue;
        if (p.carry_ws && p.segments <= 1 && npanels >= (long long)CARRY_MIN_ROUNDS * cus * per_cu &&
            p.carry_ws_words >= 2 + (long long)npanels) {
            const int ntiles = (p.NC + BN - 1) / BN;
            long long per_range = CARRY_RANGE_BYTES / ((long long)BN * p.d * 4);
            if (per_range < 4) per_range = 4;
            long long ranges = (ntiles + per_range - 1) / per_range;
            while (ranges * npanels >= (1LL << 30)) ranges = (ranges + 1) / 2;       // work items are counted in an int
            if (ranges >= 2) {
                p.carry_ranges = (int)ranges;
                const long long words = 2 + (long long)npanels;
                hipLaunchKernelGGL(zero_words_kernel, dim3((unsigned int)((words + 255) / 256)), dim3(256), 0, stream, p.carry_ws, words);
                e = hipGetLastError();
                if (e != hipSuccess) return e;
                grid = cus * per_cu;
            }
        }
        if (p.Xq_split && p.Xc_split && p.hq_split && p.hc_split && p.d % KC == 0 && dch >= SLHC_SPLIT_MIN_CHUNKS &&
            (((reinterpret_cast<uintptr_t>(p.Xq_split) | reinterpret_cast<uintptr_t>(p.Xc_split)) & 15) == 0)) {
#if SLHC_SPLIT_MIN_CHUNKS < 2
            if (dch == 1) return launch_with_lds(&sweep_kernel_qreg<KL, MASKED, 1, false, true>, grid, lds, p, stream);
#endif
            if (dch == 2) return launch_with_lds(&sweep_kernel_qreg<KL, MASKED, 2, false, true>, grid, lds, p, stream);
            if (dch == 3) return launch_with_lds(&sweep_kernel_qreg<KL, MASKED, 3, false, true>, grid, lds, p, stream);
            return launch_with_lds(&sweep_kernel_qreg<KL, MASKED, 4, false, true>, grid, lds, p, stream);
        }
        if (dch == 1) return launch_with_lds(&sweep_kernel_qreg<KL, MASKED, 1, false>, grid, lds, p, stream);
        if (dch == 2) return launch_with_lds(&sweep_kernel_qreg<KL, MASKED, 2, false>, grid, lds, p, stream);
        if (dch == 3) return launch_with_lds(&sweep_kernel_qreg<KL, MASKED, 3, false>, grid, lds, p, stream);
        return launch_with_lds(&sweep_kernel_qreg<KL, MASKED, 4, false>, grid, lds, p, stream);
    }
    // tile pruning and the slot map exist in the register-resident-query variant only
    if (p.tile_c || p.qslot || p.tile_colour || p.panel_counter || ranges) return hipErrorInvalidValue;
    if (vec4 && p.Xq_split && p.Xc_split && p.hq_split && p.hc_split && p.d >= SLHC_STREAM_SPLIT_MIN_D &&
        (((reinterpret_cast<uintptr_t>(p.Xq_split) | reinterpret_cast<uintptr_t>(p.Xc_split)) & 15) == 0))
        return launch_with_lds(&sweep_kernel<KL, MASKED, true, true>, grid, lds, p, stream);
    if (vec4) return launch_with_lds(&sweep_kernel<KL, MASKED, true>, grid, lds, p, stream);
    return launch_with_lds(&sweep_kernel<KL, MASKED, false>, grid, lds, p, stream);
}

// (dist bits << 32 | idx) keys of a segmented 1-NN sweep -> idx, dist; an untouched key: -1, +inf
__global__ void __launch_bounds__(256) unpack_keys_kernel(const unsigned long long* __restrict__ keys, int m,
                                                          int32_t* __restrict__ out_idx, float* __restrict__ out_dist)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= m) return;
    const unsigned long long key = keys[i];
    out_idx[i] = key == LIST_SENTINEL ? -1 : (int)(unsigned int)(key & 0xffffffffull);
    out_dist[i] = __uint_as_float((unsigned int)(key >> 32));
}

__global__ void __launch_bounds__(256) fill_keys_kernel(unsigned long long* __restrict__ keys, int m)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < m) keys[i] = LIST_SENTINEL;
}

// Number of candidate segments for a 1-NN sweep of m query rows.  With so few panels that 16 segments
// each would not fill the workgroup slots: one work item per slot.  Otherwise the S up to 16 (and at
// least 16 tiles per segment) that minimises the time of the busiest slot, in panel passes:
// (full rounds of work items + the last, partial round) / S, where a last round that leaves every CU
// at most one workgroup counts 0.6 (a workgroup alone on its CU is that much faster; measured).
// Segmented sweeps run in the streaming kernel; where the unsegmented sweep would run in the faster
// register-resident-query kernel (`fast_unsegmented`) a split has to win by more than that kernel's
// edge, and any split by 10 %.
int sweep_segments_for(int m, int NC, bool fast_unsegmented)
{
    int cus = 0;
    if (device_cus(&cus) != hipSuccess) return 1;
    const long long npanels = (m + BM - 1) / BM;
    const int ntiles = (NC + BN - 1) / BN;
    if (npanels < 1 || ntiles < 1) return 1;
    const long long slots = 2LL * cus;
    if (npanels * 16 <= slots) {
        long long seg = slots / npanels;
        if (seg > ntiles) seg = ntiles;
        return seg < 1 ? 1 : (int)seg;
    }
    auto passes = [&](int seg) {
        const long long items = npanels * seg;
        const long long full = items / slots, last = items % slots;
        const double tail = last == 0 ? 0.0 : (last * 2 <= slots ? 0.6 : 1.0);
        return ((double)full + tail) / seg;
    };
    int best = 1;
    double best_cost = passes(1);
    const double bar = 0.9 * best_cost;
    for (int seg = 2; seg <= 16 && ntiles / seg >= 16; ++seg) {
        double cost = passes(seg) * (1.0 + 0.004 * seg);   // per-item set-up and the merge of the minima
        if (fast_unsegmented) cost *= SLHC_SEGMENT_HANDICAP;
        if (cost < bar && cost < best_cost) { best = seg; best_cost = cost; }
    }
    return best;
}

hipError_t launch_segmented_1nn(const SweepParams& p_in, unsigned long long* keys, hipStream_t stream)
{
    SweepParams p = p_in;
    const int m = p.NQ;
    if (m < 1) return hipSuccess;
    p.k = 1;
    p.segments = sweep_segments_for(m, p.NC, p.d % 4 == 0 && p.d <= 4 * KC);
    if (p.segments <= 1) {
        p.segments = 0;
        p.out_key = nullptr;
        return launch_knn_sweep(p, stream);
    }
    p.out_key = keys;
    hipLaunchKernelGGL(fill_keys_kernel, dim3((m + 255) / 256), dim3(256), 0, stream, keys, m);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    e = launch_knn_sweep(p, stream);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(unpack_keys_kernel, dim3((m + 255) / 256), dim3(256), 0, stream, keys, m, p.out_idx, p.out_dist);
    return hipGetLastError();
}

// The cross-colour sweep for a short row list (p.m rows, p.rows): with fewer panels than the chip has
// workgroup slots a panel's pass over all candidate tiles is pure latency, so the tiles are split
// into segments exactly as in launch_segmented_1nn (streaming kernel, 64-bit minimum per query).
// Falls back to launch_cross_1nn_sweep when one segment is enough or the sweep is a pruned one.
hipError_t launch_segmented_cross_1nn(const SweepParams& p_in, unsigned long long* keys, hipStream_t stream)
{
    SweepParams p = p_in;
    const int m = p.m;
    if (m < 1) return hipSuccess;
    p.k = 1;
    if (p.tile_c && p.qslot) {
        // pruned sweep with a slot map: the caller chooses into how many parts every panel's scan is split
        if (!keys || p.segments < 2) p.segments = 1;
    } else {
        p.segments = (p.tile_c || p.qslot || !keys) ? 1 : sweep_segments_for(m, p.NC, p.d % 4 == 0 && p.d <= 4 * KC);
    }
    if (p.segments <= 1) {
        p.segments = 0;
        p.out_key = nullptr;
        return launch_cross_1nn_sweep(p, stream);
    }
    p.out_key = keys;
    hipLaunchKernelGGL(fill_keys_kernel, dim3((m + 255) / 256), dim3(256), 0, stream, keys, m);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    e = launch_cross_1nn_sweep(p, stream);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(unpack_keys_kernel, dim3((m + 255) / 256), dim3(256), 0, stream, keys, m, p.out_idx, p.out_dist);
    return hipGetLastError();
}

int sweep_grid_limit()
{
    int cus = 0;
    if (device_cus(&cus) != hipSuccess) return 0;
    return 2 * cus;
}

// The k smallest entries, by (distance, index), of a row's `segments` ascending lists of k: one thread per row.
// Unused entries of a list are (-1, +inf) and sort last.
__global__ void __launch_bounds__(256) merge_ranges_kernel(const int32_t* __restrict__ part_idx,
                                                           const float* __restrict__ part_dist, int segments, int NQ,
                                                           int k, int32_t* __restrict__ out_idx, float* __restrict__ out_dist)
{
    const int row = blockIdx.x * 256 + threadIdx.x;
    if (row >= NQ) return;
    int at[16];
#pragma unroll
    for (int s = 0; s < 16; ++s) at[s] = 0;
    for (int j = 0; j < k; ++j) {
        unsigned long long best = ~0ull;
        int from = 0;
#pragma unroll
        for (int s = 0; s < 16; ++s) {
            if (s < segments && at[s] < k) {
                const size_t o = ((size_t)s * (size_t)NQ + (size_t)row) * k + at[s];
                const unsigned long long key = ((unsigned long long)__float_as_uint(part_dist[o]) << 32) |
                                               (unsigned long long)(unsigned int)part_idx[o];
                if (key < best) { best = key; from = s; }
            }
        }
        ++at[from];
        out_idx[(size_t)row * k + j] = (int)(unsigned int)(best & 0xffffffffull);
        out_dist[(size_t)row * k + j] = __uint_as_float((unsigned int)(best >> 32));
    }
}

#ifndef SLHC_RANGE_MIN_TILES
#define SLHC_RANGE_MIN_TILES 2
#endif
constexpr int RANGE_MIN_TILES = SLHC_RANGE_MIN_TILES;      // candidate tiles a range of a split k-NN sweep holds at least

hipError_t launch_knn_sweep(const SweepParams& p_in, hipStream_t stream)
{
    SweepParams p = p_in;
    // Few panels (less than half the workgroup slots), k > 1, every tile, query fragments in registers: split the
    // candidate tiles into ranges so that the whole chip works, at least 8 tiles per range, at most 16 ranges.
    if (p.k > 1) p.segments = 0;          // (k = 1: launch_segmented_1nn has set the segments of its own scheme)
    if (p.k > 1 && p.part_idx && p.part_dist && !p.tile_c && !p.q_out_row && p.d % 4 == 0 && p.d <= 4 * KC &&
        (((reinterpret_cast<uintptr_t>(p.Xq) | reinterpret_cast<uintptr_t>(p.Xc)) & 15) == 0)) {
        int cus = 0;
        hipError_t e = device_cus(&cus);
        if (e != hipSuccess) return e;
        const int slots = 2 * cus, npanels = (p.NQ + BM - 1) / BM, ntiles = (p.NC + BN - 1) / BN;
        int s = npanels > 0 ? slots / npanels : 1;
        if (s > ntiles / RANGE_MIN_TILES) s = ntiles / RANGE_MIN_TILES;
        if (s > 16) s = 16;
        if (s >= 2 && (long long)s * p.NQ <= p.part_rows) p.segments = s;
    }
    hipError_t e;
    if (p.k == 1) e = launch_sweep_t<1, false>(p, stream);
    else if (p.k <= 8) e = launch_sweep_t<8, false>(p, stream);
    else if (p.k <= 16) e = launch_sweep_t<16, false>(p, stream);
    else if (p.k <= 32) e = launch_sweep_t<32, false>(p, stream);
    else e = launch_sweep_t<64, false>(p, stream);
    if (e != hipSuccess || p.k == 1 || p.segments < 2) return e;
    hipLaunchKernelGGL(merge_ranges_kernel, dim3((p.NQ + 255) / 256), dim3(256), 0, stream, p.part_idx, p.part_dist,
                       p.segments, p.NQ, p.k, p.out_idx, p.out_dist);
    return hipGetLastError();
}

hipError_t launch_cross_1nn_sweep(const SweepParams& p, hipStream_t stream)
{
    return launch_sweep_t<1, true>(p, stream);
}

}  // namespace slhc
