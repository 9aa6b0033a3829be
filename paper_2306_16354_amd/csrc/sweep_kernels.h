// Launch interface of the fused distance + selection sweeps (sweep_kernels.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace slhc {

// Queries and candidates are rows of two row-major matrices (the same one for a self-join).
// Row indices inside a sweep are positions in those matrices; `c_id` / `q_out_row` translate
// them back when the matrices are a reordered copy of the caller's data.
struct SweepParams {
    const float* Xq;       // [NQ, d] query rows
    const float* hq;       // [NQ]  (1-c)/2 * ||x||^2 of the query rows (launch_half_norms)
    const float* Xc;       // [NC, d] candidate rows
    const float* hc;       // [NC]
    int NQ, NC, d, k;
    // Optional (sweep_kernel_qreg: d % 32 == 0, d >= 64; the streaming sweep_kernel: d > 128, d % 4 == 0, rows of
    // split_row_stride(d) words with zeros past column d): the same two matrices with every
    // value split into two bfloat16 halves, hi = bf16(x) and lo = bf16(x - hi), laid out chunk by chunk: the 32
    // floats of columns 32c .. 32c+31 of a row are replaced by 32 hi values then 32 lo values (launch_split_bf16).
    // The tile products are then accumulated as hi*hi + hi*lo + lo*hi on the bf16 MFMA, which runs at 16 times
    // the fp32 rate.  The split copy may hold the rows translated by a common vector (launch_split_bf16's shift),
    // so it comes with half norms of its own, hq_split / hc_split: those of the translated rows, from
    // launch_half_norms with split_slack_coefficient(d), whose slack covers the dropped lo*lo terms.  A kernel that
    // multiplies the split copy reads these, one that multiplies Xq / Xc reads hq / hc.  Only the filter changes:
    // pairs that pass are re-evaluated from Xq / Xc.
    const float* Xq_split;
    const float* Xc_split;
    const float* hq_split;
    const float* hc_split;
    // Pruned k-NN sweeps of a self-join in the reordered copy (own_tile_first) may run as two launches over the
    // same output lists.  tile_region [tiles]: a region number per candidate tile (= per query panel).
    // region_mode 1: a panel only visits the tiles of its own region, for which the caller passes a split copy
    // taken relative to a vector of that region's own (rows of one cluster share their centre as an offset, which
    // a shift common to all rows does not remove: local coordinates keep it out of the filter's slack);
    // region_mode 2: a panel starts from the lists the first launch wrote and visits the other tiles only,
    // with the split copy relative to the common shift.  0: one launch, all tiles.
    const int32_t* tile_region;
    int region_mode;
    const int32_t* tile_first;  // optional, with region_mode 1: first and last tile of every tile's region (regions are
    const int32_t* tile_last;   // runs of consecutive tiles), which bound the scan
    const float* region_other_min;   // optional, with region_mode 2 and tile_gap: per panel, the smallest lower bound of a tile
                                     // outside its region; a panel whose thresholds are all below it is left alone
    int32_t* out_idx;      // k-NN: [*, k] at row q_out_row[q] (or q); cross 1-NN: [m]
    float* out_dist;       // same shape
    const int32_t* q_out_row;   // k-NN only: output row of query row q (nullptr: q itself)
    const int32_t* c_id;        // id reported for candidate row c and used to order ties (nullptr: c)
    int exclude_self;      // k-NN only: candidate row == query row is skipped (self-join)
    const int32_t* qcolour;     // cross 1-NN only: [NQ] colour of query rows
    const int32_t* ccolour;     // cross 1-NN only: [NC] colour of candidate rows
    const int32_t* rows;   // cross 1-NN only: [m] query rows, or nullptr for rows 0..m-1
    int m;                 // cross 1-NN only
    // cross 1-NN, alternative to rows/m: qslot[NQ] holds the output slot of every query row and -1
    // for rows that are not queried; panel p then serves the queried rows among rows 128p..128p+127
    // (queries stay aligned with the candidate tiles of a reordered copy)
    const int32_t* qslot;
    // Tile pruning (all nullptr / 0: every candidate tile is multiplied).  tile_c [T, d] and
    // tile_r [T] are bounding balls of the candidate tiles of 128 rows (tile_r already inflated
    // for rounding); gap_ws is scratch of gridDim.x * T floats.
    const float* tile_c;
    const float* tile_r;
    float* gap_ws;
    // optional [T, T] (order_tile_gaps): the lower bounds between all pairs of tile balls.  A panel whose query
    // rows are (a subset of) the rows of candidate tile `panel` - a self-join in the same row order with
    // own_tile_first, or the slot map `qslot` - then reads its row of this table instead of computing a ball
    // of its own and T lower bounds (for a subset the table's bounds are a little looser, never wrong).
    const float* tile_gap;
    const int32_t* tile_colour;   // cross 1-NN only, optional [T]: the colour all valid rows of a tile
                                  // share, or -1; a tile in the colour of all the panel's queries is skipped
    // cross 1-NN with pruning, optional: comp_best[c] (c < comp_count) is the lightest edge weight already
    // known out of component (colour) c, as bits of a non-negative float (+inf bits: none).  The sweep
    // uses it, read-only, as a threshold shared by all queries of that colour.  A query's answer is then
    // its exact nearest foreign row only if its distance is <= comp_best of its colour; otherwise no
    // foreign row is nearer than comp_best, which is all the caller may conclude.
    const unsigned int* comp_best;
    int comp_count;
    // optional, the same array as comp_best: the sweep also lowers comp_best[c] (atomic minimum) whenever a
    // query of colour c finds a foreign row nearer than it, and all queries of that colour run under the
    // lowered value from then on.  The rule above then holds with the value the word has when the sweep has
    // FINISHED: answers at distance <= that final value are exact, every other query only knows that no
    // foreign row is nearer than it.  The final value is min(value at launch, lightest edge from any queried
    // row of that colour to a foreign row), whatever the order in which the panels ran.
    unsigned int* comp_best_lower;
    // >= 1.  The word is lowered to comp_lower_factor times the lightest edge found, not to the edge itself:
    // with factor 1 only the queries that tie with the component's lightest edge end with an exact answer,
    // and all the others have to be asked again in a later round; a factor of 2 (in squared distance) keeps
    // the answers of nearly all rows of a compact cluster exact while still cutting off everything beyond
    // 1.4 times the distance to the nearest foreign row.
    float comp_lower_factor;
    // optional: comp_size[c] = rows of component c; only components of at least comp_lower_min_size rows
    // lower their word.  A component that fits a few panels gains little from a falling threshold, and
    // every row that ends without an exact answer has to be asked again in the next round.
    const int32_t* comp_size;
    int comp_lower_min_size;
    unsigned int* panel_counter;  // optional device word, zero at launch: panels are taken from it one at
                                  // a time instead of round-robin (use when panel costs differ widely)
    int own_tile_first;    // self-join in the same row order: start each panel at its own tile
    // cross 1-NN with a slot map, optional: the panels that hold a queried row (any order); the others are then
    // not visited at all
    const int32_t* panel_list;
    int panel_list_n;
    // k = 1 between two matrices with few query rows: the candidate tiles are split into `segments`
    // parts, one work item per (panel, part); every item merges its result into out_key[q] with a
    // 64-bit atomic minimum over (dist bits << 32 | idx), which is the (dist, idx) order.  Set by
    // launch_segmented_1nn; 0 / nullptr otherwise.
    int segments;
    unsigned long long* out_key;
    // k-NN with k > 1 and few query panels (launch_knn_sweep decides): the candidate tiles are split into
    // `segments` ranges, one work item per (panel, range); item (panel, s) writes its lists to
    // part_idx / part_dist [s][NQ][k], and a merge kernel picks the k smallest of a row's lists.  Scratch of
    // part_rows * k entries each (rows x segments must fit); nullptr: never split.
    int32_t* part_idx;
    float* part_dist;
    long long part_rows;
    // Every-tile sweeps of many panels (sweep_kernel_qreg; the launcher decides and sets carry_ranges): the work
    // items are (range of candidate tiles, panel), handed out range by range so that all workgroups sweep the
    // same few megabytes of candidates at a time, and a panel's lists travel from range to range through
    // out_idx / out_dist.  carry_ws: scratch of 2 + (panels) words (hand-out counter, spare, ranges finished
    // per panel), cleared by the launcher; nullptr: never.  carry_fault (optional device word): bit 1 is set if
    // a work item's wait for its predecessor ever runs out (never seen; the results are then not valid).
    unsigned int* carry_ws;
    long long carry_ws_words;
    int carry_ranges;
    unsigned int* carry_fault;
    unsigned long long* survivors;   // optional device counter: pairs that passed the filter
    unsigned long long* tiles_done;  // optional device counter: (panel, tile) steps multiplied
#ifdef SLHC_PHASE_TIMERS
    unsigned long long* phase_cycles;   // study builds: [8] cycles per phase of the panel loop
#endif
#ifdef SLHC_STUDY_PANEL_STEPS
    int* panel_steps;                   // study builds: [npanels] multiplied tiles and [npanels] cycles per panel
#endif
};

float filter_slack_coefficient(int d);
float split_slack_coefficient(int d);                 // the same for products accumulated from split bf16 halves
// X [N, d] -> the chunk-wise split copy described at SweepParams::Xq_split (d % 32 == 0)
// `shift` (optional, [d] device floats, 16-byte aligned): the copy holds fl(x - shift)
// `shift_tile` (optional, with shift): shift is a matrix [*, d] and the rows of tile t = row / 128 take its row shift_tile[t]
hipError_t launch_split_bf16(const float* X, int N, int d, float* Xsplit, hipStream_t stream, const float* shift = nullptr,
                             const int* shift_tile = nullptr);
// a central value of every column of X (median of the means of 64 runs of a row sample) -> mean [d];
// scratch: column_means_scratch_floats(d) device floats
size_t column_means_scratch_floats(int d);
hipError_t launch_column_means(const float* X, int N, int d, float* scratch, float* mean, hipStream_t stream);
int split_row_stride(int d);                          // words per row of the split copy: d rounded up to whole chunks of 32
// `nonfinite` (optional device word, zero at launch): set to 1 when a row's squared norm is not a finite float32
// `shift` (optional): the norms of fl(x - shift), as for launch_split_bf16
hipError_t launch_half_norms(const float* X, int N, int d, float* hn, hipStream_t stream, unsigned int* nonfinite = nullptr,
                             bool split_slack = false, const float* shift = nullptr, const int* shift_tile = nullptr);
// Launches the register-only fp32 MFMA loop (2 workgroups per CU, `iters` x 16 instructions per wavefront);
// *flop receives the floating-point operations of the launch.  `sink`: one device float.
hipError_t launch_mfma_probe(int iters, float* sink, hipStream_t stream, double* flop);
// the same with v_mfma_f32_32x32x16_bf16, the multiply of the split-product sweeps
hipError_t launch_mfma_bf16_probe(int iters, float* sink, hipStream_t stream, double* flop);
// D[t] = C[t] + sum_{k<16} A[t][k] B[t][k] by one v_mfma_f32_32x32x16_bf16 per trial (device arrays, A and B [trials][16])
hipError_t launch_mfma_bf16_values(const float* A, const float* B, const float* C, float* D, int trials, hipStream_t stream);
// The multiplies of launch_mfma_probe with the panel loop's ingredients added (steps 0..3, see the kernel);
// `stream_rows`: [rows, 128] floats to stream from (steps >= 2; rows a power of two), iters chunks of 64 multiplies.
hipError_t launch_loop_probe(int steps, int iters, const float* stream_rows, int rows, float* sink, hipStream_t stream,
                             double* flop);
int sweep_grid_limit();   // upper bound of gridDim.x of a sweep launch (for sizing gap_ws); 0 on error
hipError_t launch_knn_sweep(const SweepParams& p, hipStream_t stream);
hipError_t launch_cross_1nn_sweep(const SweepParams& p, hipStream_t stream);
// Nearest candidate row of every query row (k-NN mode parameters with k = 1, no self exclusion
// unless asked).  Splits the candidates over the chip when there are few query rows; `keys` is
// scratch of NQ 64-bit words.
hipError_t launch_segmented_1nn(const SweepParams& p, unsigned long long* keys, hipStream_t stream);
// launch_cross_1nn_sweep for a short row list: candidate tiles split into segments when the panels alone
// would not fill the chip; `keys`: p.m 64-bit words of scratch (may be nullptr: no segmentation).
hipError_t launch_segmented_cross_1nn(const SweepParams& p, unsigned long long* keys, hipStream_t stream);

}  // namespace slhc
