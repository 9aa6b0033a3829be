// Spatially coherent row order and bounding balls of candidate tiles (order_kernels.hip).
// Used to skip (query panel, candidate tile) pairs that provably cannot contribute; the paper's
// kernels multiply every tile (Sec. 3.1.1: all N^2 distances are computed).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace slhc {

hipError_t order_iota(int32_t* a, int n, hipStream_t s);
// Xp[j] = X[row_j], hp[j] = h[row_j] with row_j = floor(j * N / P): P evenly spaced rows
hipError_t order_pick_rows(const float* X, const float* h, int N, int d, int P, float* Xp, float* hp, hipStream_t s);
hipError_t order_gather_rows(const float* X, const int32_t* perm, int N, int d, float* Xs, hipStream_t s);
// out[i] = a[idx[i]] for i < n; `fallback` where the index is outside [0, limit)
hipError_t order_gather_f32(const float* a, const int32_t* idx, int n, int limit, float fallback, float* out,
                            hipStream_t s);
hipError_t order_gather_i32(const int32_t* a, const int32_t* idx, int n, int limit, int32_t fallback, int32_t* out,
                            hipStream_t s);
// out[j] = a[floor(j * N / P)]: P evenly spaced entries
hipError_t order_pick_f32(const float* a, int N, int P, float* out, hipStream_t s);
// key[i] = (dist[i] > tau) ? 0 : 1, and *count += number of rows with key 0 (count zeroed by the caller)
hipError_t order_mark_far(const float* dist, int n, float tau, uint32_t* key, int32_t* count, hipStream_t s);
// Xp[j] = X[list[floor(j * m / P)]], hp[j] = h[...]: P evenly spaced rows of a row list of length m
hipError_t order_pick_listed_rows(const float* X, const float* h, const uint32_t* list, int m, int N, int d, int P,
                                  float* Xp, float* hp, hipStream_t s);
hipError_t order_invert(const int32_t* perm, int n, int32_t* inv, hipStream_t s);
hipError_t order_fill_i32(int32_t* a, int n, int32_t value, hipStream_t s);
// counts[pid[i]] += 1 (counts zeroed by the caller)
hipError_t order_histogram(const int32_t* pid, int n, int bins, int32_t* counts, hipStream_t s);
// key[i] = rank[pid[i]]
hipError_t order_keys(const int32_t* pid, const int32_t* rank, int n, int bins, uint32_t* key, hipStream_t s);
// rows sorted by key -> padded layout: pos = j + shift[key_sorted[j]]; perm[pos] = row_sorted[j];
// inv[row_sorted[j]] = pos.  perm must be pre-filled with -1 (padding rows).
hipError_t order_scatter(const uint32_t* key_sorted, const uint32_t* row_sorted, const int32_t* shift,
                         int n, int bins, int n_padded, int32_t* perm, int32_t* inv, hipStream_t s);
// Xs[i] = X[perm[i]] (zeros where perm[i] < 0); hs[i] = h[perm[i]] (+inf where perm[i] < 0)
hipError_t order_gather_padded(const float* X, const float* h, const int32_t* perm, int n_padded, int N,
                               int d, float* Xs, float* hs, hipStream_t s);
// centre (mean) and radius (largest distance to the centre) of the valid rows (perm[i] >= 0) of
// every tile of 128 consecutive rows; a tile without valid rows gets radius -3e38 (always skipped)
hipError_t order_tile_balls(const float* Xs, const int32_t* perm, int n_padded, int d, float* tile_c,
                            float* tile_r, hipStream_t s);

// for j < m: row list[j] adopts pivot base + new_idx[j] (new_idx in [0, count)) when new_dist[j] < pdist[row]
hipError_t order_adopt_pivots(const uint32_t* list, int m, int N, const int32_t* new_idx, const float* new_dist,
                              int base, int count, int32_t* pid, float* pdist, hipStream_t s);
// tile_colour[t] = the colour shared by all rows with colour_s >= 0 of tile t, or -1
// gaps[p * T + t]: lower bound of the squared distance between any row of tile p and any row of tile t, from their
// bounding balls (rounded towards zero; NaN where either tile has no valid row).  T x T floats.
hipError_t order_tile_gaps(const float* tile_c, const float* tile_r, int T, int d, float* gaps, hipStream_t s);
// *count += number of tiles (128 consecutive entries of slot[0 .. n_padded)) with an entry >= 0; `list` (optional,
// room for every tile, *count zero at launch) receives their numbers in no particular order
hipError_t order_count_used_tiles(const int32_t* slot, int n_padded, int32_t* count, int32_t* list, hipStream_t s);
hipError_t order_tile_colours(const int32_t* colour_s, int n_padded, int32_t* tile_colour, hipStream_t s);
// slot[inv[list[q]]] = q for q < m (slot pre-filled with -1 by the caller)
hipError_t order_scatter_slots(const int32_t* inv, const int32_t* list, int m, int N, int n_padded, int32_t* slot,
                               hipStream_t s);

}  // namespace slhc
