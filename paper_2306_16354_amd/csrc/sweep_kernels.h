// Launch interface of the fused distance + selection sweeps (sweep_kernels.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace slhc {

struct SweepParams {
    const float* X;        // [N, d]
    const float* hn;       // [N]  (1-c)/2 * ||x||^2, from launch_half_norms
    int N, d, k;
    int32_t* out_idx;      // k-NN: [N, k]; cross 1-NN: [m]
    float* out_dist;       // same shape
    const int32_t* colour; // cross 1-NN only: [N]
    const int32_t* rows;   // cross 1-NN only: [m] query rows, or nullptr for rows 0..m-1
    int m;                 // cross 1-NN only
    unsigned long long* survivors;   // optional device counter: pairs that passed the filter
};

float filter_slack_coefficient(int d);
hipError_t launch_half_norms(const float* X, int N, int d, float* hn, hipStream_t stream);
hipError_t launch_knn_sweep(const SweepParams& p, hipStream_t stream);
hipError_t launch_cross_1nn_sweep(const SweepParams& p, hipStream_t stream);

}  // namespace slhc
