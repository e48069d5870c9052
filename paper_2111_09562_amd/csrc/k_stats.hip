// Semi-online statistic of the controller (COMET Sec. 3.1): the mean of |x| over a tensor, for the
// momentum and for the gradient of the loss.  Two kernels so that the result does not depend on
// the order in which workgroups finish: every workgroup leaves the fp64 sum of its slice (a fixed
// tree inside the workgroup), one workgroup adds the partial sums up in index order.
#include "comet_kernels.h"

namespace comet {

__global__ __launch_bounds__(kStatsBlock) void k_abs_sum(const float *x, uint64_t n, double *partial) {
    __shared__ double s_part[kStatsBlock / kWave];
    const uint64_t per = (n + gridDim.x - 1) / gridDim.x;               // a contiguous slice per workgroup
    const uint64_t lo = (uint64_t)blockIdx.x * per;
    const uint64_t hi = (lo + per < n) ? lo + per : n;
    double acc = 0.0;
    for (uint64_t i = lo + threadIdx.x; i < hi; i += kStatsBlock) acc += fabs((double)x[i]);
    acc = wave_sum<double>(acc);
    if (lane_id() == 0) s_part[threadIdx.x / kWave] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
#pragma unroll
        for (int w = 0; w < kStatsBlock / kWave; ++w) t += s_part[w];
        partial[blockIdx.x] = t;
    }
}

__global__ __launch_bounds__(kWave) void k_abs_mean_final(const double *partial, uint32_t n_partial, uint64_t n, double *mean_out) {
    double acc = 0.0;
    for (uint32_t i = threadIdx.x; i < n_partial; i += kWave) acc += partial[i];
    acc = wave_sum<double>(acc);
    if (threadIdx.x == 0) *mean_out = acc / (double)n;
}

}  // namespace comet
