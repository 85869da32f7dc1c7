// Per-expert token counts n_e (the n_i of Eq. (1), p_hat_i = n_i / N): the
// "distribution" that Distribution-Only Prediction forecasts.  Counts are
// privatised in LDS per workgroup and merged with integer atomics, so the
// result does not depend on the launch shape.
#include "common.h"

namespace moegps {

constexpr int kHistThreads = 1024;
constexpr int kHistItemsPerBlock = 16384;  // elements one workgroup of the wide kernel covers

// One workgroup counts everything and writes the result directly.
__global__ __launch_bounds__(kHistThreads) void hist_single_kernel(const int32_t* __restrict__ idx, int64_t n,
                                                                    int E, int32_t* __restrict__ hist) {
    __shared__ int bins[MOE_MAX_EXPERTS];
    for (int e = threadIdx.x; e < E; e += blockDim.x) bins[e] = 0;
    __syncthreads();
    for (int64_t i = threadIdx.x; i < n; i += blockDim.x) {
        const int e = idx[i];
        if (e >= 0 && e < E) atomicAdd(&bins[e], 1);
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += blockDim.x) hist[e] = bins[e];
}

__global__ void hist_zero_kernel(int32_t* __restrict__ hist, int E) {
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e < E) hist[e] = 0;
}

__global__ __launch_bounds__(kHistThreads) void hist_wide_kernel(const int32_t* __restrict__ idx, int64_t n,
                                                                  int E, int32_t* __restrict__ hist) {
    __shared__ int bins[MOE_MAX_EXPERTS];
    for (int e = threadIdx.x; e < E; e += blockDim.x) bins[e] = 0;
    __syncthreads();
    const int64_t lo = (int64_t)blockIdx.x * kHistItemsPerBlock;
    const int64_t hi = (lo + kHistItemsPerBlock < n) ? lo + kHistItemsPerBlock : n;
    for (int64_t i = lo + threadIdx.x; i < hi; i += blockDim.x) {
        const int e = idx[i];
        if (e >= 0 && e < E) atomicAdd(&bins[e], 1);
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += blockDim.x) {
        const int c = bins[e];
        if (c) atomicAdd(&hist[e], c);
    }
}

}  // namespace moegps

extern "C" int moe_histogram(const int32_t* idx, int64_t n, int E, int32_t* hist, void* stream) {
    using namespace moegps;
    if (n < 0 || E < 1) return MOE_ERR_INVALID_ARG;
    if (E > MOE_MAX_EXPERTS) return MOE_ERR_UNSUPPORTED;
    if (!hist || (n > 0 && !idx)) return MOE_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    if (n <= 4 * kHistItemsPerBlock) {
        hipLaunchKernelGGL(hist_single_kernel, dim3(1), dim3(kHistThreads), 0, st, idx, n, E, hist);
        return check_launch();
    }
    hipLaunchKernelGGL(hist_zero_kernel, dim3(ceil_div(E, 256)), dim3(256), 0, st, hist, E);
    int rc = check_launch();
    if (rc != MOE_OK) return rc;
    const int64_t grid = ceil_div64(n, kHistItemsPerBlock);
    hipLaunchKernelGGL(hist_wide_kernel, dim3((unsigned)grid), dim3(kHistThreads), 0, st, idx, n, E, hist);
    return check_launch();
}
