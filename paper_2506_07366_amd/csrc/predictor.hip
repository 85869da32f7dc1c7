// Distribution-Only predictor (Section 3.2.1, Eq. (1); Appendix A): the maximum-
// likelihood estimate of the expert distribution of a layer is p_hat_i = n_i / N over
// all tokens seen; with batches it is the running average.  The state is the
// cumulative count per expert (int64).  The prediction for a coming batch of A
// assignments is p_hat * A rounded to integers that sum to A by largest remainder
// (ties -> lowest expert).  Exact integer arithmetic (128-bit products), one
// workgroup: E is at most 1024.
#include "common.h"

namespace moegps {

__global__ __launch_bounds__(1024) void predictor_update_kernel(const int32_t* __restrict__ hist, int E,
                                                                 int64_t* __restrict__ counts) {
    const int e = threadIdx.x;
    if (e < E) {
        const int h = hist[e];
        if (h > 0) counts[e] += h;
    }
}

__global__ __launch_bounds__(1024) void predictor_predict_kernel(const int64_t* __restrict__ counts, int E,
                                                                  int64_t A, int32_t* __restrict__ hist_pred) {
    __shared__ unsigned long long rem_s[MOE_MAX_EXPERTS];
    __shared__ unsigned long long part[1024 / kWave];
    const int e = threadIdx.x;
    const int lane = e & (kWave - 1), w = e / kWave;
    // N = sum of the counts (wavefront shuffle, then across wavefronts)
    auto block_sum = [&](unsigned long long v) {
        for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
        __syncthreads();  // part[] free again
        if (lane == 0) part[w] = v;
        __syncthreads();
        unsigned long long s = 0;
        for (int i = 0; i < 1024 / kWave; ++i) s += part[i];
        return s;
    };
    const long long c_raw = e < E ? counts[e] : 0;
    unsigned long long c = c_raw > 0 ? (unsigned long long)c_raw : 0ull;
    unsigned long long N = block_sum(c);
    if (N == 0) {  // nothing seen yet: uniform
        c = e < E ? 1ull : 0ull;
        N = (unsigned long long)E;
    }
    const unsigned __int128 prod = (unsigned __int128)c * (unsigned long long)A;
    const unsigned long long base = (unsigned long long)(prod / N);
    const unsigned long long rem = (unsigned long long)(prod % N);
    if (e < E) rem_s[e] = rem;
    const unsigned long long base_sum = block_sum(e < E ? base : 0ull);
    const unsigned long long deficit = (unsigned long long)A - base_sum;  // < E
    if (e < E) {
        // place of this expert in (remainder descending, index ascending) order
        unsigned long long before = 0;
        for (int o = 0; o < E; ++o) {
            const unsigned long long ro = rem_s[o];
            before += (ro > rem || (ro == rem && o < e)) ? 1ull : 0ull;
        }
        hist_pred[e] = (int32_t)(base + (before < deficit ? 1ull : 0ull));
    }
}

}  // namespace moegps

extern "C" int moe_predictor_update(const int32_t* hist, int E, int64_t* counts, void* stream) {
    using namespace moegps;
    if (E < 1) return MOE_ERR_INVALID_ARG;
    if (E > MOE_MAX_EXPERTS) return MOE_ERR_UNSUPPORTED;
    if (!hist || !counts) return MOE_ERR_INVALID_ARG;
    hipLaunchKernelGGL(predictor_update_kernel, dim3(1), dim3(1024), 0, (hipStream_t)stream, hist, E, counts);
    return check_launch();
}

extern "C" int moe_predictor_predict(const int64_t* counts, int E, int64_t A_next, int32_t* hist_pred, void* stream) {
    using namespace moegps;
    if (E < 1 || A_next < 0) return MOE_ERR_INVALID_ARG;
    if (E > MOE_MAX_EXPERTS || A_next >= (1ll << 31)) return MOE_ERR_UNSUPPORTED;
    if (!counts || !hist_pred) return MOE_ERR_INVALID_ARG;
    hipLaunchKernelGGL(predictor_predict_kernel, dim3(1), dim3(1024), 0, (hipStream_t)stream, counts, E, A_next,
                       hist_pred);
    return check_launch();
}
