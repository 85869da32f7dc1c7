// Weighted un-permute: out[t] = sum_j w[t, j] * y_perm[row_of_assign[t*k + j]].
// Stands where the all-to-all after the expert FFN is (Background: "The same
// amount of communication happens for All-to-All shuffle after the FFN layers").
// One wavefront per token; each lane owns 16-byte pieces of the row, gathers the
// k source rows, accumulates in fp32 with j ascending and stores once.
#include "common.h"

namespace moegps {

__device__ __forceinline__ float bf16_bits_to_float(unsigned short b) {
    return __builtin_bit_cast(float, (unsigned)b << 16);
}
__device__ __forceinline__ unsigned short float_to_bf16_bits(float f) {
    return __builtin_bit_cast(unsigned short, (__bf16)f);  // round to nearest even
}

template <bool BF16>
__global__ __launch_bounds__(256) void combine_kernel(const uint4* __restrict__ y_perm,
                                                       const int32_t* __restrict__ row_of_assign,
                                                       const float* __restrict__ topk_w, uint4* __restrict__ out,
                                                       int T, int k, int chunks) {
    const int lane = threadIdx.x & (kWave - 1);
    const int t = __builtin_amdgcn_readfirstlane((int)((blockIdx.x * (unsigned)blockDim.x + threadIdx.x) / kWave));
    if (t >= T) return;
    int rows[MOE_MAX_TOPK];
    float w[MOE_MAX_TOPK];
#pragma unroll
    for (int j = 0; j < MOE_MAX_TOPK; ++j) {
        rows[j] = j < k ? row_of_assign[(size_t)t * k + j] : 0;
        w[j] = j < k ? topk_w[(size_t)t * k + j] : 0.f;
    }
    for (int c = lane; c < chunks; c += kWave) {
        constexpr int N = BF16 ? 8 : 4;
        float acc[N];
#pragma unroll
        for (int i = 0; i < N; ++i) acc[i] = 0.f;
#pragma unroll
        for (int j = 0; j < MOE_MAX_TOPK; ++j) {
            if (j < k) {
                const uint4 v = y_perm[(size_t)rows[j] * chunks + c];
                const unsigned u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (BF16) {
                        acc[2 * i] = fmaf(w[j], bf16_bits_to_float((unsigned short)(u[i] & 0xffffu)), acc[2 * i]);
                        acc[2 * i + 1] = fmaf(w[j], bf16_bits_to_float((unsigned short)(u[i] >> 16)), acc[2 * i + 1]);
                    } else {
                        acc[i] = fmaf(w[j], __builtin_bit_cast(float, u[i]), acc[i]);
                    }
                }
            }
        }
        uint4 o;
        if (BF16) {
            o.x = (unsigned)float_to_bf16_bits(acc[0]) | ((unsigned)float_to_bf16_bits(acc[1]) << 16);
            o.y = (unsigned)float_to_bf16_bits(acc[2]) | ((unsigned)float_to_bf16_bits(acc[3]) << 16);
            o.z = (unsigned)float_to_bf16_bits(acc[4]) | ((unsigned)float_to_bf16_bits(acc[5]) << 16);
            o.w = (unsigned)float_to_bf16_bits(acc[6]) | ((unsigned)float_to_bf16_bits(acc[7]) << 16);
        } else {
            o.x = __builtin_bit_cast(unsigned, acc[0]);
            o.y = __builtin_bit_cast(unsigned, acc[1]);
            o.z = __builtin_bit_cast(unsigned, acc[2]);
            o.w = __builtin_bit_cast(unsigned, acc[3]);
        }
        out[(size_t)t * chunks + c] = o;
    }
}

}  // namespace moegps

extern "C" int moe_combine(const void* y_perm, int dtype, int T, int d, int k, const int32_t* row_of_assign,
                           const float* topk_w, void* out, void* stream) {
    using namespace moegps;
    if (dtype != MOE_DTYPE_F32 && dtype != MOE_DTYPE_BF16) return MOE_ERR_INVALID_ARG;
    if (T < 0 || d < 1 || k < 1) return MOE_ERR_INVALID_ARG;
    if (k > MOE_MAX_TOPK) return MOE_ERR_UNSUPPORTED;
    if (((size_t)d * dtype_size(dtype)) % 16 != 0) return MOE_ERR_UNSUPPORTED;
    if (T == 0) return MOE_OK;
    if (!y_perm || !row_of_assign || !topk_w || !out) return MOE_ERR_INVALID_ARG;
    const int chunks = (int)((size_t)d * dtype_size(dtype) / 16);
    hipStream_t st = (hipStream_t)stream;
    if (dtype == MOE_DTYPE_BF16)
        hipLaunchKernelGGL((combine_kernel<true>), dim3(ceil_div(T, 4)), dim3(256), 0, st, (const uint4*)y_perm,
                           row_of_assign, topk_w, (uint4*)out, T, k, chunks);
    else
        hipLaunchKernelGGL((combine_kernel<false>), dim3(ceil_div(T, 4)), dim3(256), 0, st, (const uint4*)y_perm,
                           row_of_assign, topk_w, (uint4*)out, T, k, chunks);
    return check_launch();
}
