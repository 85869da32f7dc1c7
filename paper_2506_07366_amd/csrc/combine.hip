// Weighted un-permute: out[t] = sum_j w[t, j] * y_perm[row_of_assign[t*k + j]].
// Stands where the all-to-all after the expert FFN is (Background, communication
// paragraph: the return shuffle moves as many rows as the dispatch did).
// One wavefront per token (for small batches several, each on its own slice of the
// row); each lane owns 16-byte pieces of the row, gathers the k source rows,
// accumulates in fp32 with j ascending and stores once.
#include "common.h"

namespace moegps {

__device__ __forceinline__ float bf16_bits_to_float(unsigned short b) {
    return __builtin_bit_cast(float, (unsigned)b << 16);
}
__device__ __forceinline__ unsigned short float_to_bf16_bits(float f) {
    return __builtin_bit_cast(unsigned short, (__bf16)f);  // round to nearest even
}

template <bool BF16, int UNROLL>
__global__ __launch_bounds__(256) void combine_kernel(const uint4* __restrict__ y_perm,
                                                       const int32_t* __restrict__ row_of_assign,
                                                       const float* __restrict__ topk_w, uint4* __restrict__ out,
                                                       int T, int k, int chunks, int slices) {
    typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned u32x4;
    const int lane = threadIdx.x & (kWave - 1);
    // wavefront wv serves slice wv % slices of token wv / slices
    const int wv = __builtin_amdgcn_readfirstlane((int)((blockIdx.x * (unsigned)blockDim.x + threadIdx.x) / kWave));
    const int t = wv / slices, slice = wv % slices;
    if (t >= T) return;
    int rows[MOE_MAX_TOPK];
    float w[MOE_MAX_TOPK];
#pragma unroll
    for (int j = 0; j < MOE_MAX_TOPK; ++j) {
        rows[j] = j < k ? row_of_assign[(size_t)t * k + j] : 0;
        w[j] = j < k ? (topk_w ? topk_w[(size_t)t * k + j] : 1.0f) : 0.f;  // no weights: a plain sum (1 * v is exact)
    }
    const u32x4* src = (const u32x4*)y_perm;
    constexpr int N = BF16 ? 8 : 4;
    // UNROLL 16-byte pieces per lane and step keep k * UNROLL row reads in flight; every
    // byte is touched once, so loads and stores are non-temporal
    for (int c0 = lane + slice * kWave * UNROLL; c0 < chunks; c0 += kWave * UNROLL * slices) {
        float acc[UNROLL][N];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
#pragma unroll
            for (int i = 0; i < N; ++i) acc[u][i] = 0.f;
#pragma unroll
        for (int j = 0; j < MOE_MAX_TOPK; ++j) {
            if (j < k) {
                u32x4 v[UNROLL];
#pragma unroll
                for (int u = 0; u < UNROLL; ++u)
                    if (c0 + u * kWave < chunks)
                        v[u] = __builtin_nontemporal_load(src + (size_t)rows[j] * chunks + c0 + u * kWave);
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) {
                    if (c0 + u * kWave < chunks) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const unsigned bits = v[u][i];  // a copy: bit_cast must not see the vector element itself
                            if constexpr (BF16) {
                                acc[u][2 * i] = fmaf(w[j], bf16_bits_to_float((unsigned short)(bits & 0xffffu)),
                                                     acc[u][2 * i]);
                                acc[u][2 * i + 1] = fmaf(w[j], bf16_bits_to_float((unsigned short)(bits >> 16)),
                                                         acc[u][2 * i + 1]);
                            } else {
                                acc[u][i] = fmaf(w[j], __builtin_bit_cast(float, bits), acc[u][i]);
                            }
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            if (c0 + u * kWave < chunks) {
                u32x4 o;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if constexpr (BF16)
                        o[i] = (unsigned)float_to_bf16_bits(acc[u][2 * i]) |
                               ((unsigned)float_to_bf16_bits(acc[u][2 * i + 1]) << 16);
                    else {
                        const float a = acc[u][i];
                        o[i] = __builtin_bit_cast(unsigned, a);
                    }
                }
                __builtin_nontemporal_store(o, (u32x4*)out + (size_t)t * chunks + c0 + u * kWave);
            }
        }
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
    if (!y_perm || !row_of_assign || !out) return MOE_ERR_INVALID_ARG;  // topk_w may be NULL: unweighted sum
    const int chunks = (int)((size_t)d * dtype_size(dtype) / 16);
    hipStream_t st = (hipStream_t)stream;
    // pieces per lane and step: enough 16-byte reads in flight (k * pieces) without running
    // out of registers; rows too short for that many pieces per lane take fewer
    int unroll = k <= 4 ? 4 : (k <= 6 ? 2 : 1);  // measured: 16 reads in flight per lane (k = 8 x 2) is slower than 8
    while (unroll > 1 && chunks < unroll * kWave) unroll >>= 1;
    // a small batch leaves most of the chip idle with one wavefront per token: split the row
    // over several wavefronts until there are a few thousand of them
    int slices = 1;
    while (slices < 16 && (int64_t)T * slices < 4096 && chunks >= 2 * slices * kWave * unroll) slices *= 2;
    auto launch = [&](auto kern) {
        hipLaunchKernelGGL(kern, dim3((unsigned)ceil_div64((int64_t)T * slices, 4)), dim3(256), 0, st,
                           (const uint4*)y_perm, row_of_assign, topk_w, (uint4*)out, T, k, chunks, slices);
    };
    if (dtype == MOE_DTYPE_BF16) {
        if (unroll == 4) launch(combine_kernel<true, 4>);
        else if (unroll == 2) launch(combine_kernel<true, 2>);
        else launch(combine_kernel<true, 1>);
    } else {
        if (unroll == 4) launch(combine_kernel<false, 4>);
        else if (unroll == 2) launch(combine_kernel<false, 2>);
        else launch(combine_kernel<false, 1>);
    }
    return check_launch();
}
