// Gate top-k: the token->expert map f of Algorithm 1 (Background: tokens are
// routed to their top-K experts).  A group of LPT lanes of a 64-wide wavefront
// owns one token; every lane keeps VPL logits in registers and the k winners are
// found by k rounds of a cross-lane maximum and a cross-lane minimum over the indices that
// hold it (DPP lane permutes inside a row of 16 lanes; a group is at most one such row up to
// 512 experts).  Order is (logit descending, expert index ascending), so equal logits go to
// the lowest index.
// Gate weights are a softmax over the k selected logits.
#include "common.h"

namespace moegps {

// One butterfly level with a lane permute that stays inside the vector ALU (no LDS
// crossbar): every lane keeps the larger value / the smaller index of itself and its partner.
template <int CTRL>
__device__ __forceinline__ float dpp_max(float v) {
    const float o =
        __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
    return fmaxf(v, o);
}
template <int CTRL>
__device__ __forceinline__ int dpp_min(int e) {
    const int o = __builtin_amdgcn_update_dpp(0, e, CTRL, 0xf, 0xf, false);
    return o < e ? o : e;
}

// Largest value / smallest index of each group of LPT consecutive lanes, known to all its
// lanes.  Inside a row of 16 lanes: quad permutes, then the half-row and row mirrors;
// across rows one or two shuffles.
template <int LPT>
__device__ __forceinline__ float group_max(float v) {
    if constexpr (LPT >= 2) v = dpp_max<0xB1>(v);    // quad_perm [1,0,3,2]
    if constexpr (LPT >= 4) v = dpp_max<0x4E>(v);    // quad_perm [2,3,0,1]
    if constexpr (LPT >= 8) v = dpp_max<0x141>(v);   // row_half_mirror
    if constexpr (LPT >= 16) v = dpp_max<0x140>(v);  // row_mirror
    if constexpr (LPT >= 32) v = fmaxf(v, __shfl_xor(v, 16, kWave));
    if constexpr (LPT == 64) v = fmaxf(v, __shfl_xor(v, 32, kWave));
    return v;
}
template <int LPT>
__device__ __forceinline__ int group_min(int e) {
    if constexpr (LPT >= 2) e = dpp_min<0xB1>(e);
    if constexpr (LPT >= 4) e = dpp_min<0x4E>(e);
    if constexpr (LPT >= 8) e = dpp_min<0x141>(e);
    if constexpr (LPT >= 16) e = dpp_min<0x140>(e);
    if constexpr (LPT >= 32) {
        const int o = __shfl_xor(e, 16, kWave);
        e = o < e ? o : e;
    }
    if constexpr (LPT == 64) {
        const int o = __shfl_xor(e, 32, kWave);
        e = o < e ? o : e;
    }
    return e;
}

// LPT lanes own one token; lane `sub` of the group keeps the VPL consecutive logits
// [sub*VPL, (sub+1)*VPL) in registers, so a token's row is read as one contiguous run
// (16-byte loads where the row layout allows).  With more than 16 experts a group is one
// row of 16 lanes (four tokens per wavefront) and every cross-lane step stays inside the
// vector ALU's lane permutes; only above 512 experts does a group span two rows.
// Lane j of the group keeps winner j; the softmax is taken once at the end, one
// exponential per lane, summed over the group's lanes.
template <int LPT, int VPL>
__global__ __launch_bounds__(256) void route_topk_kernel(const float* __restrict__ logits, int T, int E,
                                                          int k, int32_t* __restrict__ topk_idx,
                                                          float* __restrict__ topk_w) {
    constexpr int TPW = kWave / LPT;  // tokens per wavefront
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) / kWave;
    const int sub = lane % LPT;
    const int token = wave * TPW + lane / LPT;
    const bool live = token < T;
    const int tok = live ? token : (T - 1);  // keep every lane in the lane permutes

    const float NEG_INF = -__builtin_huge_valf();
    float v[VPL];
    const float* row = logits + (size_t)tok * E;
    const int e0 = sub * VPL;
    if ((VPL % 4 == 0) && (E % 4 == 0)) {
        // rows start on 16-byte boundaries and a lane's run is a whole number of 16-byte pieces
#pragma unroll
        for (int i = 0; i < VPL; i += 4) {
            if (e0 + i < E) {
                const float4 q = *(const float4*)(row + e0 + i);
                v[i] = q.x;
                v[i + 1] = q.y;
                v[i + 2] = q.z;
                v[i + 3] = q.w;
            } else {
                v[i] = v[i + 1] = v[i + 2] = v[i + 3] = NEG_INF;
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < VPL; ++i) v[i] = (e0 + i < E) ? row[e0 + i] : NEG_INF;
    }

    // Round j: the largest remaining logit of the group (a lane maximum, then a maximum across
    // the lanes), then the lowest index among the logits that equal it (equal logits go to the
    // lowest expert), then that logit leaves the game as minus infinity.  Padding columns are
    // minus infinity from the start and can only come up once every real logit is gone, which
    // k <= E rules out.
    float l0 = 0.f, my_v = 0.f;
    int my_e = 0;
    for (int j = 0; j < k; ++j) {
        float m = v[0];
#pragma unroll
        for (int i = 1; i < VPL; ++i) m = fmaxf(m, v[i]);
        const float g = group_max<LPT>(m);
        int cand = 0x7fffffff;
#pragma unroll
        for (int i = VPL - 1; i >= 0; --i) cand = (v[i] == g) ? e0 + i : cand;
        const int w = group_min<LPT>(cand);
#pragma unroll
        for (int i = 0; i < VPL; ++i) v[i] = (e0 + i == w) ? NEG_INF : v[i];
        if (j == 0) l0 = g;
        if (sub == j) {
            my_v = g;
            my_e = w;
        }
    }
    const float ex = sub < k ? expf(my_v - l0) : 0.f;
    float sum = ex;
    if constexpr (LPT >= 2) sum += __shfl_xor(sum, 1, kWave);
    if constexpr (LPT >= 4) sum += __shfl_xor(sum, 2, kWave);
    if constexpr (LPT >= 8) sum += __shfl_xor(sum, 4, kWave);
    if constexpr (LPT >= 16) sum += __shfl_xor(sum, 8, kWave);
    if constexpr (LPT >= 32) sum += __shfl_xor(sum, 16, kWave);
    if constexpr (LPT == 64) sum += __shfl_xor(sum, 32, kWave);
    if (live && sub < k) {
        topk_idx[(size_t)token * k + sub] = my_e;
        topk_w[(size_t)token * k + sub] = ex / sum;
    }
}

template <int LPT, int VPL>
static int launch_route(const float* logits, int T, int E, int k, int32_t* idx, float* w, hipStream_t st) {
    constexpr int TPW = kWave / LPT;
    const int tokens_per_block = 4 * TPW;
    const int grid = ceil_div(T, tokens_per_block);
    hipLaunchKernelGGL((route_topk_kernel<LPT, VPL>), dim3(grid), dim3(256), 0, st, logits, T, E, k, idx, w);
    return check_launch();
}

}  // namespace moegps

extern "C" int moe_route_topk(const float* logits, int T, int E, int k, int32_t* topk_idx, float* topk_w,
                              void* stream) {
    using namespace moegps;
    if (T < 0 || E < 1 || k < 1 || k > E) return MOE_ERR_INVALID_ARG;
    if (E > MOE_MAX_EXPERTS || k > MOE_MAX_TOPK) return MOE_ERR_UNSUPPORTED;
    if (T == 0) return MOE_OK;
    if (!logits || !topk_idx || !topk_w) return MOE_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    // lanes per token: the power of two covering E up to one row of 16 lanes, which then
    // holds ceil(E/16) logits per lane; k <= min(E, 16) <= lanes always holds
    if (E <= 2) return launch_route<2, 1>(logits, T, E, k, topk_idx, topk_w, st);
    if (E <= 4) return launch_route<4, 1>(logits, T, E, k, topk_idx, topk_w, st);
    if (E <= 8) return launch_route<8, 1>(logits, T, E, k, topk_idx, topk_w, st);
    if (E <= 16) return launch_route<16, 1>(logits, T, E, k, topk_idx, topk_w, st);
    if (E <= 32) return launch_route<16, 2>(logits, T, E, k, topk_idx, topk_w, st);
    if (E <= 64) return launch_route<16, 4>(logits, T, E, k, topk_idx, topk_w, st);
    if (E <= 128) return launch_route<16, 8>(logits, T, E, k, topk_idx, topk_w, st);
    if (E <= 256) return launch_route<16, 16>(logits, T, E, k, topk_idx, topk_w, st);
    if (E <= 512) return launch_route<16, 32>(logits, T, E, k, topk_idx, topk_w, st);
    return launch_route<32, 32>(logits, T, E, k, topk_idx, topk_w, st);
}
