// Gate top-k: the token->expert map f of Algorithm 1 (Background: tokens are
// routed to their top-K experts).  A group of LPT lanes of a 64-wide wavefront
// owns one token; every lane keeps VPL logits in registers and the k winners are
// found by k rounds of a cross-lane butterfly arg-max.  Order is (logit
// descending, expert index ascending), so equal logits go to the lowest index.
// Gate weights are a softmax over the k selected logits.
#include "common.h"

namespace moegps {

struct Cand {
    float v;
    int e;
};

// true if b comes before a in (value descending, index ascending) order
__device__ __forceinline__ bool better(const Cand& b, const Cand& a) {
    return (b.v > a.v) || (b.v == a.v && b.e < a.e);
}

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
    const int tok = live ? token : (T - 1);  // keep every lane in the shuffles

    const float NEG_INF = -__builtin_huge_valf();
    float v[VPL];
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
        const int e = sub + i * LPT;
        v[i] = (e < E) ? logits[(size_t)tok * E + e] : NEG_INF;
    }

    unsigned taken = 0;
    float l0 = 0.f, sum = 0.f, my_ex = 0.f;
    int my_e = 0;
    for (int j = 0; j < k; ++j) {
        // best remaining candidate of this lane; padding columns carry their own
        // (out of range) index and so lose every tie against a real expert
        Cand best{NEG_INF, 0x7fffffff};
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            Cand c{v[i], sub + i * LPT};
            if (!((taken >> i) & 1u) && better(c, best)) best = c;
        }
#pragma unroll
        for (int m = 1; m < LPT; m <<= 1) {
            Cand o;
            o.v = __shfl_xor(best.v, m, kWave);
            o.e = __shfl_xor(best.e, m, kWave);
            if (better(o, best)) best = o;
        }
        // the owner retires the winner
        if ((best.e % LPT) == sub) taken |= 1u << (best.e / LPT);
        if (j == 0) l0 = best.v;
        const float ex = expf(best.v - l0);
        sum += ex;
        if (sub == j) {
            my_ex = ex;
            my_e = best.e;
        }
    }
    if (live && sub < k) {
        topk_idx[(size_t)token * k + sub] = my_e;
        topk_w[(size_t)token * k + sub] = my_ex / sum;
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
    // lanes per token: the power of two covering E (at most a full wavefront);
    // k <= min(E, 16) <= LPT always holds
    if (E <= 2) return launch_route<2, 1>(logits, T, E, k, topk_idx, topk_w, st);
    if (E <= 4) return launch_route<4, 1>(logits, T, E, k, topk_idx, topk_w, st);
    if (E <= 8) return launch_route<8, 1>(logits, T, E, k, topk_idx, topk_w, st);
    if (E <= 16) return launch_route<16, 1>(logits, T, E, k, topk_idx, topk_w, st);
    if (E <= 32) return launch_route<32, 1>(logits, T, E, k, topk_idx, topk_w, st);
    if (E <= 64) return launch_route<64, 1>(logits, T, E, k, topk_idx, topk_w, st);
    if (E <= 128) return launch_route<64, 2>(logits, T, E, k, topk_idx, topk_w, st);
    if (E <= 256) return launch_route<64, 4>(logits, T, E, k, topk_idx, topk_w, st);
    if (E <= 512) return launch_route<64, 8>(logits, T, E, k, topk_idx, topk_w, st);
    return launch_route<64, 16>(logits, T, E, k, topk_idx, topk_w, st);
}
