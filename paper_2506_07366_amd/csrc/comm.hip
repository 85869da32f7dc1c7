// Rows that cross the emulated expert-parallel ranks (Background, paragraph on the
// communication cost of routing: after the scatter a rank holds a share of the tokens
// wherever their experts are, and the all-to-all after the FFN moves the same rows
// back; Section 3.2.2: with Token-to-Expert prediction a correctly predicted token
// is already on the rank of its expert).  Token t is owned by rank floor(t*G/T).
// dispatch[src, dst] counts assignment rows travelling owner -> rank of their
// segment (a Token-to-Expert assignment whose true expert is among the token's
// predicted ones is in place: src = dst); combine[src, dst] counts rows travelling
// rank of their segment -> owner.  Counts are integer atomics (LDS-privatised per
// workgroup when the G x G tables fit), so the result does not depend on the launch.
#include "common.h"

namespace moegps {

constexpr int kCommThreads = 256;
constexpr int kCommItems = 4096;       // assignments per workgroup
constexpr int kCommLdsRanks = 64;      // G up to which both tables are privatised in LDS

__global__ void comm_zero_kernel(int32_t* __restrict__ a, int32_t* __restrict__ b, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        a[i] = 0;
        b[i] = 0;
    }
}

template <bool LDS_BINS>
__global__ __launch_bounds__(kCommThreads) void comm_count_kernel(int mode, int T, int k, int G, int S,
                                                                   const int32_t* __restrict__ topk_idx,
                                                                   const int32_t* __restrict__ pred_idx,
                                                                   const int32_t* __restrict__ row_of_assign,
                                                                   const int32_t* __restrict__ seg_offsets,
                                                                   int32_t* __restrict__ dispatch,
                                                                   int32_t* __restrict__ combine) {
    __shared__ int so[MOE_MAX_SEGMENTS + 1];
    __shared__ int bins[LDS_BINS ? 2 * kCommLdsRanks * kCommLdsRanks : 1];
    const int nseg = G * S;
    const int GG = G * G;
    for (int i = threadIdx.x; i <= nseg; i += blockDim.x) so[i] = seg_offsets[i];
    if (LDS_BINS)
        for (int i = threadIdx.x; i < 2 * GG; i += blockDim.x) bins[i] = 0;
    __syncthreads();
    const int64_t A = (int64_t)T * k;
    const int64_t lo = (int64_t)blockIdx.x * kCommItems;
    const int64_t hi = lo + kCommItems < A ? lo + kCommItems : A;
    for (int64_t a = lo + threadIdx.x; a < hi; a += blockDim.x) {
        const int t = (int)(a / k);
        const int row = row_of_assign[a];
        // segment sigma with so[sigma] <= row < so[sigma + 1] (empty segments have equal bounds)
        int l = 0, r = nseg;  // invariant: so[l] <= row < so[r]
        while (r - l > 1) {
            const int m = (l + r) >> 1;
            if (so[m] <= row) l = m;
            else r = m;
        }
        const int dst = l / S;
        const int own = (int)(((int64_t)t * G) / T);
        int src = own;
        if (mode == MOE_MODE_TOKEN) {
            const int e = topk_idx[a];
            for (int j = 0; j < k; ++j)
                if (pred_idx[(int64_t)t * k + j] == e) src = dst;
        }
        if (LDS_BINS) {
            atomicAdd(&bins[src * G + dst], 1);
            atomicAdd(&bins[GG + dst * G + own], 1);
        } else {
            atomicAdd(&dispatch[src * G + dst], 1);
            atomicAdd(&combine[dst * G + own], 1);
        }
    }
    if (LDS_BINS) {
        __syncthreads();
        for (int i = threadIdx.x; i < GG; i += blockDim.x) {
            if (bins[i]) atomicAdd(&dispatch[i], bins[i]);
            if (bins[GG + i]) atomicAdd(&combine[i], bins[GG + i]);
        }
    }
}

}  // namespace moegps

extern "C" int moe_comm_matrix(int mode, int T, int k, int G, int S, const int32_t* topk_idx,
                               const int32_t* pred_idx, const int32_t* row_of_assign, const int32_t* seg_offsets,
                               int32_t* dispatch, int32_t* combine, void* stream) {
    using namespace moegps;
    if (mode != MOE_MODE_NONE && mode != MOE_MODE_DISTRIBUTION && mode != MOE_MODE_TOKEN) return MOE_ERR_INVALID_ARG;
    if (T < 0 || k < 1 || G < 1 || S < 1) return MOE_ERR_INVALID_ARG;
    if (k > MOE_MAX_TOPK || G > MOE_MAX_RANKS || S > MOE_MAX_SLOTS || G * S > MOE_MAX_SEGMENTS) return MOE_ERR_UNSUPPORTED;
    if ((int64_t)T * k >= (1ll << 31)) return MOE_ERR_UNSUPPORTED;
    if (!dispatch || !combine) return MOE_ERR_INVALID_ARG;
    if (T > 0 && (!topk_idx || !row_of_assign || !seg_offsets)) return MOE_ERR_INVALID_ARG;
    if (T > 0 && mode == MOE_MODE_TOKEN && !pred_idx) return MOE_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    const int GG = G * G;
    hipLaunchKernelGGL(comm_zero_kernel, dim3(ceil_div(GG, 256)), dim3(256), 0, st, dispatch, combine, GG);
    int rc = check_launch();
    if (rc != MOE_OK || T == 0) return rc;
    const int grid = (int)ceil_div64((int64_t)T * k, kCommItems);
    if (G <= kCommLdsRanks)
        hipLaunchKernelGGL((comm_count_kernel<true>), dim3(grid), dim3(kCommThreads), 0, st, mode, T, k, G, S,
                           topk_idx, pred_idx, row_of_assign, seg_offsets, dispatch, combine);
    else
        hipLaunchKernelGGL((comm_count_kernel<false>), dim3(grid), dim3(kCommThreads), 0, st, mode, T, k, G, S,
                           topk_idx, pred_idx, row_of_assign, seg_offsets, dispatch, combine);
    return check_launch();
}
