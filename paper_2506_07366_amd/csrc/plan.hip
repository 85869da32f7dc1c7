// Expert duplication planner: Algorithm 1 (Section 3.1) in count-based form, run
// by one 64-wide wavefront with all state in LDS.  The loop is inherently serial
// (each move changes the loads the next one looks at); inside one iteration the
// wavefront evaluates every candidate cold rank in parallel and a cross-lane
// arg-min picks the coldest feasible one, which is exactly the candidate the
// serial scan "coldest rank first, hottest expert first" would reach first.
//
// State per slot sigma = g*S + s: hosted expert (-1 = empty) and planned rows.
// Ties (hottest rank, coldest rank, hottest expert) go to the lowest index.
#include "common.h"

namespace moegps {

__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long v) {
#pragma unroll
    for (int m = 1; m < kWave; m <<= 1) {
        unsigned long long o = __shfl_xor(v, m, kWave);
        v = o > v ? o : v;
    }
    return v;
}
__device__ __forceinline__ unsigned long long wave_min_u64(unsigned long long v) {
#pragma unroll
    for (int m = 1; m < kWave; m <<= 1) {
        unsigned long long o = __shfl_xor(v, m, kWave);
        v = o < v ? o : v;
    }
    return v;
}

__global__ __launch_bounds__(kWave) void plan_kernel(int mode, const int32_t* __restrict__ hist_pred, int E, int G,
                                                     int S, int c_max, int32_t* __restrict__ slot_expert,
                                                     int32_t* __restrict__ slot_quota,
                                                     int32_t* __restrict__ rank_load_pred,
                                                     int32_t* __restrict__ n_iters_out) {
    __shared__ int se[MOE_MAX_SEGMENTS];   // expert per slot
    __shared__ int q[MOE_MAX_SEGMENTS];    // planned rows per slot
    __shared__ int L[MOE_MAX_RANKS];       // planned rows per rank
    __shared__ int copies[MOE_MAX_EXPERTS];
    __shared__ int hot_ord[MOE_MAX_SLOTS];  // slots of the hot rank, hottest expert first
    __shared__ int n_hot_s;

    const int lane = threadIdx.x;
    const int nseg = G * S;
    const int H = (E + G - 1) / G;

    for (int s = lane; s < nseg; s += kWave) {
        se[s] = -1;
        q[s] = 0;
    }
    __syncthreads();
    // home placement; every predicted token starts on the only host of its expert
    for (int e = lane; e < E; e += kWave) {
        const int sigma = (e / H) * S + (e % H);
        se[sigma] = e;
        int n = hist_pred[e];
        q[sigma] = n > 0 ? n : 0;
        copies[e] = 1;
    }
    __syncthreads();
    for (int g = lane; g < G; g += kWave) {
        int sum = 0;
        for (int s = 0; s < S; ++s) sum += q[g * S + s];
        L[g] = sum;
    }
    __syncthreads();

    int n_iters = 0;
    if (mode != MOE_MODE_NONE) {
        const int i_max = 16 * nseg;
        while (n_iters < i_max) {
            // hottest rank (ties -> lowest g) and the smallest load
            unsigned long long kmax = 0ull, kmin = ~0ull;
            for (int g = lane; g < G; g += kWave) {
                const unsigned long long l = (unsigned long long)(unsigned)L[g];
                const unsigned long long hi = (l << 32) | (unsigned)(0xffffffffu - (unsigned)g);
                const unsigned long long lo = (l << 32) | (unsigned)g;
                kmax = hi > kmax ? hi : kmax;
                kmin = lo < kmin ? lo : kmin;
            }
            kmax = wave_max_u64(kmax);
            kmin = wave_min_u64(kmin);
            const int g_h = (int)(0xffffffffu - (unsigned)(kmax & 0xffffffffull));
            const int L_h = (int)(kmax >> 32);
            const int L_min = (int)(kmin >> 32);
            if (L_h - L_min <= 1) break;  // loop guard of Algorithm 1

            // slots of g_h with tokens, ordered by (rows descending, slot ascending)
            if (lane == 0) n_hot_s = 0;
            __syncthreads();
            if (lane < S) {
                const int mine = q[g_h * S + lane];
                if (mine > 0) {
                    int r = 0;
                    for (int s = 0; s < S; ++s) {
                        const int o = q[g_h * S + s];
                        if (o > mine || (o == mine && s < lane)) ++r;
                    }
                    hot_ord[r] = lane;
                    atomicAdd(&n_hot_s, 1);
                }
            }
            __syncthreads();
            const int n_hot = n_hot_s;

            // every lane tries cold ranks g_c = lane, lane+64, ...; for each it takes
            // the first feasible slot of g_h in hot order
            unsigned long long best = ~0ull;  // (L_c, g_c) packed, smaller is colder
            int best_s = -1, best_sp = -1, best_new = 0;
            for (int g_c = lane; g_c < G; g_c += kWave) {
                if (g_c == g_h) continue;
                const int L_c = L[g_c];
                if (L_h - L_c <= 1) continue;
                int f_s = -1, f_sp = -1, f_new = 0;
                for (int r = 0; r < n_hot && f_s < 0; ++r) {
                    const int s = hot_ord[r];
                    const int e = se[g_h * S + s];
                    int host = -1, empty = -1;
                    for (int sp = S - 1; sp >= 0; --sp) {
                        const int o = se[g_c * S + sp];
                        if (o == e) host = sp;
                        if (o < 0) empty = sp;
                    }
                    if (host >= 0) {
                        f_s = s;
                        f_sp = host;
                        f_new = 0;
                    } else if (copies[e] < c_max && empty >= 0) {
                        f_s = s;
                        f_sp = empty;
                        f_new = 1;
                    }
                }
                if (f_s >= 0) {
                    const unsigned long long key = ((unsigned long long)(unsigned)L_c << 32) | (unsigned)g_c;
                    if (key < best) {
                        best = key;
                        best_s = f_s;
                        best_sp = f_sp;
                        best_new = f_new;
                    }
                }
            }
            const unsigned long long win = wave_min_u64(best);
            if (win == ~0ull) break;  // nothing feasible
            // the lane that holds the winner applies the move
            if (best == win) {
                const int g_c = (int)(win & 0xffffffffull);
                const int L_c = (int)(win >> 32);
                const int from = g_h * S + best_s;
                const int to = g_c * S + best_sp;
                const int e = se[from];
                if (best_new) {  // copy weights of e* on g_c
                    se[to] = e;
                    copies[e] += 1;
                }
                const int delta = (L_h - L_c + 1) / 2;  // ceil((L_h - L_c) / 2)
                const int m = delta < q[from] ? delta : q[from];
                q[from] -= m;
                q[to] += m;
                L[g_h] = L_h - m;
                L[g_c] = L_c + m;
            }
            __syncthreads();
            ++n_iters;
        }
    }
    __syncthreads();
    for (int s = lane; s < nseg; s += kWave) {
        slot_expert[s] = se[s];
        slot_quota[s] = q[s];
    }
    for (int g = lane; g < G; g += kWave) rank_load_pred[g] = L[g];
    if (lane == 0) n_iters_out[0] = n_iters;
}

}  // namespace moegps

extern "C" int moe_plan_duplicates(int mode, const int32_t* hist_pred, int E, int G, int S, int c_max,
                                   int32_t* slot_expert, int32_t* slot_quota, int32_t* rank_load_pred,
                                   int32_t* n_iters, void* stream) {
    using namespace moegps;
    if (mode < MOE_MODE_NONE || mode > MOE_MODE_TOKEN) return MOE_ERR_INVALID_ARG;
    if (E < 1 || G < 1 || S < 1 || c_max < 1) return MOE_ERR_INVALID_ARG;
    if ((E + G - 1) / G > S) return MOE_ERR_INVALID_ARG;  // every expert needs a home slot
    if (E > MOE_MAX_EXPERTS || G > MOE_MAX_RANKS || S > MOE_MAX_SLOTS || G * S > MOE_MAX_SEGMENTS)
        return MOE_ERR_UNSUPPORTED;
    if (!hist_pred || !slot_expert || !slot_quota || !rank_load_pred || !n_iters) return MOE_ERR_INVALID_ARG;
    hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(kWave), 0, (hipStream_t)stream, mode, hist_pred, E, G, S, c_max,
                       slot_expert, slot_quota, rank_load_pred, n_iters);
    return check_launch();
}
