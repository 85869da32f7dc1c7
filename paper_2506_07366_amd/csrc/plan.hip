// Expert duplication planner: Algorithm 1 (Section 3.1) in count-based form, run
// by one 64-wide wavefront.  Two versions: state in registers, one lane per rank
// (G <= 64, further down), and state in LDS for any G (first).  The loop is inherently serial
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

// ---------------------------------------------------------------------------
// Register-resident version for G <= 64: lane g owns rank g (its load and its S
// slots live in registers; the copy count of an expert is a ballot over the lanes).  One iteration
// is a few DPP reductions, ballots and lane reads; there is no barrier.  The
// candidate a lane proposes is its first feasible slot of the hot rank in (rows
// descending, slot ascending) order; the coldest proposing lane wins, which is the
// candidate the serial scan of Algorithm 1 (with the fall-through order of the
// header) reaches first.
// ---------------------------------------------------------------------------
__device__ __forceinline__ int dpp_max_step(int v, int o) { return o > v ? o : v; }
__device__ __forceinline__ int dpp_min_step(int v, int o) { return o < v ? o : v; }

// reduction over the 64 lanes: quads and rows of 16 by DPP lane permutes, the four
// rows by lane reads.  Every lane must be active.
template <bool IS_MAX>
__device__ __forceinline__ int wave_reduce_i32(int v) {
    auto op = [](int a, int b) { return IS_MAX ? dpp_max_step(a, b) : dpp_min_step(a, b); };
    v = op(v, __builtin_amdgcn_update_dpp(v, v, 0xB1, 0xf, 0xf, false));   // quad_perm [1,0,3,2]
    v = op(v, __builtin_amdgcn_update_dpp(v, v, 0x4E, 0xf, 0xf, false));   // quad_perm [2,3,0,1]
    v = op(v, __builtin_amdgcn_update_dpp(v, v, 0x141, 0xf, 0xf, false));  // row_half_mirror
    v = op(v, __builtin_amdgcn_update_dpp(v, v, 0x140, 0xf, 0xf, false));  // row_mirror
    const int r0 = __builtin_amdgcn_readlane(v, 0), r1 = __builtin_amdgcn_readlane(v, 16);
    const int r2 = __builtin_amdgcn_readlane(v, 32), r3 = __builtin_amdgcn_readlane(v, 48);
    return op(op(r0, r1), op(r2, r3));
}

template <int SMAX>
__global__ __launch_bounds__(kWave) void plan_kernel_regs(int mode, const int32_t* __restrict__ hist_pred, int E,
                                                          int G, int S, int c_max,
                                                          int32_t* __restrict__ slot_expert,
                                                          int32_t* __restrict__ slot_quota,
                                                          int32_t* __restrict__ rank_load_pred,
                                                          int32_t* __restrict__ n_iters_out) {
    const int lane = threadIdx.x;
    const bool valid = lane < G;
    const int H = (E + G - 1) / G;
    constexpr int NONE = -2;  // slot index >= S: neither empty nor an expert
    const int IMAX = 0x7fffffff;

    int se[SMAX], q[SMAX];
    int L = 0;
#pragma unroll
    for (int s = 0; s < SMAX; ++s) {
        const int e = lane * H + s;
        const bool home = valid && s < H && e < E;
        se[s] = home ? e : (s < S ? -1 : NONE);
        int n = home ? hist_pred[e] : 0;
        q[s] = n > 0 ? n : 0;
        L += q[s];
    }

    int n_iters = 0;
    if (mode != MOE_MODE_NONE) {
        const int i_max = 16 * G * S;
        while (n_iters < i_max) {
            const int L_h = wave_reduce_i32<true>(valid ? L : -1);
            const int L_min = wave_reduce_i32<false>(valid ? L : IMAX);
            if (L_h - L_min <= 1) break;  // loop guard of Algorithm 1
            const int g_h = __ffsll((unsigned long long)__ballot(valid && L == L_h)) - 1;  // ties -> lowest g

            // lowest empty slot of this lane's rank
            int empty = -1;
#pragma unroll
            for (int t = SMAX - 1; t >= 0; --t)
                if (se[t] == -1) empty = t;

            const bool cand = valid && lane != g_h && (L_h - L > 1);
            int best_q = 0, best_s = 0, best_sp = 0, best_new = 0, best_e = 0;
#pragma unroll
            for (int s = 0; s < SMAX; ++s) {
                const int hq = __builtin_amdgcn_readlane(q[s], g_h);  // rows of the hot rank's slot s
                const int he = __builtin_amdgcn_readlane(se[s], g_h);
                if (hq > 0) {  // uniform
                    int host = -1;
#pragma unroll
                    for (int t = SMAX - 1; t >= 0; --t)
                        if (se[t] == he) host = t;
                    // every rank hosts an expert at most once: copies = number of hosting lanes
                    const int n_copies = __popcll((unsigned long long)__ballot(valid && host >= 0));
                    const bool can_copy = n_copies < c_max && empty >= 0;
                    const bool feasible = host >= 0 || can_copy;
                    if (feasible && hq > best_q) {  // strict: equal rows keep the lower slot
                        best_q = hq;
                        best_s = s;
                        best_sp = host >= 0 ? host : empty;
                        best_new = host < 0;
                        best_e = he;
                    }
                }
            }
            const bool has = cand && best_q > 0;
            const int L_c = wave_reduce_i32<false>(has ? L : IMAX);
            if (L_c == IMAX) break;  // nothing feasible
            const int g_c = __ffsll((unsigned long long)__ballot(has && L == L_c)) - 1;  // ties -> lowest g
            const int s_sel = __builtin_amdgcn_readlane(best_s, g_c);
            const int sp_sel = __builtin_amdgcn_readlane(best_sp, g_c);
            const int new_sel = __builtin_amdgcn_readlane(best_new, g_c);
            const int e_sel = __builtin_amdgcn_readlane(best_e, g_c);
            const int q_sel = __builtin_amdgcn_readlane(best_q, g_c);
            const int delta = (L_h - L_c + 1) / 2;  // ceil((L_h - L_c) / 2)
            const int m = delta < q_sel ? delta : q_sel;
            if (lane == g_h) {
#pragma unroll
                for (int t = 0; t < SMAX; ++t)
                    if (t == s_sel) q[t] -= m;
                L -= m;
            }
            if (lane == g_c) {
#pragma unroll
                for (int t = 0; t < SMAX; ++t)
                    if (t == sp_sel) {
                        q[t] += m;
                        if (new_sel) se[t] = e_sel;  // copy weights of e* on g_c
                    }
                L += m;
            }
            ++n_iters;
        }
    }
    if (valid) {
#pragma unroll
        for (int s = 0; s < SMAX; ++s)
            if (s < S) {
                slot_expert[lane * S + s] = se[s];
                slot_quota[lane * S + s] = q[s];
            }
        rank_load_pred[lane] = L;
    }
    if (lane == 0) n_iters_out[0] = n_iters;
}

}  // namespace moegps

extern "C" int moe_plan_duplicates(int mode, const int32_t* hist_pred, int E, int G, int S, int c_max,
                                   int32_t* slot_expert, int32_t* slot_quota, int32_t* rank_load_pred,
                                   int32_t* n_iters, void* stream) {
    using namespace moegps;
    if (mode < MOE_MODE_NONE || mode > MOE_MODE_TOKEN) return MOE_ERR_INVALID_ARG;
    if (E < 1 || G < 1 || S < 1 || c_max < 1) return MOE_ERR_INVALID_ARG;
    if (ceil_div(E, G) > S) return MOE_ERR_INVALID_ARG;  // every expert needs a home slot
    if (E > MOE_MAX_EXPERTS || G > MOE_MAX_RANKS || S > MOE_MAX_SLOTS || G * S > MOE_MAX_SEGMENTS)
        return MOE_ERR_UNSUPPORTED;
    if (!hist_pred || !slot_expert || !slot_quota || !rank_load_pred || !n_iters) return MOE_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    if (G <= kWave) {
        // one lane per rank, state in registers
        auto launch = [&](auto kern) {
            hipLaunchKernelGGL(kern, dim3(1), dim3(kWave), 0, st, mode, hist_pred, E, G, S, c_max, slot_expert,
                               slot_quota, rank_load_pred, n_iters);
        };
        // one instantiation per slot count: every loop over a rank's slots is unrolled to exactly S
        switch (S) {
            case 1: launch(plan_kernel_regs<1>); break;
            case 2: launch(plan_kernel_regs<2>); break;
            case 3: launch(plan_kernel_regs<3>); break;
            case 4: launch(plan_kernel_regs<4>); break;
            case 5: launch(plan_kernel_regs<5>); break;
            case 6: launch(plan_kernel_regs<6>); break;
            case 7: launch(plan_kernel_regs<7>); break;
            case 8: launch(plan_kernel_regs<8>); break;
            case 9: launch(plan_kernel_regs<9>); break;
            case 10: launch(plan_kernel_regs<10>); break;
            case 11: launch(plan_kernel_regs<11>); break;
            case 12: launch(plan_kernel_regs<12>); break;
            case 13: launch(plan_kernel_regs<13>); break;
            case 14: launch(plan_kernel_regs<14>); break;
            case 15: launch(plan_kernel_regs<15>); break;
            default: launch(plan_kernel_regs<16>); break;
        }
        return check_launch();
    }
    hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(kWave), 0, st, mode, hist_pred, E, G, S, c_max, slot_expert,
                       slot_quota, rank_load_pred, n_iters);
    return check_launch();
}
