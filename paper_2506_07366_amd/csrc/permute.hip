// Dispatch of assignments to replica segments and the token permutation: the
// dispatch d of Algorithm 1 for a given plan, standing where the all-to-all
// before the expert FFN is (Background, paragraph on the communication cost of
// routing).
//
// Everything is a deterministic stable counting sort, built from one primitive:
// the stable rank of an element among equal keys.  A workgroup owns a contiguous
// chunk of tokens; inside the chunk ranks come from wavefront ballots, across
// chunks from an exclusive scan of per-chunk key counts.  No atomics decide any
// position, so the permutation is identical for every launch.
//
//   count    : per-chunk histogram of the dispatch keys (expert ids)
//   scan1    : chunk bases per expert; per-expert replica tables from the plan
//   segment  : stable rank -> replica -> segment id; per-chunk segment histogram
//   scan2    : chunk bases per segment, seg_offsets, rank_load
//   place    : row_of_assign / assign_of_row
//   scatter  : each token row is read once and written to its k rows of x_perm
#include "common.h"
#include "block_scan.h"
#include <mutex>

namespace moegps {

constexpr int kPermThreads = 256;
constexpr int kPermWaves = kPermThreads / kWave;
constexpr int kRounds = 8;                                  // 64-element rounds per wavefront
constexpr int kChunk = kPermThreads * kRounds;              // max elements per workgroup (2048)
constexpr int kMaxKeys = MOE_MAX_SEGMENTS;                  // >= MOE_MAX_EXPERTS

__host__ __device__ inline int tokens_per_chunk(int k) { return kChunk / k > 0 ? kChunk / k : 1; }

struct PermWs {
    int32_t* bh1;       // [nb, E]    per-chunk expert counts -> chunk bases
    int32_t* bh2;       // [nb, NSEG] per-chunk segment counts -> chunk bases
    int32_t* seg;       // [A]        segment of each assignment
    int32_t* rep_cnt;   // [E]        replicas per expert (0 = everything to the home slot)
    int32_t* rep_slot;  // [E, G]     replica slots, ascending
    int32_t* rep_hi;    // [E, G]     exclusive upper bound of each replica's rank range
};

static size_t perm_ws_layout(int T, int E, int k, int G, int S, char* base, PermWs* ws) {
    const int nb = ceil_div(T > 0 ? T : 1, tokens_per_chunk(k));
    size_t off = 0;
    auto take = [&](size_t n_int) {
        int32_t* p = base ? (int32_t*)(base + off) : nullptr;
        off += align_up(n_int * sizeof(int32_t), 256);
        return p;
    };
    PermWs w;
    w.bh1 = take((size_t)nb * E);
    w.bh2 = take((size_t)nb * G * S);
    w.seg = take((size_t)T * k);
    w.rep_cnt = take(E);
    w.rep_slot = take((size_t)E * G);
    w.rep_hi = take((size_t)E * G);
    if (ws) *ws = w;
    return off;
}

__device__ __forceinline__ int clamp_key(int v, int n) { return v < 0 ? 0 : (v >= n ? n - 1 : v); }

__device__ __forceinline__ int home_slot_of(int e, int H, int S) { return (e / H) * S + (e % H); }

// ---------------------------------------------------------------------------
// Stable rank of every element of a chunk among equal keys earlier in the chunk.
// Wavefront w owns elements [w*512, (w+1)*512) of the chunk in kRounds rounds of
// 64; element p of the chunk is (w, r, lane) with p = w*512 + r*64 + lane.
// wcnt is LDS scratch of kPermWaves*nkeys ints.  On return rank[r] holds the
// rank, and (if chunk_hist) chunk_hist[key] the chunk's count per key.
// ---------------------------------------------------------------------------
__device__ void chunk_stable_rank(const int (&key)[kRounds], const bool (&valid)[kRounds], int nkeys, int* wcnt,
                                  int (&rank)[kRounds], int32_t* chunk_hist) {
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int w = tid / kWave;
    for (int i = tid; i < kPermWaves * nkeys; i += kPermThreads) wcnt[i] = 0;
    __syncthreads();
    int nbits = 1;
    while ((1 << nbits) < nkeys) ++nbits;
    const unsigned long long lt = (1ull << lane) - 1ull;
    int* mine = wcnt + w * nkeys;
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        // lanes of this round holding the same key
        unsigned long long same = __ballot(valid[r]);
        for (int b = 0; b < nbits; ++b) {
            const bool bit = (key[r] >> b) & 1;
            const unsigned long long m = __ballot(valid[r] && bit);
            same &= bit ? m : ~m;
        }
        rank[r] = 0;
        if (valid[r]) {
            const int prior = mine[key[r]];
            rank[r] = prior + __popcll(same & lt);
            if ((same & lt) == 0ull) mine[key[r]] = prior + __popcll(same);  // leader
        }
    }
    __syncthreads();
    // exclusive prefix over the wavefronts, per key
    for (int kk = tid; kk < nkeys; kk += kPermThreads) {
        int run = 0;
#pragma unroll
        for (int ww = 0; ww < kPermWaves; ++ww) {
            const int c = wcnt[ww * nkeys + kk];
            wcnt[ww * nkeys + kk] = run;
            run += c;
        }
        if (chunk_hist) chunk_hist[kk] = run;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kRounds; ++r)
        if (valid[r]) rank[r] += mine[key[r]];
}

// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kPermThreads) void perm_count_kernel(const int32_t* __restrict__ keys, int T, int k,
                                                                   int E, int32_t* __restrict__ bh1) {
    __shared__ int bins[MOE_MAX_EXPERTS];
    const int tpc = tokens_per_chunk(k);
    const int64_t lo = (int64_t)blockIdx.x * tpc * k;
    const int64_t A = (int64_t)T * k;
    const int64_t hi = lo + (int64_t)tpc * k < A ? lo + (int64_t)tpc * k : A;
    for (int e = threadIdx.x; e < E; e += blockDim.x) bins[e] = 0;
    __syncthreads();
    for (int64_t i = lo + threadIdx.x; i < hi; i += blockDim.x) atomicAdd(&bins[clamp_key(keys[i], E)], 1);
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += blockDim.x) bh1[(size_t)blockIdx.x * E + e] = bins[e];
}

// inclusive prefix sum over the 64 lanes of a wavefront (every lane active)
__device__ __forceinline__ long long wave_incl_scan(long long v) {
    const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int m = 1; m < kWave; m <<= 1) {
        const long long o = __shfl_up(v, m, kWave);
        if (lane >= m) v += o;
    }
    return v;
}

// inclusive prefix sum of 32-bit counts over the 64 lanes of a wavefront
__device__ __forceinline__ int wave_incl_scan_i32(int v) {
    const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int m = 1; m < kWave; m <<= 1) {
        const int o = __shfl_up(v, m, kWave);
        if (lane >= m) v += o;
    }
    return v;
}

// In-place exclusive scan down NC neighbouring columns (col0 .. col0 + NC - 1, those
// below ncols) of a [nb, ncols] table by one wavefront: lanes take consecutive rows, the
// NC loads of a step are independent and go out together.  total[i] = column sums.
template <int NC>
__device__ __forceinline__ void wave_columns_scan(int32_t* table, int nb, int ncols, int col0, int total[NC]) {
    const int lane = threadIdx.x & (kWave - 1);
    int carry[NC];
#pragma unroll
    for (int i = 0; i < NC; ++i) carry[i] = 0;
    for (int b0 = 0; b0 < nb; b0 += kWave) {
        const int b = b0 + lane;
        int c[NC], incl[NC];
#pragma unroll
        for (int i = 0; i < NC; ++i) c[i] = (b < nb && col0 + i < ncols) ? table[(size_t)b * ncols + col0 + i] : 0;
#pragma unroll
        for (int i = 0; i < NC; ++i) incl[i] = wave_incl_scan_i32(c[i]);
#pragma unroll
        for (int i = 0; i < NC; ++i) {
            if (b < nb && col0 + i < ncols) table[(size_t)b * ncols + col0 + i] = carry[i] + incl[i] - c[i];
            carry[i] += __shfl(incl[i], kWave - 1, kWave);
        }
    }
#pragma unroll
    for (int i = 0; i < NC; ++i) total[i] = carry[i];
}

// chunk bases per expert (in place) and the replica tables of the plan; one
// wavefront per expert column, columns dealt over the whole grid
constexpr int kScan1Threads = 256;
__global__ __launch_bounds__(kScan1Threads) void perm_scan1_kernel(int mode, int nb, int E, int G, int S,
                                                           const int32_t* __restrict__ hist_true,
                                                           const int32_t* __restrict__ hist_pred,
                                                           const int32_t* __restrict__ slot_expert,
                                                           const int32_t* __restrict__ slot_quota, PermWs ws) {
    const int nseg = G * S;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave, nwaves = blockDim.x / kWave;
    const unsigned long long lt = (1ull << lane) - 1ull;
    for (int e = blockIdx.x * nwaves + wave; e < E; e += gridDim.x * nwaves) {
        int unused[1];
        wave_columns_scan<1>(ws.bh1, nb, E, e, unused);
        // replicas of e in ascending slot id with the upper bound of their range
        long long n_true = 0, n_hat = 0;
        if (mode == MOE_MODE_DISTRIBUTION) {
            n_true = hist_true[e];
            n_hat = hist_pred[e];
        }
        int cnt = 0;
        long long cum = 0;
        if (!(mode == MOE_MODE_DISTRIBUTION && n_hat <= 0)) {
            for (int s0 = 0; s0 < nseg; s0 += kWave) {
                const int sigma = s0 + lane;
                const bool match = sigma < nseg && slot_expert[sigma] == e;
                const long long qv = match ? (long long)slot_quota[sigma] : 0ll;
                const long long incl = wave_incl_scan(qv);
                const unsigned long long m = __ballot(match);
                const int pos = cnt + __popcll(m & lt);
                if (match && pos < G) {
                    long long hi = cum + incl;                                       // Q_{r+1}
                    if (mode == MOE_MODE_DISTRIBUTION) hi = (n_true * hi) / n_hat;   // floor(n_e * Q / nhat_e)
                    if (hi > 0x7fffffffLL) hi = 0x7fffffffLL;
                    ws.rep_slot[(size_t)e * G + pos] = sigma;
                    ws.rep_hi[(size_t)e * G + pos] = (int)hi;
                }
                cnt += __popcll(m);
                cum += __shfl(incl, kWave - 1, kWave);
            }
        }
        if (lane == 0) ws.rep_cnt[e] = cnt < G ? cnt : G;
    }
}

// segment id per assignment + per-chunk segment histogram
__global__ __launch_bounds__(kPermThreads) void perm_segment_kernel(int mode, int T, int k, int E, int G, int S,
                                                                     const int32_t* __restrict__ topk_idx,
                                                                     const int32_t* __restrict__ pred_idx,
                                                                     PermWs ws) {
    __shared__ int wcnt[kPermWaves * MOE_MAX_EXPERTS];
    __shared__ int prank[kChunk];
    __shared__ int seg_bins[MOE_MAX_SEGMENTS];
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int w = tid / kWave;
    const int nseg = G * S;
    const int H = (E + G - 1) / G;
    const int tpc = tokens_per_chunk(k);
    const int64_t A = (int64_t)T * k;
    const int64_t base = (int64_t)blockIdx.x * tpc * k;
    const int n_b = (int)((base + (int64_t)tpc * k < A ? base + (int64_t)tpc * k : A) - base);

    for (int s = tid; s < nseg; s += kPermThreads) seg_bins[s] = 0;

    int key[kRounds], rank[kRounds];
    bool valid[kRounds];
    const int32_t* rank_keys = (mode == MOE_MODE_TOKEN) ? pred_idx : topk_idx;
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int p = w * (kRounds * kWave) + r * kWave + lane;
        valid[r] = p < n_b;
        key[r] = valid[r] ? clamp_key(rank_keys[base + p], E) : 0;
        rank[r] = 0;
    }
    if (mode != MOE_MODE_NONE) {
        chunk_stable_rank(key, valid, E, wcnt, rank, nullptr);
#pragma unroll
        for (int r = 0; r < kRounds; ++r) {
            const int p = w * (kRounds * kWave) + r * kWave + lane;
            if (valid[r]) prank[p] = ws.bh1[(size_t)blockIdx.x * E + key[r]] + rank[r];
        }
    }
    __syncthreads();

#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int p = w * (kRounds * kWave) + r * kWave + lane;
        if (!valid[r]) continue;
        const int e = clamp_key(topk_idx[base + p], E);
        int i = -1;  // place of this assignment in the plan's order for expert e
        if (mode == MOE_MODE_DISTRIBUTION) {
            i = prank[p];
        } else if (mode == MOE_MODE_TOKEN) {
            const int row0 = (p / k) * k;  // the token's predicted ids
            for (int jp = 0; jp < k; ++jp) {
                if (clamp_key(pred_idx[base + row0 + jp], E) == e) {
                    i = prank[row0 + jp];
                    break;
                }
            }
        }
        int sg = home_slot_of(e, H, S);
        const int cnt = ws.rep_cnt[e];
        if (i >= 0 && cnt > 0) {
            int rr = 0;
            while (rr < cnt - 1 && i >= ws.rep_hi[(size_t)e * G + rr]) ++rr;
            sg = ws.rep_slot[(size_t)e * G + rr];
        }
        ws.seg[base + p] = sg;
        atomicAdd(&seg_bins[sg], 1);
    }
    __syncthreads();
    for (int s = tid; s < nseg; s += kPermThreads) ws.bh2[(size_t)blockIdx.x * nseg + s] = seg_bins[s];
}

// chunk bases per segment (in place), seg_offsets, rank_load
__global__ __launch_bounds__(1024) void perm_scan2_kernel(int nb, int G, int S, PermWs ws,
                                                           int32_t* __restrict__ seg_offsets,
                                                           int32_t* __restrict__ rank_load) {
    __shared__ int tot[MOE_MAX_SEGMENTS + 1];
    __shared__ int wave_sum[16];
    const int nseg = G * S;
    const int tid = threadIdx.x;
    const int wave = tid / kWave, nwaves = blockDim.x / kWave;
    constexpr int NC = 4;  // neighbouring segment columns one wavefront scans together
    for (int s0 = wave * NC; s0 < nseg; s0 += nwaves * NC) {
        int total[NC];
        wave_columns_scan<NC>(ws.bh2, nb, nseg, s0, total);
        if ((tid & (kWave - 1)) == 0) {
#pragma unroll
            for (int i = 0; i < NC; ++i)
                if (s0 + i < nseg) tot[s0 + i] = total[i];
        }
    }
    __syncthreads();
    block_exclusive_scan_2048(tot, nseg, wave_sum);
    for (int s = tid; s <= nseg; s += blockDim.x) seg_offsets[s] = tot[s];
    for (int g = tid; g < G; g += blockDim.x) rank_load[g] = tot[(g + 1) * S] - tot[g * S];
}

// final position of every assignment
__global__ __launch_bounds__(kPermThreads) void perm_place_kernel(int T, int k, int G, int S, PermWs ws,
                                                                   const int32_t* __restrict__ seg_offsets,
                                                                   int32_t* __restrict__ row_of_assign,
                                                                   int32_t* __restrict__ assign_of_row) {
    __shared__ int wcnt[kPermWaves * kMaxKeys];
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int w = tid / kWave;
    const int nseg = G * S;
    const int tpc = tokens_per_chunk(k);
    const int64_t A = (int64_t)T * k;
    const int64_t base = (int64_t)blockIdx.x * tpc * k;
    const int n_b = (int)((base + (int64_t)tpc * k < A ? base + (int64_t)tpc * k : A) - base);
    int key[kRounds], rank[kRounds];
    bool valid[kRounds];
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int p = w * (kRounds * kWave) + r * kWave + lane;
        valid[r] = p < n_b;
        key[r] = valid[r] ? ws.seg[base + p] : 0;
    }
    chunk_stable_rank(key, valid, nseg, wcnt, rank, nullptr);
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int p = w * (kRounds * kWave) + r * kWave + lane;
        if (!valid[r]) continue;
        const int row = seg_offsets[key[r]] + ws.bh2[(size_t)blockIdx.x * nseg + key[r]] + rank[r];
        row_of_assign[base + p] = row;
        assign_of_row[row] = (int)(base + p);
    }
}

// x_perm[row_of_assign[t*k + j], :] = x[t, :]: one wavefront per token, the row is
// read once (16 bytes per lane per piece, UNROLL pieces in flight) and stored to its k
// destinations.
template <int UNROLL>
__global__ __launch_bounds__(256) void perm_scatter_rows_kernel(const uint4* __restrict__ x,
                                                                 uint4* __restrict__ x_perm,
                                                                 const int32_t* __restrict__ row_of_assign, int T,
                                                                 int k, int chunks, int slices) {
    typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned u32x4;
    const int lane = threadIdx.x & (kWave - 1);
    // wavefront wv serves slice wv % slices of token wv / slices (several per token only for small batches)
    const int wv = __builtin_amdgcn_readfirstlane((int)((blockIdx.x * (unsigned)blockDim.x + threadIdx.x) / kWave));
    const int t = wv / slices, slice = wv % slices;
    if (t >= T) return;
    int rows[MOE_MAX_TOPK];
#pragma unroll
    for (int j = 0; j < MOE_MAX_TOPK; ++j) rows[j] = j < k ? row_of_assign[(size_t)t * k + j] : 0;
    const u32x4* src = (const u32x4*)x + (size_t)t * chunks;
    u32x4* dst = (u32x4*)x_perm;
    for (int c0 = lane + slice * kWave * UNROLL; c0 < chunks; c0 += kWave * UNROLL * slices) {
        u32x4 v[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
            if (c0 + u * kWave < chunks) v[u] = src[c0 + u * kWave];
#pragma unroll
        for (int j = 0; j < MOE_MAX_TOPK; ++j)
            if (j < k) {
#pragma unroll
                for (int u = 0; u < UNROLL; ++u)
                    if (c0 + u * kWave < chunks) dst[(size_t)rows[j] * chunks + c0 + u * kWave] = v[u];
            }
    }
}

}  // namespace moegps

extern "C" size_t moe_permute_workspace_bytes(int T, int E, int k, int G, int S) {
    using namespace moegps;
    if (T < 0 || E < 1 || k < 1 || G < 1 || S < 1) return 0;
    if (E > MOE_MAX_EXPERTS || k > MOE_MAX_TOPK || G > MOE_MAX_RANKS || S > MOE_MAX_SLOTS || G * S > MOE_MAX_SEGMENTS ||
        (int64_t)T * k >= (1ll << 31))
        return 0;
    return perm_ws_layout(T, E, k, G, S, nullptr, nullptr);
}

namespace moegps {
static int permute_impl(int mode, const void* x, int dtype, int T, int d, int E, int k, int G, int S,
                        const int32_t* topk_idx, const int32_t* pred_idx, const int32_t* hist_true,
                        const int32_t* hist_pred, const int32_t* slot_expert, const int32_t* slot_quota,
                        int32_t* seg_offsets, int32_t* row_of_assign, int32_t* assign_of_row, void* x_perm,
                        int32_t* rank_load, void* workspace, size_t workspace_bytes, void* stream) {
    if (mode < MOE_MODE_NONE || mode > MOE_MODE_TOKEN) return MOE_ERR_INVALID_ARG;
    if (dtype != MOE_DTYPE_F32 && dtype != MOE_DTYPE_BF16) return MOE_ERR_INVALID_ARG;
    if (T < 0 || d < 1 || E < 1 || k < 1 || k > E || G < 1 || S < 1) return MOE_ERR_INVALID_ARG;
    if (E > MOE_MAX_EXPERTS || k > MOE_MAX_TOPK || G > MOE_MAX_RANKS || S > MOE_MAX_SLOTS ||
        G * S > MOE_MAX_SEGMENTS)
        return MOE_ERR_UNSUPPORTED;
    if (ceil_div(E, G) > S) return MOE_ERR_INVALID_ARG;
    if ((int64_t)T * k >= (1ll << 31)) return MOE_ERR_UNSUPPORTED;
    if (((size_t)d * dtype_size(dtype)) % 16 != 0) return MOE_ERR_UNSUPPORTED;
    if (!seg_offsets || !rank_load || !slot_expert || !slot_quota || !workspace) return MOE_ERR_INVALID_ARG;
    if (T > 0 && (!topk_idx || !row_of_assign || !assign_of_row)) return MOE_ERR_INVALID_ARG;
    if (mode == MOE_MODE_TOKEN && T > 0 && !pred_idx) return MOE_ERR_INVALID_ARG;
    if (mode == MOE_MODE_DISTRIBUTION && (!hist_true || !hist_pred)) return MOE_ERR_INVALID_ARG;
    if (x_perm && T > 0 && !x) return MOE_ERR_INVALID_ARG;
    PermWs ws;
    const size_t need = perm_ws_layout(T, E, k, G, S, (char*)workspace, &ws);
    if (workspace_bytes < need) return MOE_ERR_WORKSPACE_TOO_SMALL;

    hipStream_t st = (hipStream_t)stream;
    const int nb = T > 0 ? ceil_div(T, tokens_per_chunk(k)) : 0;
    int rc;
    if (nb > 0 && mode != MOE_MODE_NONE) {
        const int32_t* keys = (mode == MOE_MODE_TOKEN) ? pred_idx : topk_idx;
        hipLaunchKernelGGL(perm_count_kernel, dim3(nb), dim3(kPermThreads), 0, st, keys, T, k, E, ws.bh1);
        if ((rc = check_launch()) != MOE_OK) return rc;
    }
    if (mode != MOE_MODE_NONE) {
        hipLaunchKernelGGL(perm_scan1_kernel, dim3(ceil_div(E, kScan1Threads / kWave)), dim3(kScan1Threads), 0, st,
                           mode, nb, E, G, S, hist_true, hist_pred, slot_expert, slot_quota, ws);
        if ((rc = check_launch()) != MOE_OK) return rc;
    }
    if (nb > 0) {
        hipLaunchKernelGGL(perm_segment_kernel, dim3(nb), dim3(kPermThreads), 0, st, mode, T, k, E, G, S, topk_idx,
                           pred_idx, ws);
        if ((rc = check_launch()) != MOE_OK) return rc;
    }
    hipLaunchKernelGGL(perm_scan2_kernel, dim3(1), dim3(1024), 0, st, nb, G, S, ws, seg_offsets, rank_load);
    if ((rc = check_launch()) != MOE_OK) return rc;
    if (nb > 0) {
        hipLaunchKernelGGL(perm_place_kernel, dim3(nb), dim3(kPermThreads), 0, st, T, k, G, S, ws, seg_offsets,
                           row_of_assign, assign_of_row);
        if ((rc = check_launch()) != MOE_OK) return rc;
        if (x_perm) {
            const int chunks = (int)((size_t)d * dtype_size(dtype) / 16);
            const int unroll = chunks >= 4 * kWave ? 4 : 1;
            // a small batch: split every row over several wavefronts until there are a few thousand
            int slices = 1;
            while (slices < 16 && (int64_t)T * slices < 4096 && chunks >= 2 * slices * kWave * unroll) slices *= 2;
            auto launch = [&](auto kern) {
                hipLaunchKernelGGL(kern, dim3((unsigned)ceil_div64((int64_t)T * slices, 4)), dim3(256), 0, st,
                                   (const uint4*)x, (uint4*)x_perm, row_of_assign, T, k, chunks, slices);
            };
            if (unroll == 4) launch(perm_scatter_rows_kernel<4>);
            else launch(perm_scatter_rows_kernel<1>);
            if ((rc = check_launch()) != MOE_OK) return rc;
        }
    }
    return MOE_OK;
}
}  // namespace moegps

extern "C" int moe_permute(int mode, const void* x, int dtype, int T, int d, int E, int k, int G, int S,
                           const int32_t* topk_idx, const int32_t* pred_idx, const int32_t* hist_true,
                           const int32_t* hist_pred, const int32_t* slot_expert, const int32_t* slot_quota,
                           int32_t* seg_offsets, int32_t* row_of_assign, int32_t* assign_of_row, void* x_perm,
                           int32_t* rank_load, void* workspace, size_t workspace_bytes, void* stream) {
    return moegps::permute_impl(mode, x, dtype, T, d, E, k, G, S, topk_idx, pred_idx, hist_true, hist_pred,
                                slot_expert, slot_quota, seg_offsets, row_of_assign, assign_of_row, x_perm, rank_load,
                                workspace, workspace_bytes, stream);
}

// ---------------------------------------------------------------------------
// The same permutation for callers that cannot allocate: the counters, chunk bases and
// segment ids live in a fixed array in device memory that belongs to the library.
// ---------------------------------------------------------------------------
namespace moegps {
static __device__ __align__(256) unsigned char scratch[MOE_PERMUTE_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each GPU, looked up once

// Address of this GPU's copy of the array (every GPU that loads the library holds its own,
// at its own address).  The array's name is only a host-side handle: kernels get this pointer.
static int static_scratch(void** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) {
        set_last_hip_error(e);
        return MOE_ERR_HIP;
    }
    if (dev < 0 || dev >= kMaxDevices) return MOE_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            set_last_hip_error(e);
            return MOE_ERR_HIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return MOE_OK;
}
}  // namespace moegps

extern "C" int moe_permute_static(int mode, const void* x, int dtype, int T, int d, int E, int k, int G, int S,
                                  const int32_t* topk_idx, const int32_t* pred_idx, const int32_t* hist_true,
                                  const int32_t* hist_pred, const int32_t* slot_expert, const int32_t* slot_quota,
                                  int32_t* seg_offsets, int32_t* row_of_assign, int32_t* assign_of_row, void* x_perm,
                                  int32_t* rank_load, void* stream) {
    using namespace moegps;
    if (T < 0 || E < 1 || k < 1 || G < 1 || S < 1) return MOE_ERR_INVALID_ARG;
    // sizes whose counters do not fit the fixed array are refused before anything is enqueued
    if (perm_ws_layout(T, E, k, G, S, nullptr, nullptr) > (size_t)MOE_PERMUTE_STATIC_SCRATCH_BYTES)
        return MOE_ERR_WORKSPACE_TOO_SMALL;
    void* ptr = nullptr;
    const int rc = static_scratch(&ptr);
    if (rc != MOE_OK) return rc;
    return permute_impl(mode, x, dtype, T, d, E, k, G, S, topk_idx, pred_idx, hist_true, hist_pred, slot_expert,
                        slot_quota, seg_offsets, row_of_assign, assign_of_row, x_perm, rank_load, ptr,
                        (size_t)MOE_PERMUTE_STATIC_SCRATCH_BYTES, stream);
}
