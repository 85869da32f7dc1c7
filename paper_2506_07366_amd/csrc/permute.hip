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
//
// A batch of at most 8192 assignments (decode, short prefill) takes the five index steps in
// one workgroup and one launch: the same ranks and scans, the chunk being the whole batch.
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
// The workgroup has NWAVES wavefronts; wcnt is LDS scratch of NWAVES*nkeys ints.
// On return rank[r] holds the rank, and (if chunk_hist) chunk_hist[key] the chunk's
// count per key.  Only the first `rounds` rounds hold elements (uniform over the workgroup).
// ---------------------------------------------------------------------------
template <int NWAVES>
__device__ void chunk_stable_rank(const int (&key)[kRounds], const bool (&valid)[kRounds], int nkeys, int* wcnt,
                                  int (&rank)[kRounds], int32_t* chunk_hist, int rounds = kRounds) {
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int w = tid / kWave;
    for (int i = tid; i < NWAVES * nkeys; i += NWAVES * kWave) wcnt[i] = 0;
    __syncthreads();
    int nbits = 1;
    while ((1 << nbits) < nkeys) ++nbits;
    const unsigned long long lt = (1ull << lane) - 1ull;
    int* mine = wcnt + w * nkeys;
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        rank[r] = 0;
        if (r >= rounds) continue;
        // lanes of this round holding the same key
        unsigned long long same = __ballot(valid[r]);
        for (int b = 0; b < nbits; ++b) {
            const bool bit = (key[r] >> b) & 1;
            const unsigned long long m = __ballot(valid[r] && bit);
            same &= bit ? m : ~m;
        }
        if (valid[r]) {
            const int prior = mine[key[r]];
            rank[r] = prior + __popcll(same & lt);
            if ((same & lt) == 0ull) mine[key[r]] = prior + __popcll(same);  // leader
        }
    }
    __syncthreads();
    // exclusive prefix over the wavefronts, per key
    for (int kk = tid; kk < nkeys; kk += NWAVES * kWave) {
        int c[NWAVES];  // all reads, then all writes: the reads overlap
#pragma unroll
        for (int ww = 0; ww < NWAVES; ++ww) c[ww] = wcnt[ww * nkeys + kk];
        int run = 0;
#pragma unroll
        for (int ww = 0; ww < NWAVES; ++ww) {
            wcnt[ww * nkeys + kk] = run;
            run += c[ww];
        }
        if (chunk_hist) chunk_hist[kk] = run;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kRounds; ++r)
        if (r < rounds && valid[r]) rank[r] += mine[key[r]];
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

// Replicas of expert e in ascending slot id with the exclusive upper bound of each
// replica's range of ranks, by one wavefront (every lane active).
__device__ __forceinline__ void replica_table(int e, int mode, int G, int nseg, const int32_t* __restrict__ hist_true,
                                              const int32_t* __restrict__ hist_pred,
                                              const int32_t* __restrict__ slot_expert,
                                              const int32_t* __restrict__ slot_quota, const PermWs& ws) {
    const int lane = threadIdx.x & (kWave - 1);
    const unsigned long long lt = (1ull << lane) - 1ull;
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

// chunk bases per expert (in place) and the replica tables of the plan; one
// wavefront per expert column, columns dealt over the whole grid
constexpr int kScan1Threads = 256;
__global__ __launch_bounds__(kScan1Threads) void perm_scan1_kernel(int mode, int nb, int E, int G, int S,
                                                           const int32_t* __restrict__ hist_true,
                                                           const int32_t* __restrict__ hist_pred,
                                                           const int32_t* __restrict__ slot_expert,
                                                           const int32_t* __restrict__ slot_quota, PermWs ws) {
    const int nseg = G * S;
    const int wave = threadIdx.x / kWave, nwaves = blockDim.x / kWave;
    for (int e = blockIdx.x * nwaves + wave; e < E; e += gridDim.x * nwaves) {
        int unused[1];
        wave_columns_scan<1>(ws.bh1, nb, E, e, unused);
        replica_table(e, mode, G, nseg, hist_true, hist_pred, slot_expert, slot_quota, ws);
    }
}

// Segment of an assignment to expert e that stands at place i of the plan's order for e
// (i < 0: the assignment is outside the plan's order and goes to the home slot).
__device__ __forceinline__ int segment_of(int e, int i, int H, int S, int G, const PermWs& ws) {
    int sg = home_slot_of(e, H, S);
    if (i < 0) return sg;
    const int cnt = ws.rep_cnt[e];
    if (cnt > 0) {
        int rr = 0;
        while (rr < cnt - 1 && i >= ws.rep_hi[(size_t)e * G + rr]) ++rr;
        sg = ws.rep_slot[(size_t)e * G + rr];
    }
    return sg;
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
        chunk_stable_rank<kPermWaves>(key, valid, E, wcnt, rank, nullptr);
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
        const int sg = segment_of(e, i, H, S, G, ws);
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
    chunk_stable_rank<kPermWaves>(key, valid, nseg, wcnt, rank, nullptr);
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int p = w * (kRounds * kWave) + r * kWave + lane;
        if (!valid[r]) continue;
        const int row = seg_offsets[key[r]] + ws.bh2[(size_t)blockIdx.x * nseg + key[r]] + rank[r];
        row_of_assign[base + p] = row;
        assign_of_row[row] = (int)(base + p);
    }
}

// All five index steps for a batch of at most kSmallA assignments, E and G*S at most
// kSmallKeys, in one workgroup of 1024 threads: the chunk is the whole batch, so the chunk
// bases are zero and both scans run in LDS.  A thread's time here goes by the number of
// instructions it runs one after the other, so the batch is dealt over all 16 wavefronts in
// as few rounds of 64 as hold it.  The replica tables live in LDS, one entry per slot: the
// upper bound of the slot's range of ranks and the next slot of the same expert (ascending
// slot id), plus every expert's first slot.  Same ranks, same results as the kernels above.
constexpr int kSmallThreads = 1024;
constexpr int kSmallWaves = kSmallThreads / kWave;
constexpr int kSmallA = kSmallThreads * kRounds;  // 8192
constexpr int kSmallKeys = 512;

// The per-slot tables, by one wavefront, 64 slots at a time in ascending order: the lanes
// holding one expert find each other by ballots; what earlier chunks hold for the expert
// (slots, quota, last slot) is carried in LDS.
struct SmallTables {
    int* s_e;         // [kSmallKeys] expert of the slot (-1 beyond the plan's slots)
    int* s_q;         // [kSmallKeys] its quota
    long long* s_cum; // [kSmallKeys] quota of the expert's slots up to and including this one
    int* s_next;      // [kSmallKeys] next slot of the same expert, -1: none
    int* e_first;     // [kSmallKeys] first slot of the expert, -1: home slot only
    int* e_cnt;       // [kSmallKeys] slots of the expert so far
    int* e_last;      // [kSmallKeys] the last of them
    long long* e_cum; // [kSmallKeys] their quota
};
__device__ __forceinline__ void small_slot_tables(int E, int nseg, const SmallTables& t) {
    const int lane = threadIdx.x & (kWave - 1);
    const unsigned long long bit = 1ull << lane;
    const unsigned long long lt = bit - 1ull;
    int nbits = 1;
    while ((1 << nbits) < E) ++nbits;
    for (int s0 = 0; s0 < nseg; s0 += kWave) {
        const int sigma = s0 + lane;
        const int e = sigma < nseg ? t.s_e[sigma] : -1;
        const bool ok = e >= 0 && e < E;
        const int q = ok ? t.s_q[sigma] : 0;
        unsigned long long same = __ballot(ok);
        for (int b = 0; b < nbits; ++b) {
            const bool one = (e >> b) & 1;
            const unsigned long long m = __ballot(ok && one);
            same &= one ? m : ~m;
        }
        if (!ok) same = 0ull;
        // quota of the expert's slots of this chunk up to this one: lanes take the set bits of
        // their mask one by one, as many steps as the largest group of the chunk has lanes
        long long cum = 0;
        unsigned long long todo = same & (lt | bit);
        while (__any(todo != 0ull)) {
            const int src = todo ? __ffsll((long long)todo) - 1 : lane;
            const int qs = __shfl(q, src, kWave);
            cum += todo ? (long long)qs : 0ll;
            todo &= todo - 1ull;
        }
        if (ok) {
            const int prior = t.e_cnt[e];
            const int last = t.e_last[e];
            cum += t.e_cum[e];
            const unsigned long long above = same & ~(lt | bit);
            t.s_cum[sigma] = cum;
            t.s_next[sigma] = above ? s0 + __ffsll((long long)above) - 1 : -1;
            if ((same & lt) == 0ull) {  // first lane of the expert in this chunk
                if (prior == 0) t.e_first[e] = sigma;
                else t.s_next[last] = sigma;
            }
            if (above == 0ull) {        // last lane: hand the totals on
                t.e_cnt[e] = prior + __popcll(same);
                t.e_cum[e] = cum;
                t.e_last[e] = sigma;
            }
        }
    }
}

__global__ __launch_bounds__(kSmallThreads) void perm_small_kernel(
    int mode, int T, int k, int E, int G, int S, const int32_t* __restrict__ topk_idx,
    const int32_t* __restrict__ pred_idx, const int32_t* __restrict__ hist_true, const int32_t* __restrict__ hist_pred,
    const int32_t* __restrict__ slot_expert, const int32_t* __restrict__ slot_quota,
    int32_t* __restrict__ seg_offsets, int32_t* __restrict__ row_of_assign, int32_t* __restrict__ assign_of_row,
    int32_t* __restrict__ rank_load) {
    // one buffer, three lives: wavefront counters of the first rank; rank and key by position
    // (token-to-expert mode looks up those of the token's predicted ids); counters of the second
    __shared__ int buf[kSmallWaves * kSmallKeys];
    static_assert(kSmallWaves * kSmallKeys >= kSmallA, "ranks by position share the counters' buffer");
    static_assert(kSmallA <= (1 << 16) && kSmallKeys <= (1 << 15), "rank and key share one int");
    __shared__ int s_e[kSmallKeys], s_q[kSmallKeys], s_hi[kSmallKeys], s_next[kSmallKeys];
    __shared__ int e_first[kSmallKeys], e_cnt[kSmallKeys], e_last[kSmallKeys], e_true[kSmallKeys], e_hat[kSmallKeys];
    __shared__ int e_home[kSmallKeys];  // home slot of the expert
    __shared__ long long e_cum[kSmallKeys], s_cum[kSmallKeys];
    __shared__ int tot[kSmallKeys + 1];
    __shared__ int wave_sum[16];
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int w = tid / kWave;
    const int nseg = G * S;
    const int H = (E + G - 1) / G;
    const int n_b = T * k;
    // rounds of 64 per wavefront that hold the batch; element p is (w, r, lane) with
    // p = (w * rounds + r) * 64 + lane
    const int rounds = (n_b + kSmallThreads - 1) / kSmallThreads;

    int key[kRounds], rank[kRounds], expert[kRounds];
    bool valid[kRounds];
    const int32_t* rank_keys = (mode == MOE_MODE_TOKEN) ? pred_idx : topk_idx;
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int p = (w * rounds + r) * kWave + lane;
        valid[r] = r < rounds && p < n_b;
        key[r] = valid[r] ? clamp_key(rank_keys[p], E) : 0;
        expert[r] = key[r];
        rank[r] = 0;
    }
    if (mode == MOE_MODE_TOKEN) {
#pragma unroll
        for (int r = 0; r < kRounds; ++r) {
            const int p = (w * rounds + r) * kWave + lane;
            if (valid[r]) expert[r] = clamp_key(topk_idx[p], E);
        }
    }
    for (int e = tid; e < E; e += kSmallThreads) e_home[e] = home_slot_of(e, H, S);
    if (mode != MOE_MODE_NONE) {
        for (int i = tid; i < kSmallKeys; i += kSmallThreads) {
            s_e[i] = i < nseg ? slot_expert[i] : -1;
            s_q[i] = i < nseg ? slot_quota[i] : 0;
            e_first[i] = e_last[i] = -1;
            e_cnt[i] = 0;
            e_cum[i] = 0ll;
            if (mode == MOE_MODE_DISTRIBUTION && i < E) {
                e_true[i] = hist_true[i];
                e_hat[i] = hist_pred[i];
            }
        }
        __syncthreads();
        if (w == kSmallWaves - 1) {
            const SmallTables t{s_e, s_q, s_cum, s_next, e_first, e_cnt, e_last, e_cum};
            small_slot_tables(E, nseg, t);
        }
        chunk_stable_rank<kSmallWaves>(key, valid, E, buf, rank, nullptr, rounds);
        __syncthreads();  // the counters are dead, the buffer becomes rank and key by position
#pragma unroll
        for (int r = 0; r < kRounds; ++r) {
            const int p = (w * rounds + r) * kWave + lane;
            if (valid[r]) buf[p] = rank[r] | (key[r] << 16);
        }
        // upper bound of every slot's range of ranks from the quota up to it, all slots at once
        if (tid < nseg) {
            const int e = s_e[tid];
            long long hi = s_cum[tid];                                                  // Q_{r+1}
            if (mode == MOE_MODE_DISTRIBUTION && e >= 0 && e < E && e_hat[e] > 0)
                hi = ((long long)e_true[e] * hi) / e_hat[e];                            // floor(n_e * Q / nhat_e)
            if (hi > 0x7fffffffLL) hi = 0x7fffffffLL;
            s_hi[tid] = (int)hi;
        }
        // an expert nobody is predicted for keeps its home slot
        if (mode == MOE_MODE_DISTRIBUTION && tid < E && e_hat[tid] <= 0) e_first[tid] = -1;
    }
    __syncthreads();

    // segment of every assignment: its place i in the plan's order for its expert (-1: none),
    // then a walk over the expert's slots, at most G of them, to the one whose range holds i;
    // the rounds walk in step so that their LDS reads overlap
    int sg[kRounds], place[kRounds];
    bool walking[kRounds];
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int p = (w * rounds + r) * kWave + lane;
        sg[r] = 0;
        place[r] = -1;
        walking[r] = false;
        if (!valid[r]) continue;
        if (mode == MOE_MODE_DISTRIBUTION) {
            place[r] = rank[r];
        } else if (mode == MOE_MODE_TOKEN) {
            const int row0 = (p / k) * k;  // the token's predicted ids
            for (int jp = 0; jp < k; ++jp) {
                const int v = buf[row0 + jp];
                if ((v >> 16) == expert[r]) {
                    place[r] = v & 0xffff;
                    break;
                }
            }
        }
        sg[r] = e_home[expert[r]];
        if (place[r] >= 0) {
            const int first = e_first[expert[r]];
            if (first >= 0) {
                sg[r] = first;
                walking[r] = true;
            }
        }
    }
    for (int seen = 1; mode != MOE_MODE_NONE && seen < G; ++seen) {
        bool more = false;
#pragma unroll
        for (int r = 0; r < kRounds; ++r) {  // no branches: sg[r] is a slot in any case, the reads overlap
            if (r >= rounds) continue;       // (uniform)
            const int nx = s_next[sg[r]];
            const int hi = s_hi[sg[r]];
            walking[r] = walking[r] && nx >= 0 && place[r] >= hi;
            sg[r] = walking[r] ? nx : sg[r];
            more = more || walking[r];
        }
        if (!__any(more)) break;
    }
    __syncthreads();  // every look-up of a rank is done before the buffer holds counters again

    chunk_stable_rank<kSmallWaves>(sg, valid, nseg, buf, rank, tot, rounds);
    block_exclusive_scan_2048(tot, nseg, wave_sum);
    for (int s = tid; s <= nseg; s += kSmallThreads) seg_offsets[s] = tot[s];
    for (int g = tid; g < G; g += kSmallThreads) rank_load[g] = tot[(g + 1) * S] - tot[g * S];
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int p = (w * rounds + r) * kWave + lane;
        if (!valid[r]) continue;
        const int row = tot[sg[r]] + rank[r];
        row_of_assign[p] = row;
        assign_of_row[row] = p;
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
    const bool small = (int64_t)T * k <= kSmallA && E <= kSmallKeys && G * S <= kSmallKeys;
    if (small) {
        hipLaunchKernelGGL(perm_small_kernel, dim3(1), dim3(kSmallThreads), 0, st, mode, T, k, E, G, S, topk_idx,
                           pred_idx, hist_true, hist_pred, slot_expert, slot_quota, seg_offsets, row_of_assign,
                           assign_of_row, rank_load);
        if ((rc = check_launch()) != MOE_OK) return rc;
    } else {
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
        }
    }
    if (nb > 0) {
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
