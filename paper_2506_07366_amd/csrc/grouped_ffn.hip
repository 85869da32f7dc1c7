// Grouped SwiGLU expert FFN (Section 3.4: Mixtral-style FFN with SwiGLU; the
// dominant cost of the layer per the Background's performance discussion):
//     y = ( silu(x W1_e) * (x W3_e) ) W2_e      for every row of a segment whose
//                                               slot hosts expert e.
//
// bf16 path: two persistent grouped GEMMs on the MFMA units.
//   GEMM-1: H[A, ffn]  = swiglu( X[A, d] * [W1|W3]_e )    (gate/up columns interleaved
//           by 32 in the packed weights, so the SwiGLU happens on the accumulators)
//   GEMM-2: Y[A, d]    = H[A, ffn] * W2_e
// Packed weights are stored "column-major" ([N][K], K contiguous), the same shape
// as the activations, so both operands stream as K-contiguous 16-byte pieces
// straight from global memory into LDS (global_load_lds_dwordx4) and feed
// v_mfma_f32_16x16x32_bf16 fragments with one ds_read_b128 each.
//
// Rows are tiled by EXPERT, not by segment: replicas of an expert hold the same
// weights, so the rows of all its segments in the launched slot range are listed
// one after the other (a device-built row list) and cut into M-tiles together;
// an expert then has one ragged tile however many replicas the plan gave it, and
// its weight panels stream once.  The hidden activations are stored in list
// order; the second product writes each result to its own row of y_perm.
// Workgroups claim (M-tile, N-tile) pairs from per-XCD counters in an order that
// keeps the tiles running at the same time on a shared set of weight and
// activation panels.  When the second product has only a few tiles per
// workgroup, its closing tiles are computed as several parts of K (fp32 partial
// sums, added up by a small kernel in a fixed order), so that the last items a
// workgroup claims are short.  The hidden width is padded to a multiple of 64
// inside the packed weights.
//
// The ReLU form (Discussion: Switch Transformer's FFN), y = max(x W1_e, 0) W2_e, runs
// the same two products with another epilogue on the first.
//
// fp32 path (small reference-precision configs): a plain LDS-tiled FMA kernel.
#include "common.h"
#include "block_scan.h"
#include <atomic>
#include <type_traits>
#include <utility>

namespace moegps {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef unsigned short bf16_t;  // storage

// One entry of an M-tile table: up to BM consecutive positions of the row list, all of one
// expert, and the part of the K range this entry covers.
struct MTile {
    int list0;   // first position in the row list
    int rows;    // valid rows (<= BM)
    int expert;  // expert whose weights the rows take
    int kt0;     // k-tiles [kt0, kt1) of the product belong to this entry; kt1 == 0: all of them
    int kt1;
    int part;    // < 0: results go to the output; else fp32 partial sums go to slab `part`
    int pad0, pad1;
};
// An M-tile whose K range is split, for the pass that adds up the partial sums
struct SplitInfo {
    int list0, rows;
};
constexpr int kGemmGrid = 256;  // persistent workgroups of a GEMM launch: 8 XCDs x 32
constexpr int kPartRows = 256;  // rows of one slab of partial sums (the tallest tile shape)
constexpr int kMaxParts = 4;    // parts of K of a split tile

// counts[] of a table: number of entries, end of the first pass (whole full-height tiles),
// end of the second pass (whole ragged tiles; the third pass holds the parts of split
// tiles), number of split M-tiles
constexpr int kCntEntries = 0, kCntPass0 = 1, kCntPass1 = 2, kCntSplit = 3, kCntStride = 4;

// ---------------------------------------------------------------------------
// weight packing (one-off, weights are static across inputs)
// ---------------------------------------------------------------------------
// The packed form of a weight matrix is what the GEMM's loads want to find: the transposed
// matrix W^T [N_out][K_out] cut into tiles of kPackN rows by kPackK columns, tiles of one
// row block side by side along K, every tile 32 KiB in one piece and laid out exactly as
// it sits in LDS (row r, 16-byte piece c of the row at piece c ^ swz(r)).  A k-tile of a
// weight panel is then one contiguous read instead of 256 pieces of 128 bytes a row apart,
// which the memory system serves a quarter slower at some row lengths (8 KiB among them).
constexpr int kPackN = 256, kPackK = 64;
// 16-byte piece `slot` of LDS row `row` holds piece slot ^ swz(row) of the row.  The LDS
// has 64 four-byte banks and serves a ds_read_b128 sixteen lanes at a time, so the
// 16 consecutive rows one such group touches must land on 16 distinct 16-byte bank
// groups of a 256-byte span: with 128-byte rows that is (row&1, slot) -> xor with
// (row>>1)&7.
__host__ __device__ inline int swz(int row) { return (row >> 1) & 7; }
__host__ __device__ inline size_t packed_index(int n, int k, int K_out) {
    const int row = n % kPackN, kk = k % kPackK;
    const size_t tile = (size_t)(n / kPackN) * (K_out / kPackK) + k / kPackK;
    return (tile * kPackN + row) * kPackK + (((kk >> 3) ^ swz(row)) << 3) + (kk & 7);
}

// out[packed_index(n, k)] = in[k][n] for one expert per blockIdx.z, zero where k >= K or
// n >= N (the output is K_out x N_out, padded); optional interleave of the output row
// index: rows of W1 go to (n/32)*64 + n%32, rows of W3 32 further.
__global__ __launch_bounds__(256) void pack_transpose_kernel(const bf16_t* __restrict__ in, bf16_t* __restrict__ out,
                                                              int K, int N, int K_out, int N_out,
                                                              size_t in_expert_stride, size_t out_expert_stride,
                                                              int interleave, int sel) {
    __shared__ bf16_t tile[32][33];
    const bf16_t* src = in + (size_t)blockIdx.z * in_expert_stride;
    bf16_t* dst = out + (size_t)blockIdx.z * out_expert_stride;
    const int n0 = blockIdx.x * 32, k0 = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
    for (int r = ty; r < 32; r += 8) {
        const int kk = k0 + r, nn = n0 + tx;
        tile[r][tx] = (kk < K && nn < N) ? src[(size_t)kk * N + nn] : (bf16_t)0;
    }
    __syncthreads();
    for (int r = ty; r < 32; r += 8) {
        const int nn = n0 + r, kk = k0 + tx;
        if (nn < N_out && kk < K_out) {
            const int orow = interleave ? ((nn / 32) * 64 + sel * 32 + (nn % 32)) : nn;
            dst[packed_index(orow, kk, K_out)] = tile[tx][r];
        }
    }
}

__global__ void copy_u4_kernel(const uint4* __restrict__ in, uint4* __restrict__ out, size_t n) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) out[i] = in[i];
}

// ---------------------------------------------------------------------------
// row list and M-tile tables from the ragged segments
// ---------------------------------------------------------------------------
// What one product's table is built for.
struct TableSpec {
    MTile* tiles;       // out
    int32_t* counts;    // out, kCntStride ints
    SplitInfo* splits;  // out (split tiles only), may be null when parts <= 1
    int bm;             // tile height
    int capacity;       // entries `tiles` has room for
    int kt;             // k-tiles of the product
    int parts;          // parts of K of a split tile (<= 1: no tile is split)
    int n_ntiles;       // N-tiles of the product and workgroups of its launch: they decide how much
    int grid;           //   work is split at the end of the order (see build_tables_kernel)
    int split_all;      // split every tile (tests)
    int split_capacity; // split M-tiles `splits` and the slabs have room for
};

// Row list: position p holds a row of x_perm; the rows of an expert's segments (ascending
// slot id, rows ascending) are consecutive, experts ascending.  M-tile tables: first every
// full-height tile by expert, so that neighbours read the same expert's weights; then the
// ragged last tile of every expert, tallest first, so that the cheap tiles come last and
// fill the gaps at the end of the launch.  With parts > 1 the closing M-tiles of that order are
// listed once per part of K instead, part by part, each entry writing fp32 partial sums to a
// slab of its own (slab = split tile * parts + part).  How many: the work of the product,
// counted in tiles (a ragged tile of r rows as (BM + r) / 2BM of a tile: its weight panel
// streams in full), is so many whole rounds of one tile per workgroup plus a remainder; the
// rounds run as whole tiles, and the remainder -- what would otherwise be a last round with
// most workgroups idle -- is what gets split, smallest tiles first, unless it is most of a
// round anyway (more than 5/8: splitting would add traffic and save little).
// Every workgroup rebuilds the small per-segment and per-expert tables in LDS and then
// fills its stripe of the row list; workgroup 0 writes the first table and clears the claim
// counters, workgroup 1 (0 if it is alone) the second.
__global__ __launch_bounds__(1024) void build_tables_kernel(const int32_t* __restrict__ seg_offsets,
                                                             const int32_t* __restrict__ slot_expert, int seg_begin,
                                                             int seg_end, int E, TableSpec t1, TableSpec t2,
                                                             int32_t* __restrict__ rowlist,
                                                             int32_t* __restrict__ queues, int n_queues) {
    __shared__ __align__(16) int s_rows[MOE_MAX_SEGMENTS];  // rows of the segment (0: not live)
    __shared__ __align__(16) int s_ex[MOE_MAX_SEGMENTS];    // its expert
    __shared__ int s_first[MOE_MAX_SEGMENTS];      // first row of x_perm
    __shared__ int srt_base[MOE_MAX_SEGMENTS + 1]; // list position of the j-th segment in list order
    __shared__ int srt_first[MOE_MAX_SEGMENTS];    // its first row of x_perm
    __shared__ int e_rows[MOE_MAX_EXPERTS + 1];    // rows per expert -> list base per expert
    __shared__ int e_segs[MOE_MAX_EXPERTS + 1];    // live segments per expert -> base in list order; later: whole
                                                   //   ragged tiles of the experts below
    __shared__ int e_full[MOE_MAX_EXPERTS + 1];    // full-height tiles per expert -> base
    __shared__ __align__(16) int e_tail[MOE_MAX_EXPERTS];  // rows of the expert's ragged tile
    __shared__ int e_rank[MOE_MAX_EXPERTS];        // its place among the ragged tiles, tallest first
    __shared__ int wave_sum[32];
    __shared__ int total_tail, tail_rows;
    const int tid = threadIdx.x;
    const int ns = seg_end - seg_begin;
    if (blockIdx.x == 0)
        for (int i = tid; i < n_queues; i += blockDim.x) queues[i] = 0;
    for (int e = tid; e < E; e += blockDim.x) e_rows[e] = e_segs[e] = 0;
    __syncthreads();
    for (int i = tid; i < ns; i += blockDim.x) {
        const int s = seg_begin + i;
        const int lo = seg_offsets[s];
        const int rows = seg_offsets[s + 1] - lo;
        const int e = slot_expert[s];
        const bool live = rows > 0 && e >= 0 && e < E;
        s_rows[i] = live ? rows : 0;
        s_ex[i] = e;
        s_first[i] = lo;
        if (live) {
            atomicAdd(&e_rows[e], rows);
            atomicAdd(&e_segs[e], 1);
        }
    }
    __syncthreads();
    // e_rows[e] = list base, e_rows[E] = rows in the range; e_segs[e] = base in list order
    block_exclusive_scan2_2048(e_rows, e_segs, E, wave_sum);
    const int n_list = e_rows[E], n_live = e_segs[E];
    // place of every live segment in list order: behind the segments of lower experts and the
    // lower segments of its own expert.  A thread's time goes by the instructions it runs one
    // after the other, so the pairs (segment, lower segment) are dealt over the whole workgroup:
    // `share` threads split the lower segments of one segment between them and add their
    // counts up in LDS (srt_base / srt_first hold them by segment until the places are known).
    for (int i = tid; i < ns; i += blockDim.x) srt_base[i] = srt_first[i] = 0;
    __syncthreads();
    {
        int width = kWave;  // threads side by side on different segments
        while (width < ns && width < (int)blockDim.x) width <<= 1;
        const int share = blockDim.x / width, part = tid / width;
        const int per = ceil_div(ceil_div(ns, 4), share);  // groups of four lower segments per thread
        for (int i = tid % width; i < ns; i += width) {
            if (s_rows[i] == 0) continue;
            const int e = s_ex[i];
            int before = 0, rows_before = 0;
            const int g_end = (part + 1) * per < ceil_div(i, 4) ? (part + 1) * per : ceil_div(i, 4);
            for (int g = part * per; g < g_end; ++g) {  // four segments per LDS read, no branches
                const int j0 = 4 * g;
                const int4 r4 = *reinterpret_cast<const int4*>(&s_rows[j0]);
                const int4 x4 = *reinterpret_cast<const int4*>(&s_ex[j0]);
                const int rs[4] = {r4.x, r4.y, r4.z, r4.w};
                const int xs[4] = {x4.x, x4.y, x4.z, x4.w};
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const bool same = j0 + u < i && rs[u] > 0 && xs[u] == e;
                    before += same ? 1 : 0;
                    rows_before += same ? rs[u] : 0;
                }
            }
            if (before) {
                atomicAdd(&srt_base[i], before);
                atomicAdd(&srt_first[i], rows_before);
            }
        }
    }
    __syncthreads();
    {
        constexpr int kPer = MOE_MAX_SEGMENTS / 1024;  // segments per thread
        int before[kPer], rows_before[kPer];
#pragma unroll
        for (int q = 0; q < kPer; ++q) {
            const int i = tid + q * (int)blockDim.x;
            before[q] = i < ns ? srt_base[i] : 0;
            rows_before[q] = i < ns ? srt_first[i] : 0;
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < kPer; ++q) {
            const int i = tid + q * (int)blockDim.x;
            if (i >= ns || s_rows[i] == 0) continue;
            const int e = s_ex[i];
            srt_base[e_segs[e] + before[q]] = e_rows[e] + rows_before[q];
            srt_first[e_segs[e] + before[q]] = s_first[i];
        }
    }
    if (tid == 0) srt_base[n_live] = n_list;
    __syncthreads();
    // row list: binary search of the position among the segments in list order
    for (int p = blockIdx.x * blockDim.x + tid; p < n_list; p += gridDim.x * blockDim.x) {
        int lo = 0, hi = n_live - 1;
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (srt_base[mid] <= p) lo = mid;
            else hi = mid - 1;
        }
        rowlist[p] = srt_first[lo] + (p - srt_base[lo]);
    }
    // tables
    const bool second = (gridDim.x > 1) ? blockIdx.x == 1 : true;
    const bool first = blockIdx.x == 0;
    if (!first && !second) return;
    for (int which = 0; which < 2; ++which) {  // uniform per workgroup
        if (which == 0 ? !first : !second) continue;
        const TableSpec& ts = which == 0 ? t1 : t2;
        if (!ts.tiles) continue;
        const int BM = ts.bm;
        __syncthreads();
        if (tid == 0) total_tail = tail_rows = 0;
        __syncthreads();
        {   // (E <= blockDim.x: one expert per thread; one LDS atomic per wavefront)
            const int e = tid;
            const int rows = e < E ? e_rows[e + 1] - e_rows[e] : 0;
            const int tl = rows % BM;
            if (e < E) {
                e_full[e] = rows / BM;
                e_tail[e] = tl;
            }
            const int n_t = wave_sum_i32(tl > 0 ? 1 : 0), r_t = wave_sum_i32(tl);
            if ((tid & (kWave - 1)) == 0 && n_t) {
                atomicAdd(&total_tail, n_t);
                atomicAdd(&tail_rows, r_t);
            }
        }
        __syncthreads();
        block_exclusive_scan_2048(e_full, E, wave_sum);
        const int n_full = e_full[E], n_tail = total_tail;
        // tiles split at the end of the order: the smallest ragged ones first, then full-height ones
        int n_fsplit = 0, n_rsplit = 0, n_split = 0;
        long long want = 0;  // half-rows of M-tiles to split
        const int P = ts.parts > kMaxParts ? kMaxParts : ts.parts;
        if (P > 1) {
            const long long units = (long long)n_full * 2 * BM + (long long)n_tail * BM + tail_rows;  // half-rows
            const long long round_units = (long long)ts.grid * 2 * BM;  // one tile per workgroup, times n_ntiles
            const long long rem = (units * ts.n_ntiles) % round_units;
            if (ts.split_all) want = units;
            else if (rem > 0 && rem * 8 <= round_units * 5) want = (rem + ts.n_ntiles - 1) / ts.n_ntiles;
        }
        // ragged tile of expert e: rank in the order (tallest first) and the half-rows of the ragged
        // tiles behind it; it is split if those do not reach `want` yet
        __syncthreads();
        if (tid == 0) total_tail = 0;  // reused: number of split ragged tiles, their half-rows in tail_rows
        __syncthreads();
        if (tid == 0) tail_rows = 0;
        __syncthreads();
        // (pairs of experts dealt over the workgroup like the pairs of segments above; the
        // half-rows behind a ragged tile are counted in srt_first, free since the row list is
        // written: at most E * 2 * BM, an int)
        int* e_behind = srt_first;
        for (int e = tid; e < E; e += blockDim.x) e_rank[e] = e_behind[e] = 0;
        __syncthreads();
        {
            int width = kWave;
            while (width < E && width < (int)blockDim.x) width <<= 1;
            const int share = blockDim.x / width, part = tid / width;
            const int per = ceil_div(ceil_div(E, 4), share);
            const int e = tid % width;
            const int tl = e < E ? e_tail[e] : 0;
            if (tl > 0) {
                int rank = 0, behind = 0;
                const int g_end = (part + 1) * per < ceil_div(E, 4) ? (part + 1) * per : ceil_div(E, 4);
                for (int g = part * per; g < g_end; ++g) {
                    const int j0 = 4 * g;
                    const int4 t4 = *reinterpret_cast<const int4*>(&e_tail[j0]);
                    const int ts4[4] = {t4.x, t4.y, t4.z, t4.w};
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int j = j0 + u, tj = ts4[u];
                        const bool live = j < E && tj > 0;
                        const bool ahead = tj > tl || (tj == tl && j < e);
                        rank += (live && ahead) ? 1 : 0;
                        behind += (live && !ahead && j != e) ? BM + tj : 0;
                    }
                }
                if (rank) atomicAdd(&e_rank[e], rank);
                if (behind) atomicAdd(&e_behind[e], behind);
            }
        }
        __syncthreads();
        {
            const int e = tid;
            const int tl = e < E ? e_tail[e] : 0;
            const bool cut = tl > 0 && (long long)e_behind[e] < want;
            const int n_c = wave_sum_i32(cut ? 1 : 0), r_c = wave_sum_i32(cut ? BM + tl : 0);
            if ((tid & (kWave - 1)) == 0 && n_c) {
                atomicAdd(&total_tail, n_c);
                atomicAdd(&tail_rows, r_c);
            }
        }
        __syncthreads();
        n_rsplit = total_tail;
        {
            const long long have = tail_rows;
            const long long f = want > have ? (want - have + 2 * BM - 1) / (2 * BM) : 0;
            n_fsplit = f < n_full ? (int)f : n_full;
        }
        n_split = n_fsplit + n_rsplit;
        if (n_split > ts.split_capacity) n_fsplit = n_rsplit = n_split = 0;  // stay in bounds (the host sizes for the rule)
        const bool split = n_split > 0;
        const int n_whole_full = n_full - n_fsplit;
        const int n_whole_tail = n_tail - n_rsplit;
        const int n_whole = n_whole_full + n_whole_tail;
        const int n_entries = n_whole + n_split * P;
        const bool fits = n_entries <= ts.capacity;
        auto part_range = [&](int part, int& k0, int& k1) {
            k0 = (int)((long long)ts.kt * part / P);
            k1 = (int)((long long)ts.kt * (part + 1) / P);
        };
        auto emit = [&](int list0, int rows, int expert, int whole_index, int split_index) {
            MTile mt;
            mt.list0 = list0;
            mt.rows = rows;
            mt.expert = expert;
            mt.kt0 = mt.kt1 = 0;
            mt.part = -1;
            mt.pad0 = mt.pad1 = 0;
            if (split_index < 0) {
                ts.tiles[whole_index] = mt;
                return;
            }
            for (int part = 0; part < P; ++part) {
                part_range(part, mt.kt0, mt.kt1);
                mt.part = split_index * P + part;
                ts.tiles[n_whole + part * n_split + split_index] = mt;
            }
            ts.splits[split_index].list0 = list0;
            ts.splits[split_index].rows = rows;
        };
        // whole ragged tiles of the experts below e (each sits right behind its expert's full tiles)
        for (int e = tid; e < E; e += blockDim.x) e_segs[e] = (e_tail[e] > 0 && e_rank[e] < n_whole_tail) ? 1 : 0;
        __syncthreads();
        block_exclusive_scan_2048(e_segs, E, wave_sum);
        auto whole_tails_below = [&](int e) { return e_segs[e]; };
        if (fits) {
            // full-height tiles: tile t belongs to the expert whose range of tile numbers holds it
            for (int t = tid; t < n_full; t += blockDim.x) {
                int lo = 0, hi = E - 1;
                while (lo < hi) {
                    const int mid = (lo + hi + 1) >> 1;
                    if (e_full[mid] <= t) lo = mid;
                    else hi = mid - 1;
                }
                const int list0 = e_rows[lo] + (t - e_full[lo]) * BM;
                if (t < n_whole_full) emit(list0, BM, lo, t + whole_tails_below(lo), -1);
                else emit(list0, BM, lo, 0, t - n_whole_full);
            }
            // ragged tiles, tallest first (ties: lower expert first); the last n_rsplit of them are split
            for (int e = tid; e < E; e += blockDim.x) {
                const int tl = e_tail[e];
                if (tl == 0) continue;
                const int rank = e_rank[e];
                const int list0 = e_rows[e] + (e_full[e + 1] - e_full[e]) * BM;
                if (rank >= n_whole_tail) emit(list0, tl, e, 0, n_fsplit + rank - n_whole_tail);
                else emit(list0, tl, e, (e_full[e + 1] < n_whole_full ? e_full[e + 1] : n_whole_full) + whole_tails_below(e), -1);
            }
        }
        if (tid == 0) {
            ts.counts[kCntEntries] = fits ? n_entries : 0;
            ts.counts[kCntPass0] = fits ? n_whole : 0;
            ts.counts[kCntPass1] = fits ? n_whole : 0;
            ts.counts[kCntSplit] = fits ? n_split : 0;
        }
    }
}

// ---------------------------------------------------------------------------
// bf16 grouped GEMM on MFMA
// ---------------------------------------------------------------------------
// s_waitcnt with only vmcnt set (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[15:14])
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt range");
    __builtin_amdgcn_s_waitcnt((N & 0xf) | (0x7 << 4) | (0xf << 8) | ((N >> 4) << 14));
}

// compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>)
template <int... I, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F&& f) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
    static_for_impl(std::make_integer_sequence<int, N>{}, f);
}

// LDS fragment read issued as an instruction of its own: the compiler does not track
// when the data lands, the kernel waits with lds_wait<N>() ("at most N LDS reads of
// this wavefront still in flight"; LDS reads complete in issue order) and then ties
// the destination registers with lds_landed() before they are used.
template <int OFF>
__device__ __forceinline__ void lds_read_b128(bf16x8& dst, unsigned addr) {
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF) : "memory");
}
template <int N>
__device__ __forceinline__ void lds_wait() {
    static_assert(N >= 0 && N < 16, "lgkmcnt range");
    __builtin_amdgcn_s_waitcnt(0xc07f | (N << 8));  // vmcnt and expcnt untouched
}
__device__ __forceinline__ void lds_landed(bf16x8& v) { asm volatile("" : "+v"(v)); }

// A copy of a lane-dependent value that the compiler cannot trace back: what is computed
// from it is computed where it is used (per tile) instead of once per kernel and then kept
// in a register, or in scratch memory, across the K loop.
__device__ __forceinline__ int opaque(int v) {
    asm volatile("" : "+v"(v));
    return v;
}
// the same for a value that is uniform over the wavefront (scalar register)
__device__ __forceinline__ int opaque_uniform(int v) {
    asm volatile("" : "+s"(v));
    return v;
}

// With the wavefront seen as four quarters of 16 lanes, p = [p0 p1 p2 p3] and q = [q0 q1 q2 q3]
// become p = [p0 p2 q0 q2] and q = [p1 p3 q1 q3] (two register-to-register swap instructions).
__device__ __forceinline__ void lane_swap_pairs(unsigned& p, unsigned& q) {
    auto r = __builtin_amdgcn_permlane32_swap(p, q, false, false);  // p: [p0 p1 q0 q1], q: [p2 p3 q2 q3]
    auto t = __builtin_amdgcn_permlane16_swap(r[0], r[1], false, false);
    p = t[0];
    q = t[1];
}

// 16 bytes per lane from global memory straight into LDS: lane l's piece comes from
// base + voff (uniform 64-bit base in scalar registers, 32-bit byte offset per lane: an
// addressing mode of the instruction, so a load costs no vector ALU work and one address
// register) and lands at LDS byte address lds_addr + 16 * l (uniform, handed over in M0).
// Counts on vmcnt like any load.
__device__ __forceinline__ void global_to_lds_b128(const void* base, unsigned voff, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(base)
                 : "memory");
}

// two floats rounded to bf16 (nearest even) and packed, low half first: one conversion instruction
__device__ __forceinline__ unsigned pack_bf16x2(float lo, float hi) {
    typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
    typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
}

// silu(g) = g / (1 + exp(-g)) with the hardware reciprocal (1 ulp) and the hardware
// exponential in place of an IEEE division and expf; the result is rounded to bf16 right after.
__device__ __forceinline__ float silu_f(float g) { return g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)); }

// EPI selects what happens to the accumulators before they are stored: kEpiNone (plain
// product, optionally scaled per row), kEpiSwiglu (silu(gate) * up on interleaved column
// pairs, half as many output columns), kEpiRelu (max(., 0)).
constexpr int kEpiNone = 0, kEpiSwiglu = 1, kEpiRelu = 2;

// Where the rows of a product live.  List position p of an M-tile is
//   operand row  a_rows ? a_rows[p] : p, and then, with a_rows2, a_rows2[that] / a_div
//                (the first product reads x_perm through the row list, or the token rows
//                of x through the row list and assign_of_row);
//   output row   c_rows ? c_rows[p] : p  (the second product writes y_perm through the row list);
//   output scale scale ? scale[scale_idx[output row]] : 1  (gate weight of the row's assignment).
struct RowMap {
    const int32_t* a_rows;
    const int32_t* a_rows2;
    int a_div;
    const int32_t* c_rows;
    const int32_t* scale_idx;
    const float* scale;
};

template <int BM, int BN, int BK, int WGM, int WGN, int NSTAGE, int EPI>
__global__ __launch_bounds__(WGM* WGN * 64) void grouped_gemm_bf16_kernel(
    const bf16_t* __restrict__ A, int lda,           // activations [rows, K]
    const bf16_t* __restrict__ Bp, size_t b_stride,  // packed weights [E][N-tile][k-tile][kPackN x kPackK]
    bf16_t* __restrict__ C, int ldc,                 // output [rows, SWIGLU ? N/2 : N]
    const MTile* __restrict__ mtiles, const int32_t* __restrict__ counts, int32_t* __restrict__ queues,
    int N, int K, int group_n, RowMap rm,
    float* __restrict__ partials) {  // [slab][kPartRows][N] fp32 sums of entries that cover part of K (plain product only)
    constexpr bool SWIGLU = EPI == kEpiSwiglu;
    constexpr int NW = WGM * WGN;
    constexpr int WTM = BM / WGM, WTN = BN / WGN;
    constexpr int CPR = BK / 8;                 // 16-byte pieces per tile row
    constexpr int IA = BM * CPR / 64;           // wave-wide load instructions per A tile
    constexpr int IB = BN * CPR / 64;
    // per wavefront.  A tile of few rows has fewer activation loads than the workgroup has
    // wavefronts; the upper wavefronts then repeat the lower ones' loads (same pieces to the
    // same place), so that every wavefront counts the same number of loads per k-tile.
    constexpr bool A_SHARED = IA < NW;
    constexpr int IAW = A_SHARED ? 1 : IA / NW, IBW = IB / NW;
    constexpr int LPT = IAW + IBW;              // loads per thread per k-tile
    constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE_BYTES = A_BYTES + B_BYTES;
    constexpr int TM16 = WTM / 16, TN16 = WTN / 16;
    static_assert((A_SHARED ? NW % IA == 0 : IA % NW == 0) && IB % NW == 0, "tile loads must divide over the wavefronts");
    static_assert(WTM % 16 == 0 && WTN % 16 == 0, "wave tile is a grid of 16x16 MFMA tiles");
    static_assert(!SWIGLU || (WTN % 64 == 0), "gate/up pairs must sit in one wavefront");
    static_assert(LPT * NSTAGE < 64, "vmcnt range");
    static_assert(CPR == 8 && BK == 64 && TM16 + TN16 <= 12, "the K loop is written for 64-deep k-tiles");
    static_assert(BN == kPackN && BK == kPackK, "a weight tile is one tile of the packed form");
    // With two stages every wait drains all loads, so loads of rows past the end of a
    // ragged M-tile can simply be left out; with deeper prefetch the wait counts a fixed
    // number of loads per k-tile and such rows are clamped to the last valid row instead.
    constexpr bool SKIP_TAIL_LOADS = (NSTAGE == 2);
    constexpr int ROWS_PER_LOAD = 64 / CPR;

    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;

    const int n_entries = counts[kCntEntries];
    const int pass0_end = counts[kCntPass0];  // whole full-height tiles
    const int pass1_end = counts[kCntPass1];  // whole ragged tiles; behind them the parts of split tiles
    const int n_ntiles = (N + BN - 1) / BN;

    // Tile order.  The (entry, N-tile) space is walked in three passes: the full-height
    // M-tiles, the ragged ones (tallest first), the parts of split tiles (part by part).
    // Inside a pass tiles are numbered in groups of group_n neighbouring N-tiles; inside a
    // group the N-tile index runs fastest, then the entry (full M-tiles are sorted by expert),
    // so a run of 32 consecutive tiles is a patch of about 32/group_n x group_n tiles that
    // share their activation and weight panels.  Workgroups are dealt to the 8 XCDs
    // round-robin (workgroup b runs on XCD b % 8) and every XCD has its own L2, so run c of
    // the numbering belongs to XCD c % 8: its workgroups claim the tiles of its runs one by
    // one from a counter (tiles differ in cost, a fixed deal would leave workgroups idle at
    // the end) and so work side by side on one patch, sharing its panels through that L2; the
    // 8 XCDs are on 8 consecutive runs (further along M under the same weight panels, shared
    // through the memory-side cache).  A workgroup whose own XCD has no tile left claims from
    // the other XCDs' counters.
    const int xcd = blockIdx.x & 7;
    constexpr int run = kGemmGrid / 8;  // the launch is always kGemmGrid workgroups
    const int total = n_entries * n_ntiles;
    const int total0 = pass0_end * n_ntiles, total1 = pass1_end * n_ntiles;
    __shared__ volatile int next_tile;
    // The claims are the business of wavefront 0, and every value involved is the same in
    // all its lanes, so the state lives in scalar registers (lane 0 performs the atomic, its
    // result is broadcast): nothing of it occupies a vector register across the K loop
    // except the pending result of the claim made ahead.
    int dry = 0;  // bit q set = counter q has run out
    // tile number for claim i of XCD q's counter, -1 if that counter has run out
    auto tile_of_claim = [&](int q, int i) {
        const int t = (q + 8 * (i / run)) * run + i % run;
        return t < total ? t : -1;  // claims only grow: past the end once, past the end for good
    };
    // number of claims counter q can serve: its runs are q, q + 8, ... of which the first
    // total / run are whole and run number total / run holds the remainder
    auto claims_of = [&](int q, int total) {  // (total handed in opaque: worked out only when needed)
        const int whole = total / run, part = total - whole * run;
        return (whole > q ? (whole - q + 7) / 8 * run : 0) + ((whole >= q && ((whole - q) & 7) == 0) ? part : 0);
    };
    // the counter to claim from next, own XCD first; -1 when all have run out
    auto next_counter = [&]() {
        for (int j = 0; j < 8; ++j) {
            const int q = (xcd + j) & 7;
            if (!((dry >> q) & 1)) return q;
        }
        return -1;
    };
    auto claim_from = [&](int q) {  // one claim, result not yet waited for (lane 0 holds it)
        int r = 0;
        if (lane == 0) r = atomicAdd(&queues[q], 1);
        return r;
    };
    // Turns a claim made ahead of time (or none: q < 0) into a tile, making further claims as
    // needed; -1 when every counter has run out.  Once a claim has come back empty all eight
    // counters are read in one go (one round trip, not one per counter), and those that stand
    // at their limit are struck off.
    auto settle_claim = [&](int q, int i) {
        for (;;) {
            if (q >= 0) {
                const int t = tile_of_claim(q, i);
                if (t >= 0) return t;
                dry |= 1 << q;
                const int seen = __hip_atomic_load(&queues[opaque(lane) & 7], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const int total_now = opaque_uniform(total);
#pragma unroll
                for (int c = 0; c < 8; ++c)
                    if (__builtin_amdgcn_readlane(seen, c) >= claims_of(c, total_now)) dry |= 1 << c;
            }
            q = next_counter();
            if (q < 0) return -1;
            i = __builtin_amdgcn_readfirstlane(claim_from(q));
        }
    };
    if (wave == 0) next_tile = settle_claim(-1, 0);
    for (;;) {
        lds_wait<0>();                 // thread 0's store of next_tile
        __builtin_amdgcn_s_barrier();  // also: every wavefront is done reading the previous tile's stages
        const int t_all = __builtin_amdgcn_readfirstlane(next_tile);
        if (t_all < 0) break;
        // the claim for the tile after this one is made now and looked at after the K loop
        int ahead_q = -1, ahead_pending = 0;
        if (wave == 0) {
            ahead_q = next_counter();
            if (ahead_q >= 0) ahead_pending = claim_from(ahead_q);
        }
        const int pass = t_all < total0 ? 0 : (t_all < total1 ? 1 : 2);
        const int t = pass == 0 ? t_all : (pass == 1 ? t_all - total0 : t_all - total1);
        const int m_base = pass == 0 ? 0 : (pass == 1 ? pass0_end : pass1_end);
        const int m_count = pass == 0 ? pass0_end : (pass == 1 ? pass1_end - pass0_end : n_entries - pass1_end);
        const int per_group = m_count * group_n;
        const int grp = t / per_group;
        const int rem = t - grp * per_group;
        const int gw = (n_ntiles - grp * group_n) < group_n ? (n_ntiles - grp * group_n) : group_n;
        const int mt_i = m_base + rem / gw;
        const int nt_i = grp * group_n + rem % gw;
        const MTile mt = mtiles[mt_i];
        const int n0 = nt_i * BN;
        // k-tiles of this entry: all of K, or the part of it a split tile covers
        const int KT = mt.kt1 > 0 ? mt.kt1 - mt.kt0 : K / BK;
        // rows that go through a list are addressed from the start of A (32-bit byte offsets:
        // the host checks that A fits), rows in place from the tile's first row
        const bf16_t* Ab = (rm.a_rows ? A : A + (size_t)mt.list0 * lda) + mt.kt0 * BK;
        const bf16_t* Bb = Bp + (size_t)mt.expert * b_stride + ((size_t)nt_i * (K / BK) + mt.kt0) * (BN * BK);
        const int n_valid = (N - n0) < BN ? (N - n0) : BN;

        // per-lane byte offsets of the pieces this lane fetches (activation rows beyond the
        // segment are clamped to the last valid row, weight rows beyond the matrix edge are
        // zero rows of the packed form; their products are computed and dropped in the
        // epilogue).  (uniform base) + (32-bit lane offset) is an addressing mode of the load
        // instruction, so the loads spend no vector ALU work on addresses.  A weight tile is
        // stored as it sits in LDS: load i of the wavefront takes its 1 KiB of it as it comes, so
        // one lane offset serves all of them and the rest of the address is uniform.  Whether
        // that offset is kept in a register or worked out at each load (one instruction) decides,
        // at the 256 registers of the tallest shape, which of the three epilogues the compiler
        // fits without scratch memory: the form below keeps all of them at none.
        constexpr bool KEEP_OFFB = SWIGLU;
        unsigned offA_b[IAW];
        unsigned offB_kept[KEEP_OFFB ? IBW : 1];
        const int lane_p = opaque(lane);
        const int wave_a = A_SHARED ? wave % IA : wave;
#pragma unroll
        for (int i = 0; i < IAW; ++i) {
            const int p = (wave_a + i * NW) * 64 + lane_p;
            const int row = p / CPR, slot = p % CPR;
            int r = row < mt.rows ? row : mt.rows - 1;
            if (rm.a_rows) {
                r = rm.a_rows[mt.list0 + r];
                if (rm.a_rows2) r = rm.a_rows2[r] / opaque_uniform(rm.a_div);
            }
            offA_b[i] = ((unsigned)r * (unsigned)lda + (unsigned)((slot ^ swz(row)) * 8)) * 2u;
        }
        if constexpr (KEEP_OFFB) {
#pragma unroll
            for (int i = 0; i < IBW; ++i) offB_kept[i] = (unsigned)(((wave + i * NW) * 64 + lane_p) * 16);
        }


        // load l of this wavefront's LPT loads of k-tile kt (activations first), one instruction
        const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)smem;
        const unsigned lds_wave = lds_base + (unsigned)wave * 1024u;
        const unsigned lds_wave_a = lds_base + (unsigned)wave_a * 1024u;
        auto issue_load_n = [&](auto L, int kt, int stage) {
            constexpr int l = decltype(L)::value;
            const unsigned sA = lds_wave + (unsigned)(stage * STAGE_BYTES);
            if constexpr (l < IAW) {
                const unsigned char* base = (const unsigned char*)Ab + (size_t)(kt * (BK * 2));
                if (!SKIP_TAIL_LOADS || (wave + l * NW) * ROWS_PER_LOAD < mt.rows)
                    global_to_lds_b128(base, offA_b[l], lds_wave_a + (unsigned)(stage * STAGE_BYTES + l * NW * 1024));
            } else {
                if constexpr (KEEP_OFFB) {
                    const unsigned char* base = (const unsigned char*)Bb + (size_t)kt * B_BYTES;
                    global_to_lds_b128(base, offB_kept[l - IAW], sA + (unsigned)(A_BYTES + (l - IAW) * NW * 1024));
                } else {
                    const unsigned char* base =
                        (const unsigned char*)Bb + ((size_t)kt * B_BYTES + (l - IAW) * NW * 1024);
                    global_to_lds_b128(base, (unsigned)((wave * 64 + opaque(lane)) * 16),
                                       sA + (unsigned)(A_BYTES + (l - IAW) * NW * 1024));
                }
            }
        };
        auto issue_loads = [&](int kt, int stage) {
            static_for<LPT>([&](auto L) { issue_load_n(L, kt, stage); });
        };

        // the first k-tiles are requested before the accumulators are cleared: the clearing
        // then runs while the loads are under way
#pragma unroll
        for (int s = 0; s < NSTAGE; ++s)
            if (s < KT) issue_loads(s, s);
        __builtin_amdgcn_sched_barrier(0);

        // Accumulators hold the transposed product: the weight fragment is the MFMA's row
        // operand and the activation fragment its column operand, so element r of lane
        // (l16, g16) in tile (i, j) is output row i*16 + l16 and output column j*16 + g16*4 + r:
        // four consecutive columns per lane.
        f32x4 acc16[TM16][TN16];
#pragma unroll
        for (int i = 0; i < TM16; ++i)
#pragma unroll
            for (int j = 0; j < TN16; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc16[i][j][r] = 0.f;
        const int lane_k = opaque(lane);
        const int l16 = lane_k & 15, g16 = lane_k >> 4;

        // K loop.  A step is 32 deep: TM16 activation fragments (16 rows each) and TN16 weight
        // fragments, TM16 * TN16 MFMAs, taken row of tiles by row of tiles.  The weight
        // fragments are double-buffered; an activation fragment is free once its row of tiles
        // has been issued, so its register is refilled for the next step right behind that
        // row.  LDS reads complete in issue order (weights of a step first, then its activation
        // fragments 0, 1, ...), which fixes how many may still be in flight before each row.
        // The hand-over to the next k-tile (own loads landed, barrier, refill of the stage just
        // left) opens a k-tile's last step, when every fragment of that k-tile is in a
        // register; the loads of the refill go out one or two per row of tiles.  The loop
        // exists twice: FULL (every 16-row sub-tile of this wavefront is valid, no conditions
        // inside) and ragged (sub-tiles past the end of the M-tile are not multiplied); both run
        // the same sequence of barriers, so wavefronts of one workgroup may take different ones.
        auto k_loop16 = [&](auto full_tag) {
            constexpr bool FULL = decltype(full_tag)::value;
            constexpr int ROW_BYTES = CPR * 16;
            const int rows_w16 = mt.rows - wm * WTM;
            const int tmv16 = rows_w16 <= 0 ? 0 : (rows_w16 >= WTM ? TM16 : (rows_w16 + 15) / 16);
            const int sw16 = swz(l16);  // rows differ by multiples of 16 -> same swizzle
            const unsigned a_base = lds_base + (unsigned)((wm * WTM + l16) * ROW_BYTES);
            const unsigned b_base = lds_base + (unsigned)(A_BYTES + (wn * WTN + l16) * ROW_BYTES);
            bf16x8 af[TM16], bfr[2][TN16];
            auto piece_of = [&](int kt, int ks) {
                return (unsigned)((kt % NSTAGE) * STAGE_BYTES + (((ks * 4 + g16) ^ sw16) * 16));
            };
            auto read_a = [&](auto I, unsigned piece) {
                constexpr int i = decltype(I)::value;
                // read even where the rows lie past the end of a ragged tile (whatever the stage
                // holds there: those tiles are not multiplied), so the count of reads in flight
                // is the same for every wavefront
                lds_read_b128<i * 16 * ROW_BYTES>(af[i], a_base + piece);
            };
            auto read_b_all = [&](int buf, unsigned piece) {
                static_for<TN16>([&](auto J) {
                    constexpr int j = decltype(J)::value;
                    lds_read_b128<j * 16 * ROW_BYTES>(bfr[buf][j], b_base + piece);
                });
            };
            auto row_mfmas = [&](auto I, int buf) {
                constexpr int i = decltype(I)::value;
                lds_landed(af[i]);
                __builtin_amdgcn_sched_barrier(0);
                if (FULL || i < tmv16) {
#pragma unroll
                    for (int j = 0; j < TN16; ++j)
                        acc16[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bfr[buf][j], af[i], acc16[i][j], 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
            };
            // One step.  On entry the reads of its own fragments are in flight or done, in the
            // order weights, activation 0, 1, ...  NEXT: a step follows and its fragments are read
            // here.  HANDOVER: this is the last step of k-tile kt and k-tile kt + 1 exists.
            auto step = [&](int kt, auto ks_tag, auto next_tag, auto hand_tag) {
                constexpr int ks = decltype(ks_tag)::value;
                constexpr bool NEXT = decltype(next_tag)::value, HANDOVER = decltype(hand_tag)::value;
                constexpr int cur = ks & 1, nxt = cur ^ 1;
                const unsigned np = HANDOVER ? piece_of(kt + 1, 0) : piece_of(kt, ks + 1);
                if constexpr (NEXT && !HANDOVER)
                    lds_wait<TM16 - 1>();  // the weights and activation fragment 0 have landed
                else
                    lds_wait<0>();
#pragma unroll
                for (int j = 0; j < TN16; ++j) lds_landed(bfr[cur][j]);
                if constexpr (NEXT && !HANDOVER) read_b_all(nxt, np);
                static_for<TM16>([&](auto I) {
                    constexpr int i = decltype(I)::value;
                    if constexpr (HANDOVER && i == 0) {
                        // every fragment of k-tile kt is in a register (waited for on entry); this
                        // wavefront's pieces of k-tile kt + 1 have landed; the barrier extends both
                        // to every wavefront, so the stage of k-tile kt can be refilled
                        if (KT - 2 - kt >= NSTAGE - 2)
                            wait_vmcnt<LPT*(NSTAGE - 2)>();
                        else
                            wait_vmcnt<0>();
                        __builtin_amdgcn_s_barrier();
                        read_b_all(nxt, np);
                    }
                    if constexpr (i > 0 && NEXT && !HANDOVER)
                        lds_wait<TM16 - 1 + TN16>();  // activation fragment i has landed
                    row_mfmas(I, cur);
                    if constexpr (NEXT) read_a(I, np);
                    if constexpr (HANDOVER) {
                        // the refill of the stage k-tile kt has left: this wavefront's loads of
                        // k-tile kt + NSTAGE, dealt over the rows of tiles behind the hand-over so
                        // that a load waiting for the CU's one address unit holds up a few MFMAs of
                        // this wavefront, not the SIMD (its other wavefront keeps issuing)
                        constexpr int l0 = i * LPT / TM16, l1 = (i + 1) * LPT / TM16;
                        if (kt + NSTAGE < KT)
                            static_for<l1 - l0>([&](auto D) {
                                issue_load_n(std::integral_constant<int, l0 + decltype(D)::value>{}, kt + NSTAGE,
                                             kt % NSTAGE);
                            });
                    }
                });
            };
            if ((!SKIP_TAIL_LOADS || mt.rows == BM) && KT >= NSTAGE)
                wait_vmcnt<LPT*(NSTAGE - 1)>();  // k-tile 0 landed, the others may be in flight
            else
                wait_vmcnt<0>();
            __builtin_amdgcn_s_barrier();
            read_b_all(0, piece_of(0, 0));
            static_for<TM16>([&](auto I) { read_a(I, piece_of(0, 0)); });
            int kt = 0;
            for (; kt + 1 < KT; ++kt) {
                step(kt, std::integral_constant<int, 0>{}, std::true_type{}, std::false_type{});
                step(kt, std::integral_constant<int, 1>{}, std::true_type{}, std::true_type{});
            }
            step(kt, std::integral_constant<int, 0>{}, std::true_type{}, std::false_type{});
            step(kt, std::integral_constant<int, 1>{}, std::false_type{}, std::false_type{});
        };
        if (mt.rows - wm * WTM >= WTM)
            k_loop16(std::true_type{});
        else
            k_loop16(std::false_type{});
        // every wavefront has read next_tile (the K loop holds a barrier)
        if (wave == 0) next_tile = settle_claim(ahead_q, __builtin_amdgcn_readfirstlane(ahead_pending));

        // epilogue: 4 consecutive columns per lane and tile -> 8-byte stores (16 bytes of fp32 partial sums)
        const int lane_e = opaque(lane);
        const int l16e = lane_e & 15, g16e = lane_e >> 4;
        const int n_out = SWIGLU ? N / 2 : N;
        const int col0 = (SWIGLU ? (n0 + wn * WTN) / 2 : (n0 + wn * WTN));
        constexpr int TNO16 = SWIGLU ? TN16 / 2 : TN16;  // 16-column tiles of output per wavefront
        static_assert(!SWIGLU || TN16 % 4 == 0, "gate and up tiles pair up inside 64 packed columns");
        float* slab = nullptr;
        if constexpr (EPI == kEpiNone)
            if (mt.part >= 0) slab = partials + (size_t)mt.part * kPartRows * N;
        // output row and scale of this lane's TM16 rows, fetched as one batch (row by row each
        // would wait out a memory round trip, and with it the stores of the row before)
        int crow_of[TM16];
        float sc_of[TM16];
#pragma unroll
        for (int i = 0; i < TM16; ++i) {
            const int row = wm * WTM + i * 16 + l16e;
            crow_of[i] = mt.list0 + (row < mt.rows ? row : mt.rows - 1);
            sc_of[i] = 1.0f;
        }
        if constexpr (EPI == kEpiNone) {
            if (!slab) {
                if (rm.c_rows) {
#pragma unroll
                    for (int i = 0; i < TM16; ++i) crow_of[i] = rm.c_rows[crow_of[i]];
                }
                if (rm.scale) {
                    int si[TM16];
#pragma unroll
                    for (int i = 0; i < TM16; ++i) si[i] = rm.scale_idx[crow_of[i]];
#pragma unroll
                    for (int i = 0; i < TM16; ++i) sc_of[i] = rm.scale[si[i]];
                }
            }
        }
        // values of output tile jo (16 columns) of row block i for this lane: 4 consecutive columns
        auto tile_values = [&](int i, int jo, float sc, float (&v)[4]) {
            // output tile jo: packed tiles (jo/2)*4 + jo%2 (gate) and + 2 (up) with SwiGLU
            const int jg = SWIGLU ? (jo / 2) * 4 + (jo % 2) : jo;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (SWIGLU)
                    v[c] = silu_f(acc16[i][jg][c]) * acc16[i][jg + 2][c];
                else if (EPI == kEpiRelu)
                    v[c] = fmaxf(acc16[i][jg][c], 0.f);
                else
                    v[c] = acc16[i][jg][c] * sc;
            }
        };
        if (slab) {
#pragma unroll
            for (int i = 0; i < TM16; ++i) {
                const int row = wm * WTM + i * 16 + l16e;
                if (row < mt.rows) {
#pragma unroll
                    for (int jo = 0; jo < TNO16; ++jo)
                        if (col0 + jo * 16 < n_out) {
                            float v[4];
                            tile_values(i, jo, 1.0f, v);
                            float4 o;
                            o.x = v[0];
                            o.y = v[1];
                            o.z = v[2];
                            o.w = v[3];
                            *(float4*)(slab + (size_t)row * N + col0 + jo * 16 + g16e * 4) = o;
                        }
                }
            }
        } else {
            // Rounded to bf16 a lane holds 8 bytes of a row per output tile.  Two tiles side by
            // side are regrouped with the two lane-swap instructions (quarter q of the wavefront
            // = lanes 16q .. 16q+15, all of one row set): swapping the upper half of the first
            // tile's register with the lower half of the second's, then the odd quarters of the
            // first with the even quarters of the second, leaves quarter q with columns 8q .. 8q+3
            // of the 32 in the first register and 8q+4 .. 8q+7 in the second: 16 bytes in a row
            // per lane, half as many store instructions, each writing 64-byte pieces.
            static_assert(TNO16 % 2 == 0, "output tiles are stored in pairs");
#pragma unroll
            for (int i = 0; i < TM16; ++i) {
                const int row = wm * WTM + i * 16 + l16e;
                bf16_t* crow = C + (size_t)crow_of[i] * ldc + col0 + g16e * 8;
#pragma unroll
                for (int jo = 0; jo < TNO16; jo += 2) {
                    float v0[4], v1[4];
                    tile_values(i, jo, sc_of[i], v0);
                    tile_values(i, jo + 1, sc_of[i], v1);
                    unsigned px = pack_bf16x2(v0[0], v0[1]), py = pack_bf16x2(v0[2], v0[3]);
                    unsigned qx = pack_bf16x2(v1[0], v1[1]), qy = pack_bf16x2(v1[2], v1[3]);
                    lane_swap_pairs(px, qx);
                    lane_swap_pairs(py, qy);
                    if (row < mt.rows && col0 + jo * 16 < n_out) {
                        uint4 o;
                        o.x = px;
                        o.y = py;
                        o.z = qx;
                        o.w = qy;
                        *(uint4*)(crow + jo * 16) = o;
                    }
                }
            }
        }
    }
}

// Adds up the fp32 slabs of every split M-tile in the order of the parts and writes the rows
// as bf16: y[c_rows[list0 + r]] = scale * (((P_0[r] + P_1[r]) + P_2[r]) + ...).  blockIdx.x =
// split tile, blockIdx.y strides over its rows; counts[kCntSplit] = number of such tiles.
__global__ __launch_bounds__(256) void add_partials_kernel(const float* __restrict__ partials,
                                                            const SplitInfo* __restrict__ splits,
                                                            const int32_t* __restrict__ counts, int parts,
                                                            bf16_t* __restrict__ C, int ldc, int N, RowMap rm) {
    const int n_split = counts[kCntSplit];
    const int n4 = N / 4;
    for (int t = blockIdx.x; t < n_split; t += gridDim.x) {
        const SplitInfo si = splits[t];
        const float* p0 = partials + (size_t)t * parts * kPartRows * N;
        for (int r = blockIdx.y; r < si.rows; r += gridDim.y) {
            int crow = si.list0 + r;
            float sc = 1.0f;
            if (rm.c_rows) crow = rm.c_rows[crow];
            if (rm.scale) sc = rm.scale[rm.scale_idx[crow]];
            uint2* out = (uint2*)(C + (size_t)crow * ldc);
            for (int c = threadIdx.x; c < n4; c += blockDim.x) {
                float4 s = ((const float4*)(p0 + (size_t)r * N))[c];
                for (int q = 1; q < parts; ++q) {
                    const float4 v = ((const float4*)(p0 + ((size_t)q * kPartRows + r) * N))[c];
                    s.x += v.x;
                    s.y += v.y;
                    s.z += v.z;
                    s.w += v.w;
                }
                uint2 o;
                o.x = pack_bf16x2(s.x * sc, s.y * sc);
                o.y = pack_bf16x2(s.z * sc, s.w * sc);
                out[c] = o;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// fp32 grouped GEMM (plain FMA, k ascending): 64x64 tile, 4x4 per thread
// ---------------------------------------------------------------------------
template <bool SWIGLU>
__global__ __launch_bounds__(256) void grouped_gemm_f32_kernel(const float* __restrict__ A, int lda,
                                                                const float* __restrict__ B1,
                                                                const float* __restrict__ B3, size_t b_stride,
                                                                float* __restrict__ C, int ldc,
                                                                const MTile* __restrict__ mtiles,
                                                                const int32_t* __restrict__ counts, int N,
                                                                int K, RowMap rm, int relu) {
    constexpr int BM = 64, BN = 64, BK = 16;
    __shared__ float sA[BK][BM + 4];
    __shared__ float sB1[BK][BN + 4];
    __shared__ float sB3[SWIGLU ? BK : 1][BN + 4];
    __shared__ int srow[BM];
    const int n_mtiles = counts[kCntEntries];
    const int n_ntiles = (N + BN - 1) / BN;
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;  // 16 x 16 threads, 4x4 outputs each
    for (int tile = blockIdx.x; tile < n_mtiles * n_ntiles; tile += gridDim.x) {
        const MTile mt = mtiles[tile / n_ntiles];
        const int n0 = (tile % n_ntiles) * BN;
        const float* b1 = B1 + (size_t)mt.expert * b_stride;
        const float* b3 = SWIGLU ? B3 + (size_t)mt.expert * b_stride : nullptr;
        __syncthreads();
        if (tid < BM) {
            int r = mt.list0 + (tid < mt.rows ? tid : mt.rows - 1);
            if (rm.a_rows) {
                r = rm.a_rows[r];
                if (rm.a_rows2) r = rm.a_rows2[r] / rm.a_div;
            }
            srow[tid] = r;
        }
        float acc1[4][4] = {}, acc3[4][4] = {};
        for (int k0 = 0; k0 < K; k0 += BK) {
            __syncthreads();
            for (int i = tid; i < BM * BK; i += 256) {
                const int r = i / BK, c = i % BK;
                sA[c][r] = (k0 + c < K) ? A[(size_t)srow[r] * lda + k0 + c] : 0.f;
            }
            for (int i = tid; i < BK * BN; i += 256) {
                const int r = i / BN, c = i % BN;
                const bool ok = (k0 + r < K) && (n0 + c < N);
                sB1[r][c] = ok ? b1[(size_t)(k0 + r) * N + n0 + c] : 0.f;
                if (SWIGLU) sB3[r][c] = ok ? b3[(size_t)(k0 + r) * N + n0 + c] : 0.f;
            }
            __syncthreads();
#pragma unroll
            for (int kk = 0; kk < BK; ++kk) {
                float a[4], p[4], q[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) a[i] = sA[kk][ty * 4 + i];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    p[j] = sB1[kk][tx * 4 + j];
                    q[j] = SWIGLU ? sB3[kk][tx * 4 + j] : 0.f;
                }
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        acc1[i][j] = fmaf(a[i], p[j], acc1[i][j]);
                        if (SWIGLU) acc3[i][j] = fmaf(a[i], q[j], acc3[i][j]);
                    }
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = ty * 4 + i;
            if (row >= mt.rows) continue;
            int crow = mt.list0 + row;
            float sc = 1.0f;
            if (rm.c_rows) crow = rm.c_rows[crow];
            if (rm.scale) sc = rm.scale[rm.scale_idx[crow]];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int col = n0 + tx * 4 + j;
                if (col < N) {
                    float v = acc1[i][j];
                    if (SWIGLU) v = v / (1.0f + expf(-v)) * acc3[i][j];
                    else if (relu) v = fmaxf(v, 0.f);
                    C[(size_t)crow * ldc + col] = v * sc;
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
struct FfnWs {
    void* h;            // [A, ffn] hidden activations, in row-list order
    int32_t* rowlist;   // [A] row of x_perm / y_perm at each list position
    MTile* tiles1;      // M-tile table of the first product
    MTile* tiles2;      // and of the second
    int32_t* counts;    // kCntStride ints per table
    int32_t* queues;    // [0..7], [8..15]: per-XCD claim counters of the two products
    SplitInfo* splits;  // split M-tiles of the second product, else null
    float* partials;    // their fp32 slabs: [split tile][part][kPartRows][d]
    int capacity;       // entries per table
    int split_capacity; // split M-tiles (0: the second product is never split)
    int parts;          // parts of K of a split tile
    int split_all;      // every tile is split (tests)
};

constexpr int kMinBM = 32;  // the lowest tile shape

// Process-wide overrides of the automatic choices (moe_grouped_ffn_set_option); -1 / 0 = automatic.
static std::atomic<int> g_opt_tile1{-1}, g_opt_tile2{-1}, g_opt_split{-1}, g_opt_group_n{0};

// The bf16 kernels work on a hidden width padded to a multiple of 64: the packed weights
// carry zero columns (W1, W3) and zero rows (W2) for the padding, so the padded hidden
// activations are exact zeros and add nothing to the second product.
// Widths above this are refused: it keeps every size computed on the host inside 64 bits and
// every tile offset computed on the device inside 32.
constexpr int kMaxWidth = 1 << 22;
static inline bool ffn_shape_in_range(int64_t A, int d, int ffn, int nseg, int dtype) {
    return (dtype == MOE_DTYPE_F32 || dtype == MOE_DTYPE_BF16) && A >= 0 && A < (1ll << 31) && d >= 1 &&
           d <= kMaxWidth && ffn >= 1 && ffn <= kMaxWidth && nseg >= 1 && nseg <= MOE_MAX_SEGMENTS;
}

static inline int padded_ffn(int ffn, int dtype) {
    return dtype == MOE_DTYPE_BF16 ? (int)align_up((size_t)ffn, 64) : ffn;
}
// rows of a packed bf16 weight matrix: whole tiles
static inline size_t packed_rows(size_t n) { return align_up(n, (size_t)kPackN); }
// elements of one expert's packed matrices: the first product's n1 matrices, the second product's
static inline size_t packed_elems1(int n1, int d, int fp) { return packed_rows((size_t)n1 * fp) * d; }
static inline size_t packed_elems2(int d, int fp) { return packed_rows((size_t)d) * fp; }

// Whether (and how) the closing tiles of the second product are computed as parts of K.  It
// pays when the product has only a few rounds of tiles per workgroup, so that the uneven end
// of the launch matters, and the segments are not slivers (decode streams weights; splitting K
// would only add traffic).  Decided from the sizes the workspace is laid out for, so that the
// layout and the call agree.  split_capacity bounds the M-tiles the table builder may split:
// at most 5/8 of a round of tiles, each M-tile at least half a tile's worth per N-tile.
static void split_plan(int64_t A, int d, int ffn, int nseg, int dtype, int* split_capacity, int* parts,
                       int* split_all) {
    *split_capacity = *parts = *split_all = 0;
    if (dtype != MOE_DTYPE_BF16 || A < 1) return;
    const int mode = g_opt_split.load();  // 0: never, 1: every tile whenever the kernels can (for tests), -1: rule
    if (mode == 0) return;
    const int kt = padded_ffn(ffn, dtype) / 64;
    const int n_ntiles = ceil_div(d, 256);
    const int64_t all_mtiles = ceil_div64(A, 128) + (A < nseg ? A : nseg);
    if (mode == 1) {
        if (kt < 2) return;
        *parts = kt >= kMaxParts ? kMaxParts : 2;
        *split_all = 1;
        *split_capacity = (int)(ceil_div64(A, kMinBM) + (A < nseg ? A : nseg));  // every M-tile of any shape
        return;
    }
    if (kt < 4 * kMaxParts) return;
    // slivers of rows stream weights: splitting a tile of a few k-tiles only adds traffic, but a
    // long one (64 k-tiles and more) is worth splitting where the tiles do not fill the chip
    // (8 experts of hidden width 14336 at a few tokens: 96 tiles of 224 k-tiles for 256 workgroups)
    // (eight parts instead of four: 5 % faster at 16 and 32 tokens, 5-20 % slower from 64 on, where
    // adding up the slabs costs more than the extra round saves)
    if (A < (int64_t)64 * nseg && kt < 64) return;
    const int64_t est_tiles = (A / 256 + (nseg + 1) / 2) * n_ntiles;
    if (est_tiles > 8 * kGemmGrid) return;
    *parts = kMaxParts;
    const int64_t by_rule = (int64_t)2 * ceil_div(5 * kGemmGrid / 8, n_ntiles) + 2;
    *split_capacity = (int)(by_rule < all_mtiles ? by_rule : all_mtiles);
}

static size_t ffn_ws_layout(int64_t A, int d, int ffn, int nseg, int dtype, char* base, FfnWs* ws) {
    size_t off = 0;
    auto take = [&](size_t bytes) {
        void* p = base ? (void*)(base + off) : nullptr;
        off += align_up(bytes, 256);
        return p;
    };
    const int64_t A1 = A > 0 ? A : 1;
    FfnWs w;
    split_plan(A, d, ffn, nseg, dtype, &w.split_capacity, &w.parts, &w.split_all);
    w.capacity = (int)(ceil_div64(A1, kMinBM) + nseg + (int64_t)w.split_capacity * kMaxParts);
    w.h = take((size_t)A1 * padded_ffn(ffn, dtype) * dtype_size(dtype));
    w.rowlist = (int32_t*)take((size_t)A1 * sizeof(int32_t));
    w.tiles1 = (MTile*)take((size_t)w.capacity * sizeof(MTile));
    w.tiles2 = (MTile*)take((size_t)w.capacity * sizeof(MTile));
    w.counts = (int32_t*)take(256);
    w.queues = w.counts ? w.counts + 2 * kCntStride : nullptr;
    w.splits = nullptr;
    w.partials = nullptr;
    if (w.split_capacity > 0) {
        w.splits = (SplitInfo*)take((size_t)w.split_capacity * sizeof(SplitInfo));
        w.partials = (float*)take((size_t)w.split_capacity * w.parts * kPartRows * d * sizeof(float));
    }
    if (ws) *ws = w;
    return off;
}

struct GemmVariant {
    int bm, bn, bk;
    size_t lds;
    int threads;
    void (*kern)(const bf16_t*, int, const bf16_t*, size_t, bf16_t*, int, const MTile*, const int32_t*, int32_t*, int,
                 int, int, RowMap, float*);
    std::atomic<unsigned long long>* attr_set;  // bit per device: the dynamic-LDS attribute has been raised
};

template <int BM, int BN, int BK, int WGM, int WGN, int NSTAGE, int EPI>
static GemmVariant make_variant() {
    static std::atomic<unsigned long long> attr_set{0};
    GemmVariant v;
    v.bm = BM;
    v.bn = BN;
    v.bk = BK;
    v.lds = (size_t)NSTAGE * (BM + BN) * BK * 2;
    v.threads = WGM * WGN * 64;
    v.kern = grouped_gemm_bf16_kernel<BM, BN, BK, WGM, WGN, NSTAGE, EPI>;
    v.attr_set = &attr_set;
    return v;
}

// Tile shapes built into the library: 0 = 256x256x64 with two LDS stages, 1 = 128x256x64 with
// three (for products with too few 256-row tiles to fill the chip twice), 2 = 32x256x64 with
// four (for slivers of a few rows per expert, where the product only streams weights: three
// k-tiles of a weight panel in flight per workgroup instead of two, and an eighth of the
// activation tile to fetch for rows that are not there).
constexpr int kNumVariants = 3;
static const GemmVariant kGemmSwiglu[kNumVariants] = {make_variant<256, 256, 64, 2, 4, 2, kEpiSwiglu>(),
                                                      make_variant<128, 256, 64, 2, 4, 3, kEpiSwiglu>(),
                                                      make_variant<32, 256, 64, 2, 4, 4, kEpiSwiglu>()};
static const GemmVariant kGemmRelu[kNumVariants] = {make_variant<256, 256, 64, 2, 4, 2, kEpiRelu>(),
                                                    make_variant<128, 256, 64, 2, 4, 3, kEpiRelu>(),
                                                    make_variant<32, 256, 64, 2, 4, 4, kEpiRelu>()};
static const GemmVariant kGemmPlain[kNumVariants] = {make_variant<256, 256, 64, 2, 4, 2, kEpiNone>(),
                                                     make_variant<128, 256, 64, 2, 4, 3, kEpiNone>(),
                                                     make_variant<32, 256, 64, 2, 4, 4, kEpiNone>()};

// timing hook: events recorded around the two products of the next call on this thread
static thread_local hipEvent_t g_time_events[4];
static thread_local bool g_time_armed = false;

static int num_cus() {
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
            cus = prop.multiProcessorCount;
        if (cus <= 0) cus = 256;
    }
    return cus;
}

static int launch_gemm_bf16(const GemmVariant& v, const bf16_t* A, int lda, const bf16_t* Bp, size_t b_stride,
                            bf16_t* C, int ldc, const MTile* tiles, const int32_t* counts, int32_t* queues, int N,
                            int K, int group_n, const RowMap& rm, float* partials, hipStream_t st) {
    // the kernels use more LDS than the default limit: raised once per kernel and device
    int dev = 0;
    (void)hipGetDevice(&dev);
    const unsigned long long bit = 1ull << (dev & 63);
    if (!(v.attr_set->load() & bit)) {
        hipError_t e = hipFuncSetAttribute((const void*)v.kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)v.lds);
        if (e != hipSuccess) {
            set_last_hip_error(e);
            return MOE_ERR_HIP;
        }
        v.attr_set->fetch_or(bit);
    }
    // 32 workgroups for each of the 8 XCDs; they claim tiles from `queues` (cleared by the table builder)
    hipLaunchKernelGGL(v.kern, dim3(kGemmGrid), dim3(v.threads), v.lds, st, A, lda, Bp, b_stride, C, ldc, tiles,
                       counts, queues, N, K, group_n, rm, partials);
    return check_launch();
}

}  // namespace moegps

extern "C" int moe_grouped_ffn_set_option(int option, int value) {
    using namespace moegps;
    switch (option) {
        case MOE_FFN_OPT_TILE1:
        case MOE_FFN_OPT_TILE2:
            if (value < -1 || value >= kNumVariants) return MOE_ERR_INVALID_ARG;
            (option == MOE_FFN_OPT_TILE1 ? g_opt_tile1 : g_opt_tile2).store(value);
            return MOE_OK;
        case MOE_FFN_OPT_SPLIT_K:
            if (value < -1 || value > 1) return MOE_ERR_INVALID_ARG;
            g_opt_split.store(value);
            return MOE_OK;
        case MOE_FFN_OPT_GROUP_N:
            if (value < 0) return MOE_ERR_INVALID_ARG;
            g_opt_group_n.store(value);
            return MOE_OK;
        default:
            return MOE_ERR_INVALID_ARG;
    }
}

extern "C" size_t moe_packed_weights_bytes(int E, int d, int ffn, int dtype) {
    using namespace moegps;
    if (E < 1 || E > MOE_MAX_EXPERTS || !ffn_shape_in_range(0, d, ffn, 1, dtype)) return 0;
    if (dtype != MOE_DTYPE_BF16) return (size_t)3 * E * d * ffn * dtype_size(dtype);
    const int fp = padded_ffn(ffn, dtype);
    return (size_t)E * (packed_elems1(2, d, fp) + packed_elems2(d, fp)) * sizeof(bf16_t);
}

namespace moegps {
// W3 == nullptr packs the ReLU form (no gate matrix): [W1 | W2] instead of [W1 W3 | W2]
static int pack_weights_impl(const void* W1, const void* W3, const void* W2, int dtype, int E, int d, int ffn,
                             void* packed, void* stream) {
    if (dtype != MOE_DTYPE_F32 && dtype != MOE_DTYPE_BF16) return MOE_ERR_INVALID_ARG;
    if (E < 1 || d < 1 || ffn < 1 || !W1 || !W2 || !packed) return MOE_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    const size_t per = (size_t)E * d * ffn;
    if (dtype == MOE_DTYPE_F32) {
        if ((per * 4) % 16 != 0) return MOE_ERR_UNSUPPORTED;
        const void* src[3] = {W1, W3 ? W3 : W2, W2};
        const int n = W3 ? 3 : 2;
        for (int i = 0; i < n; ++i) {
            hipLaunchKernelGGL(copy_u4_kernel, dim3(1024), dim3(256), 0, st, (const uint4*)src[i],
                               (uint4*)((float*)packed + i * per), per * 4 / 16);
            int rc = check_launch();
            if (rc != MOE_OK) return rc;
        }
        return MOE_OK;
    }
    if (d % 64 != 0) return MOE_ERR_UNSUPPORTED;
    if (E > 65535) return MOE_ERR_UNSUPPORTED;
    const int fp = padded_ffn(ffn, dtype);
    const int n1 = W3 ? 2 : 1;              // matrices in the first product
    const size_t es = (size_t)d * ffn;      // one expert's matrix as given
    const size_t e1 = packed_elems1(n1, d, fp), e2 = packed_elems2(d, fp);  // and packed
    bf16_t* p1 = (bf16_t*)packed;           // [E] packed [n1*fp][d]; gate/up interleaved by 32 columns when n1 = 2
    bf16_t* p2 = p1 + (size_t)E * e1;       // [E] packed [d][fp]
    // W1 (, W3): in[k = d][n = ffn] -> rows n' of the packed matrix, zero rows for n >= ffn and up
    // to whole tiles of rows
    const int rows1 = (int)(packed_rows((size_t)n1 * fp) / n1);  // rows per matrix, padding included
    dim3 g13(rows1 / 32, d / 32, E);
    hipLaunchKernelGGL(pack_transpose_kernel, g13, dim3(256), 0, st, (const bf16_t*)W1, p1, d, ffn, d, rows1, es, e1,
                       W3 ? 1 : 0, 0);
    int rc = check_launch();
    if (rc != MOE_OK) return rc;
    if (W3) {
        hipLaunchKernelGGL(pack_transpose_kernel, g13, dim3(256), 0, st, (const bf16_t*)W3, p1, d, ffn, d, rows1, es,
                           e1, 1, 1);
        if ((rc = check_launch()) != MOE_OK) return rc;
    }
    // W2: in[k = ffn][n = d] -> packed [n = d][k = fp], zero for k >= ffn and rows n >= d
    const int rows2 = (int)packed_rows((size_t)d);
    dim3 g2(rows2 / 32, fp / 32, E);
    hipLaunchKernelGGL(pack_transpose_kernel, g2, dim3(256), 0, st, (const bf16_t*)W2, p2, ffn, d, fp, rows2, es, e2,
                       0, 0);
    return check_launch();
}
}  // namespace moegps

extern "C" int moe_pack_weights(const void* W1, const void* W3, const void* W2, int dtype, int E, int d, int ffn,
                                void* packed, void* stream) {
    if (!W3) return MOE_ERR_INVALID_ARG;
    return moegps::pack_weights_impl(W1, W3, W2, dtype, E, d, ffn, packed, stream);
}

extern "C" size_t moe_packed_weights_relu_bytes(int E, int d, int ffn, int dtype) {
    using namespace moegps;
    if (E < 1 || E > MOE_MAX_EXPERTS || !ffn_shape_in_range(0, d, ffn, 1, dtype)) return 0;
    if (dtype != MOE_DTYPE_BF16) return (size_t)2 * E * d * ffn * dtype_size(dtype);
    const int fp = padded_ffn(ffn, dtype);
    return (size_t)E * (packed_elems1(1, d, fp) + packed_elems2(d, fp)) * sizeof(bf16_t);
}

extern "C" int moe_pack_weights_relu(const void* W1, const void* W2, int dtype, int E, int d, int ffn, void* packed,
                                     void* stream) {
    return moegps::pack_weights_impl(W1, nullptr, W2, dtype, E, d, ffn, packed, stream);
}

extern "C" size_t moe_grouped_ffn_workspace_bytes(int64_t A, int d, int ffn, int nseg, int dtype) {
    using namespace moegps;
    if (!ffn_shape_in_range(A, d, ffn, nseg, dtype)) return 0;
    return ffn_ws_layout(A, d, ffn, nseg, dtype, nullptr, nullptr);
}

namespace moegps {
// Rows of the first product: x_perm rows in place (gather_rows == nullptr; `rows_in` = A), or
// row r is x[gather_rows[r] / gather_div] (`rows_in` = rows of x).  With `scale`, row r of
// the output is multiplied by scale[scale_idx[r]] before it is rounded.
static int grouped_ffn_impl(int relu, const void* x_in, int64_t rows_in, const int32_t* gather_rows, int gather_div,
                            const int32_t* scale_idx, const float* scale, int dtype, int64_t A, int d, int ffn,
                            int E, const int32_t* seg_offsets, const int32_t* slot_expert, int nseg, int seg_begin,
                            int seg_end, const void* packed, void* y_perm, void* workspace, size_t workspace_bytes,
                            void* stream) {
    const bool timed = g_time_armed;
    g_time_armed = false;  // the hook belongs to this call, whatever becomes of it
    if (dtype != MOE_DTYPE_F32 && dtype != MOE_DTYPE_BF16) return MOE_ERR_INVALID_ARG;
    if (A < 0 || d < 1 || ffn < 1 || E < 1 || nseg < 1) return MOE_ERR_INVALID_ARG;
    if (seg_begin < 0 || seg_end > nseg || seg_begin > seg_end) return MOE_ERR_INVALID_ARG;
    if (nseg > MOE_MAX_SEGMENTS || E > MOE_MAX_EXPERTS || A >= (1ll << 31)) return MOE_ERR_UNSUPPORTED;
    if (d > kMaxWidth || ffn > kMaxWidth) return MOE_ERR_UNSUPPORTED;
    if (dtype == MOE_DTYPE_BF16 && d % 64 != 0) return MOE_ERR_UNSUPPORTED;
    if (dtype == MOE_DTYPE_F32 && (d % 4 != 0 || ffn % 4 != 0)) return MOE_ERR_UNSUPPORTED;
    if ((int64_t)256 * (d > ffn + 63 ? d : ffn + 63) >= (1ll << 31)) return MOE_ERR_UNSUPPORTED;  // 32-bit tile offsets
    if (dtype == MOE_DTYPE_BF16 && rows_in * (int64_t)d >= (1ll << 31)) return MOE_ERR_UNSUPPORTED;  // 32-bit row offsets
    if (!seg_offsets || !slot_expert || !packed || !workspace) return MOE_ERR_INVALID_ARG;
    if (A > 0 && (!x_in || !y_perm)) return MOE_ERR_INVALID_ARG;
    if ((scale != nullptr) != (scale_idx != nullptr)) return MOE_ERR_INVALID_ARG;
    FfnWs ws;
    const size_t need = ffn_ws_layout(A, d, ffn, nseg, dtype, (char*)workspace, &ws);
    if (workspace_bytes < need) return MOE_ERR_WORKSPACE_TOO_SMALL;
    if (A == 0 || seg_begin == seg_end) return MOE_OK;
    hipStream_t st = (hipStream_t)stream;
    const size_t per = (size_t)E * d * ffn;
    const int nrange = seg_end - seg_begin;
    const int build_grid = (int)(A / 4096 < 2 ? 2 : (A / 4096 > 64 ? 64 : A / 4096));
    int rc;
    RowMap rm1{ws.rowlist, gather_rows, gather_div, nullptr, nullptr, nullptr};
    RowMap rm2{nullptr, nullptr, 1, ws.rowlist, scale_idx, scale};

    if (dtype == MOE_DTYPE_F32) {
        TableSpec t1{ws.tiles1, ws.counts, nullptr, 64, ws.capacity, 0, 0, 1, 1, 0, 0};
        TableSpec none{};
        hipLaunchKernelGGL(build_tables_kernel, dim3(build_grid), dim3(1024), 0, st, seg_offsets, slot_expert,
                           seg_begin, seg_end, E, t1, none, ws.rowlist, (int32_t*)nullptr, 0);
        if ((rc = check_launch()) != MOE_OK) return rc;
        const float* w1 = (const float*)packed;
        const float* w3 = w1 + per;
        const float* w2 = relu ? w3 : w3 + per;
        const int grid = 4 * num_cus();
        if (relu)
            hipLaunchKernelGGL((grouped_gemm_f32_kernel<false>), dim3(grid), dim3(256), 0, st, (const float*)x_in, d,
                               w1, (const float*)nullptr, (size_t)d * ffn, (float*)ws.h, ffn, ws.tiles1, ws.counts,
                               ffn, d, rm1, 1);
        else
            hipLaunchKernelGGL((grouped_gemm_f32_kernel<true>), dim3(grid), dim3(256), 0, st, (const float*)x_in, d,
                               w1, w3, (size_t)d * ffn, (float*)ws.h, ffn, ws.tiles1, ws.counts, ffn, d, rm1, 0);
        if ((rc = check_launch()) != MOE_OK) return rc;
        hipLaunchKernelGGL((grouped_gemm_f32_kernel<false>), dim3(grid), dim3(256), 0, st, (const float*)ws.h, ffn,
                           w2, (const float*)nullptr, (size_t)d * ffn, (float*)y_perm, d, ws.tiles1, ws.counts, d,
                           ffn, rm2, 0);
        return check_launch();
    }

    // Tile shape per product: 256x256 unless the product has too few such tiles to keep 256
    // workgroups busy for two rounds, or the segments are slivers of a few rows each
    // (decode), then 128x256 with three stages.  The tile count is only known on the device;
    // the host estimates it from the row count.  A product of slivers with few k-tiles per tile
    // (the second product at the hidden widths of fine-grained experts) takes 32x256 with four
    // stages: the taller shapes fetch their whole activation tile every k-tile, rows that are
    // not there as copies of the last one, half as many bytes again as the weights at 128 rows
    // (decode at 128 experts, 24 k-tiles: 0.201 -> 0.192 ms; 64x256 with four stages stays at
    // 0.200); on long tiles that does not make up for the extra M-tiles of experts with more
    // than 32 rows (same batch, first product, 64 k-tiles: 0.369 -> 0.392 ms).
    auto pick = [&](int forced, int n_cols, int k_tiles) {
        if (forced >= 0) return forced;
        if (A < (int64_t)16 * nrange && k_tiles <= 32) return 2;
        if (A < (int64_t)64 * nrange) return 1;
        // fewer than 256 rows per expert on average: most 256-row tiles would be ragged (128
        // experts, 16384 rows: 623 against 683 us for the first product; 64 experts, 12288 rows:
        // 226 against 258 us; at 256 rows per expert the shapes are within 4 % of each other, at
        // 384 equal)
        const int64_t experts = E < nrange ? E : nrange;
        if (A < 256 * experts) return 1;
        // few tiles: the 128-row shape fills the chip better, unless the experts are large
        // enough for whole 256-row tiles and those still make more than one round (8 experts,
        // 4096 rows, second product: 476 against 521 us)
        const int64_t est_tiles = (A / 256 + (nrange + 1) / 2) * ceil_div(n_cols, 256);
        if (A >= 512 * experts) return est_tiles > kGemmGrid ? 0 : 1;
        return est_tiles > 2 * kGemmGrid ? 0 : 1;
    };
    const int fp = padded_ffn(ffn, dtype);  // hidden width the kernels see
    const int n1 = relu ? 1 : 2;            // matrices in the first product
    const int v1 = pick(g_opt_tile1.load(), n1 * fp, d / 64);
    const int v2 = pick(g_opt_tile2.load(), d, fp / 64);
    // N-tiles walked side by side under one run of M-tiles.  A run of 32 tiles is 32/g M-tiles
    // under g weight panels; every group streams the activation rows again.  Up to 12 N-tiles
    // are walked together, so the rows are read once.  Wider outputs are walked in groups: of 4
    // while the rows stay in the memory-side cache (8 M-tiles share each weight panel), else of
    // 6, the near-square patch that fetches the fewest panels per run; 13 to 16 N-tiles over
    // more than 1 GiB of rows are walked in two groups of 8.  Measured: Mixtral-shaped gate/up
    // at 64 MiB of rows, 4 is 3-4 % faster than 8; at 512 MiB, 6 is 1 % faster than 8 and 4 is
    // 1.5 % slower; down products of 16 N-tiles, 6 is 2-8 % faster than 16 below 1 GiB of rows,
    // 8 is 2 % faster than 6 at 1.9 GiB.
    const int group_opt = g_opt_group_n.load();
    auto group_for = [&](int n_cols, int bn, int64_t a_bytes) {
        if (group_opt > 0) return group_opt;
        const int n_ntiles = ceil_div(n_cols, bn);
        if (n_ntiles <= 12) return n_ntiles;
        if (n_ntiles <= 16) return a_bytes <= ((int64_t)1 << 30) ? 6 : 8;
        return a_bytes <= ((int64_t)96 << 20) ? 4 : 6;
    };
    const GemmVariant& g1 = relu ? kGemmRelu[v1] : kGemmSwiglu[v1];
    const GemmVariant& g2 = kGemmPlain[v2];
    const bool split = ws.split_capacity > 0;
    // one launch builds the row list and both tables; the second product shares the first one's
    // table when it has the same tile height and splits nothing
    const bool own2 = g2.bm != g1.bm || split;
    TableSpec t1{ws.tiles1, ws.counts, nullptr, g1.bm, ws.capacity, d / g1.bk, 0, 1, kGemmGrid, 0, 0};
    TableSpec t2{own2 ? ws.tiles2 : nullptr, ws.counts + kCntStride, ws.splits, g2.bm, ws.capacity, fp / g2.bk,
                 split ? ws.parts : 0, ceil_div(d, g2.bn), kGemmGrid, ws.split_all, ws.split_capacity};
    hipLaunchKernelGGL(build_tables_kernel, dim3(build_grid), dim3(1024), 0, st, seg_offsets, slot_expert, seg_begin,
                       seg_end, E, t1, t2, ws.rowlist, ws.queues, 16);
    if ((rc = check_launch()) != MOE_OK) return rc;
    const MTile* tiles2 = own2 ? ws.tiles2 : ws.tiles1;
    const int32_t* count2 = own2 ? ws.counts + kCntStride : ws.counts;
    const bf16_t* p13 = (const bf16_t*)packed;
    const bf16_t* p2 = p13 + (size_t)E * packed_elems1(n1, d, fp);
    if (timed) (void)hipEventRecord(g_time_events[0], st);
    rc = launch_gemm_bf16(g1, (const bf16_t*)x_in, d, p13, packed_elems1(n1, d, fp), (bf16_t*)ws.h, fp, ws.tiles1,
                          ws.counts, ws.queues, n1 * fp, d, group_for(n1 * fp, g1.bn, A * (int64_t)d * 2), rm1, nullptr, st);
    if (timed) (void)hipEventRecord(g_time_events[1], st);
    if (rc != MOE_OK) return rc;
    if (timed) (void)hipEventRecord(g_time_events[2], st);
    rc = launch_gemm_bf16(g2, (const bf16_t*)ws.h, fp, p2, packed_elems2(d, fp), (bf16_t*)y_perm, d, tiles2, count2,
                          ws.queues + 8, d, fp, group_for(d, g2.bn, A * (int64_t)fp * 2), rm2, ws.partials, st);
    if (rc == MOE_OK && split) {
        hipLaunchKernelGGL(add_partials_kernel, dim3(ws.split_capacity < 64 ? ws.split_capacity : 64, 32), dim3(256),
                           0, st, ws.partials, ws.splits, count2, ws.parts, (bf16_t*)y_perm, d, d, rm2);
        rc = check_launch();
    }
    if (timed) (void)hipEventRecord(g_time_events[3], st);
    return rc;
}
}  // namespace moegps

extern "C" int moe_grouped_ffn(const void* x_perm, int dtype, int64_t A, int d, int ffn, int E,
                               const int32_t* seg_offsets, const int32_t* slot_expert, int nseg, int seg_begin,
                               int seg_end, const void* packed, void* y_perm, void* workspace,
                               size_t workspace_bytes, void* stream) {
    return moegps::grouped_ffn_impl(0, x_perm, A, nullptr, 1, nullptr, nullptr, dtype, A, d, ffn, E, seg_offsets,
                                    slot_expert, nseg, seg_begin, seg_end, packed, y_perm, workspace, workspace_bytes,
                                    stream);
}

extern "C" int moe_grouped_ffn_relu(const void* x_perm, int dtype, int64_t A, int d, int ffn, int E,
                                    const int32_t* seg_offsets, const int32_t* slot_expert, int nseg, int seg_begin,
                                    int seg_end, const void* packed, void* y_perm, void* workspace,
                                    size_t workspace_bytes, void* stream) {
    return moegps::grouped_ffn_impl(1, x_perm, A, nullptr, 1, nullptr, nullptr, dtype, A, d, ffn, E, seg_offsets,
                                    slot_expert, nseg, seg_begin, seg_end, packed, y_perm, workspace, workspace_bytes,
                                    stream);
}

extern "C" int moe_grouped_ffn_fused(const void* x, int dtype, int T, int k, const int32_t* assign_of_row,
                                     const float* topk_w, int d, int ffn, int E, const int32_t* seg_offsets,
                                     const int32_t* slot_expert, int nseg, int seg_begin, int seg_end,
                                     const void* packed, void* y_perm, void* workspace, size_t workspace_bytes,
                                     void* stream) {
    if (T < 0 || k < 1 || d < 1) return MOE_ERR_INVALID_ARG;
    if ((int64_t)T * d >= (1ll << 31)) return MOE_ERR_UNSUPPORTED;  // 32-bit element offsets into x
    if (T > 0 && !assign_of_row) return MOE_ERR_INVALID_ARG;
    return moegps::grouped_ffn_impl(0, x, T, assign_of_row, k, topk_w ? assign_of_row : nullptr, topk_w, dtype,
                                    (int64_t)T * k, d, ffn, E, seg_offsets, slot_expert, nseg, seg_begin, seg_end,
                                    packed, y_perm, workspace, workspace_bytes, stream);
}

extern "C" int moe_grouped_ffn_gather(const void* x, int dtype, int T, int k, const int32_t* assign_of_row, int d,
                                      int ffn, int E, const int32_t* seg_offsets, const int32_t* slot_expert,
                                      int nseg, int seg_begin, int seg_end, const void* packed, void* y_perm,
                                      void* workspace, size_t workspace_bytes, void* stream) {
    return moe_grouped_ffn_fused(x, dtype, T, k, assign_of_row, nullptr, d, ffn, E, seg_offsets, slot_expert, nseg,
                                 seg_begin, seg_end, packed, y_perm, workspace, workspace_bytes, stream);
}

extern "C" int moe_grouped_ffn_time_next_call(void* const* events) {
    using namespace moegps;
    if (!events) {
        g_time_armed = false;
        return MOE_OK;
    }
    for (int i = 0; i < 4; ++i) {
        if (!events[i]) return MOE_ERR_INVALID_ARG;
        g_time_events[i] = (hipEvent_t)events[i];
    }
    g_time_armed = true;
    return MOE_OK;
}
