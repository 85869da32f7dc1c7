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
// v_mfma_f32_16x16x32_bf16 (or 32x32x16) fragments with one ds_read_b128 each.
// A device-built table of M-tiles follows the ragged segments; workgroups claim
// (M-tile, N-tile) pairs from per-XCD counters in an order that keeps the tiles
// running at the same time on a shared set of weight and activation panels.
// The hidden width is padded to a multiple of 64 inside the packed weights.
//
// The ReLU form (Discussion: Switch Transformer's FFN), y = max(x W1_e, 0) W2_e, runs
// the same two products with another epilogue on the first.
//
// fp32 path (small reference-precision configs): a plain LDS-tiled FMA kernel.
#include "common.h"
#include <stdlib.h>
#include <type_traits>
#include <utility>

namespace moegps {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef unsigned short bf16_t;  // storage

struct MTile {
    int row0;    // first row of the tile in x_perm
    int rows;    // valid rows (<= BM)
    int expert;  // expert hosted by the segment's slot
    int kt0;     // k-tiles [kt0, kt1) of the product belong to this entry; kt1 == 0: all of them
    int kt1;
    int part;    // < 0: results go to the output; else fp32 partial sums go to slab `part`
    int pad0, pad1;
};
// The ragged tile of a segment, for the pass that adds up split partial sums
struct TailInfo {
    int row0, rows;
};
constexpr int kPartRows = 256;  // rows of one slab of partial sums (the tallest tile shape)

// ---------------------------------------------------------------------------
// weight packing (one-off, weights are static across inputs)
// ---------------------------------------------------------------------------
// out[n][k] = in[k][n] for one expert per blockIdx.z, zero where k >= K or n >= N (the
// output is K_out x N_out, padded); optional interleave of the output row index: rows
// of W1 go to (n/32)*64 + n%32, rows of W3 32 further.
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
            dst[(size_t)orow * K_out + kk] = tile[tx][r];
        }
    }
}

__global__ void copy_u4_kernel(const uint4* __restrict__ in, uint4* __restrict__ out, size_t n) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) out[i] = in[i];
}

// ---------------------------------------------------------------------------
// M-tile table from the ragged segments
// ---------------------------------------------------------------------------
// Order of the table: first every full-height tile, by (expert, segment), so that
// neighbours mostly read the same expert's weights; then the ragged last tile of
// every segment, tallest first.  Workgroups claim tiles in table order, so the cheap
// tiles come last and fill the gaps at the end of the launch.
// n_tiles[0] = number of tiles, n_tiles[1] = number of full-height tiles; `queues`
// (the claim counters of the launches that walk the table) is cleared here.
// With split_kt > 0 (the product's number of k-tiles) every ragged tile is listed twice,
// once per half of the K range, each half writing fp32 partial sums to its own slab
// (2 * rank + half); tails[rank] and n_tiles[2] = number of ragged tiles describe them for
// the pass that adds the halves up.  Halving the cost of the last tiles claimed evens out
// the end of a launch that has only a few tiles per workgroup.
__global__ __launch_bounds__(1024) void build_mtiles_kernel(const int32_t* __restrict__ seg_offsets,
                                                             const int32_t* __restrict__ slot_expert, int seg_begin,
                                                             int seg_end, int E, int BM, MTile* __restrict__ tiles,
                                                             int capacity, int32_t* __restrict__ n_tiles,
                                                             int32_t* __restrict__ queues, int n_queues,
                                                             int split_kt, TailInfo* __restrict__ tails) {
    __shared__ int nfull[MOE_MAX_SEGMENTS];  // full-height tiles of the segment
    __shared__ int tail[MOE_MAX_SEGMENTS];   // rows of its ragged last tile (0: none)
    __shared__ int ex[MOE_MAX_SEGMENTS];
    __shared__ int total_full, total_tail;
    const int ns = seg_end - seg_begin;
    if (threadIdx.x == 0) total_full = total_tail = 0;
    for (int i = threadIdx.x; i < n_queues; i += blockDim.x) queues[i] = 0;
    __syncthreads();
    for (int i = threadIdx.x; i < ns; i += blockDim.x) {
        const int s = seg_begin + i;
        const int rows = seg_offsets[s + 1] - seg_offsets[s];
        const int e = slot_expert[s];
        const bool live = rows > 0 && e >= 0 && e < E;
        nfull[i] = live ? rows / BM : 0;
        tail[i] = live ? rows % BM : 0;
        ex[i] = e;
        if (nfull[i]) atomicAdd(&total_full, nfull[i]);
        if (tail[i]) atomicAdd(&total_tail, 1);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < ns; i += blockDim.x) {
        const int nf = nfull[i], tl = tail[i];
        if (nf == 0 && tl == 0) continue;
        int base = 0, rank = 0;
        for (int j = 0; j < ns; ++j) {
            const bool before = ex[j] < ex[i] || (ex[j] == ex[i] && j < i);
            if (before) base += nfull[j];
            if (tail[j] > tl || (tail[j] == tl && before)) ++rank;  // tail[j] > 0 whenever tl > 0 reaches here
        }
        const int s = seg_begin + i;
        const int lo = seg_offsets[s];
        MTile mt;
        mt.expert = ex[i];
        mt.kt0 = mt.kt1 = 0;
        mt.part = -1;
        mt.pad0 = mt.pad1 = 0;
        for (int t = 0; t < nf; ++t) {
            if (base + t < capacity) {
                mt.row0 = lo + t * BM;
                mt.rows = BM;
                tiles[base + t] = mt;
            }
        }
        if (tl > 0) {
            mt.row0 = lo + nf * BM;
            mt.rows = tl;
            if (split_kt > 0) {
                if (total_full + 2 * rank + 1 < capacity) {
                    mt.kt0 = 0;
                    mt.kt1 = split_kt / 2;
                    mt.part = 2 * rank;
                    tiles[total_full + 2 * rank] = mt;
                    mt.kt0 = split_kt / 2;
                    mt.kt1 = split_kt;
                    mt.part = 2 * rank + 1;
                    tiles[total_full + 2 * rank + 1] = mt;
                    tails[rank].row0 = mt.row0;
                    tails[rank].rows = tl;
                }
            } else if (total_full + rank < capacity) {
                tiles[total_full + rank] = mt;
            }
        }
    }
    if (threadIdx.x == 0) {
        const int all = total_full + (split_kt > 0 ? 2 : 1) * total_tail;
        n_tiles[0] = all < capacity ? all : capacity;
        n_tiles[1] = total_full < capacity ? total_full : capacity;
        if (split_kt > 0) n_tiles[2] = all <= capacity ? total_tail : 0;
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

// two floats rounded to bf16 (nearest even) and packed, low half first: one conversion instruction
__device__ __forceinline__ unsigned pack_bf16x2(float lo, float hi) {
    typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
    typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
}

// silu(g) = g / (1 + exp(-g)) with the hardware reciprocal (1 ulp) in place of an IEEE division,
// which is ten instructions per value; the result is rounded to bf16 right after.
__device__ __forceinline__ float silu_f(float g) { return g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)); }

// 16-byte piece `slot` of LDS row `row` holds global piece slot ^ swz(row).  The LDS
// has 64 four-byte banks and serves a ds_read_b128 sixteen lanes at a time, so the
// 16 consecutive rows one such group touches must land on 16 distinct 16-byte bank
// groups of a 256-byte span: with 128-byte rows that is (row&1, slot) -> xor with
// (row>>1)&7; with 64-byte rows (row&3, slot) -> xor with (row>>2)&3.
template <int CPR>
__device__ __forceinline__ int swz(int row) {
    if (CPR == 8) return (row >> 1) & 7;
    if (CPR == 4) return (row >> 2) & 3;
    return 0;
}

// EPI selects what happens to the accumulators before they are stored: kEpiNone (plain
// product), kEpiSwiglu (silu(gate) * up on interleaved column pairs, half as many output
// columns), kEpiRelu (max(., 0)).
constexpr int kEpiNone = 0, kEpiSwiglu = 1, kEpiRelu = 2;

// SCHED selects the K loop: kSchedInterleaved (every wavefront interleaves its own LDS reads
// with its MFMAs) or kSchedAlternate (the two wavefronts of a SIMD take turns: one issues
// only MFMAs while the other issues only memory instructions), or kSchedFine (one wavefront
// per SIMD; every memory instruction sits between two MFMAs of the same wavefront).
constexpr int kSchedInterleaved = 0, kSchedAlternate = 1, kSchedFine = 2;

// MI selects the matrix instruction: 32 (v_mfma_f32_32x32x16_bf16) or 16 (v_mfma_f32_16x16x32_bf16,
// interleaved schedule only).  Both run at the same peak rate; the 16x16x32 form goes twice as
// deep in K per accumulator read and write, and on operands with random bits -- where the chip
// holds its clock below the maximum -- sustains about a tenth more.
template <int BM, int BN, int BK, int WGM, int WGN, int NSTAGE, int EPI, int SCHED = kSchedInterleaved, int MI = 32>
__global__ __launch_bounds__(WGM* WGN * 64) void grouped_gemm_bf16_kernel(
    const bf16_t* __restrict__ A, int lda,           // activations [rows, K]
    const bf16_t* __restrict__ Bp, size_t b_stride,  // packed weights [E][N][K]
    bf16_t* __restrict__ C, int ldc,                 // output [rows, SWIGLU ? N/2 : N]
    const MTile* __restrict__ mtiles, const int32_t* __restrict__ n_mtiles_ptr, int32_t* __restrict__ queues,
    int N, int K, int group_n,
    const int32_t* __restrict__ gather_rows, int gather_div,  // optional: A row r is A[gather_rows[r] / gather_div]
    float* __restrict__ partials) {  // [slab][kPartRows][N] fp32 sums of tiles that cover part of K (plain product only)
    constexpr bool SWIGLU = EPI == kEpiSwiglu;
    constexpr int NW = WGM * WGN;
    constexpr int WTM = BM / WGM, WTN = BN / WGN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int CPR = BK / 8;                 // 16-byte pieces per tile row
    constexpr int IA = BM * CPR / 64;           // wave-wide load instructions per A tile
    constexpr int IB = BN * CPR / 64;
    constexpr int IAW = IA / NW, IBW = IB / NW;  // per wavefront
    constexpr int LPT = IAW + IBW;              // loads per thread per k-tile
    constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE_BYTES = A_BYTES + B_BYTES;
    static_assert(IA % NW == 0 && IB % NW == 0, "tile loads must divide over the wavefronts");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile is a grid of 32x32 MFMA tiles");
    static_assert(!SWIGLU || (WTN % 64 == 0), "gate/up pairs must sit in one wavefront");
    static_assert(LPT * NSTAGE < 64, "vmcnt range");
    static_assert((BK / 16) % 2 == 0, "fragment buffers alternate with an even number of steps per k-tile");
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
    const int l32 = lane & 31, half = lane >> 5;

    const int n_mtiles = n_mtiles_ptr[0];
    const int n_full = n_mtiles_ptr[1];  // the table lists these full-height tiles first
    const int n_ntiles = (N + BN - 1) / BN;

    // Tile order.  The (M-tile, N-tile) space is walked in two passes, the full-height
    // M-tiles first and the ragged ones (tallest first) after them.  Inside a pass tiles
    // are numbered in groups of group_n neighbouring N-tiles; inside a group the N-tile
    // index runs fastest, then the M-tile (full M-tiles are sorted by expert), so a run of
    // 32 consecutive tiles is a patch of about 32/group_n x group_n tiles that share their
    // activation and weight panels.  Workgroups are dealt to the 8 XCDs round-robin
    // (workgroup b runs on XCD b % 8) and every XCD has its own L2, so run c of the
    // numbering belongs to XCD c % 8: its workgroups claim the tiles of its runs one by
    // one from a counter (tiles differ in cost, a fixed deal would leave workgroups idle
    // at the end) and so work side by side on one patch, sharing its panels through that
    // L2; the 8 XCDs are on 8 consecutive runs (further along M under the same weight
    // panels, shared through the memory-side cache).  A workgroup whose own XCD has no
    // tile left claims from the other XCDs' counters.
    const int xcd = blockIdx.x & 7;
    const int run = (int)(gridDim.x >> 3);
    const int total = n_mtiles * n_ntiles;
    const int total_full = n_full * n_ntiles;
    __shared__ volatile int next_tile;
    int q_done = 0;  // thread 0: counters xcd .. xcd + q_done - 1 (mod 8) have run out
    // tile number for claim i of XCD q's counter, -1 if that counter has run out
    auto tile_of_claim = [&](int q, int i) {
        const int t = (q + 8 * (i / run)) * run + i % run;
        return t < total ? t : -1;  // claims only grow: past the end once, past the end for good
    };
    // thread 0 only: turns a claim made ahead of time (or none: q < 0) into a tile, making
    // further claims as needed; -1 when every counter has run out
    auto settle_claim = [&](int q, int i) {
        for (;;) {
            if (q >= 0) {
                const int t = tile_of_claim(q, i);
                if (t >= 0) return t;
                if (q == ((xcd + q_done) & 7)) ++q_done;
            }
            if (q_done >= 8) return -1;
            q = (xcd + q_done) & 7;
            i = atomicAdd(&queues[q], 1);
        }
    };
    if (tid == 0) next_tile = settle_claim(-1, 0);
    for (;;) {
        lds_wait<0>();                 // thread 0's store of next_tile
        __builtin_amdgcn_s_barrier();  // also: every wavefront is done reading the previous tile's stages
        const int t_all = __builtin_amdgcn_readfirstlane(next_tile);
        if (t_all < 0) break;
        // the claim for the tile after this one is made now and looked at after the K loop
        int ahead_q = -1, ahead_i = 0;
        if (tid == 0 && q_done < 8) {
            ahead_q = (xcd + q_done) & 7;
            ahead_i = atomicAdd(&queues[ahead_q], 1);
        }
        const bool ragged_pass = t_all >= total_full;
        const int t = ragged_pass ? t_all - total_full : t_all;
        const int m_base = ragged_pass ? n_full : 0;
        const int m_count = ragged_pass ? n_mtiles - n_full : n_full;
        const int per_group = m_count * group_n;
        const int grp = t / per_group;
        const int rem = t - grp * per_group;
        const int gw = (n_ntiles - grp * group_n) < group_n ? (n_ntiles - grp * group_n) : group_n;
        const int mt_i = m_base + rem / gw;
        const int nt_i = grp * group_n + rem % gw;
        const MTile mt = mtiles[mt_i];
        const int n0 = nt_i * BN;
        // with a gather list the activation rows are fetched straight from their source
        // (row gather_rows[r] / gather_div of A), otherwise from row r
        // k-tiles of this entry: all of K, or the part of it a split tile covers
        const int KT = mt.kt1 > 0 ? mt.kt1 - mt.kt0 : K / BK;
        const bf16_t* Ab = (gather_rows ? A : A + (size_t)mt.row0 * lda) + mt.kt0 * BK;
        const bf16_t* Bb = Bp + (size_t)mt.expert * b_stride + (size_t)n0 * K + mt.kt0 * BK;
        const int n_valid = (N - n0) < BN ? (N - n0) : BN;

        // per-lane element offsets of the pieces this lane fetches (rows beyond the
        // segment / matrix edge are clamped to the last valid row; their products
        // are computed and dropped in the epilogue)
        int offA[IAW], offB[IBW];
#pragma unroll
        for (int i = 0; i < IAW; ++i) {
            const int p = (wave + i * NW) * 64 + lane;
            const int row = p / CPR, slot = p % CPR;
            int r = row < mt.rows ? row : mt.rows - 1;
            if (gather_rows) r = gather_rows[mt.row0 + r] / gather_div;
            offA[i] = r * lda + ((slot ^ swz<CPR>(row)) * 8);
        }
#pragma unroll
        for (int i = 0; i < IBW; ++i) {
            const int p = (wave + i * NW) * 64 + lane;
            const int row = p / CPR, slot = p % CPR;
            const int r = row < n_valid ? row : n_valid - 1;
            offB[i] = r * K + ((slot ^ swz<CPR>(row)) * 8);
        }

        // the same offsets in bytes, unsigned: (uniform base) + (32-bit lane offset) is an addressing
        // mode of the load instruction, so the loads spend no vector ALU work on addresses
        unsigned offA_b[IAW], offB_b[IBW];
#pragma unroll
        for (int i = 0; i < IAW; ++i) offA_b[i] = (unsigned)offA[i] * 2u;
#pragma unroll
        for (int i = 0; i < IBW; ++i) offB_b[i] = (unsigned)offB[i] * 2u;

        auto issue_loads = [&](int kt, int stage) {
            unsigned char* sA = smem + stage * STAGE_BYTES;
            unsigned char* sB = sA + A_BYTES;
            const unsigned char* a = (const unsigned char*)Ab + (size_t)(kt * (BK * 2));
            const unsigned char* b = (const unsigned char*)Bb + (size_t)(kt * (BK * 2));
#pragma unroll
            for (int i = 0; i < IAW; ++i)
                if (!SKIP_TAIL_LOADS || (wave + i * NW) * ROWS_PER_LOAD < mt.rows)
                    __builtin_amdgcn_global_load_lds(
                        (const __attribute__((address_space(1))) void*)(a + (size_t)offA_b[i]),
                        (__attribute__((address_space(3))) void*)(sA + (wave + i * NW) * 1024), 16, 0, 0);
#pragma unroll
            for (int i = 0; i < IBW; ++i)
                __builtin_amdgcn_global_load_lds(
                    (const __attribute__((address_space(1))) void*)(b + (size_t)offB_b[i]),
                    (__attribute__((address_space(3))) void*)(sB + (wave + i * NW) * 1024), 16, 0, 0);
        };

        // the first k-tiles are requested before the accumulators are cleared: the clearing
        // then runs while the loads are under way
#pragma unroll
        for (int s = 0; s < NSTAGE; ++s)
            if (s < KT) issue_loads(s, s);
        __builtin_amdgcn_sched_barrier(0);

        // Accumulators hold the transposed product: the weight fragment is the MFMA's
        // row operand and the activation fragment its column operand, so element r of
        // lane (l32, half) in tile (i, j) is output row i*32 + l32 and output column
        // j*32 + (r/4)*8 + half*4 + r%4: four consecutive columns per lane.
        f32x16 acc[MI == 32 ? TM : 1][MI == 32 ? TN : 1];
        if constexpr (MI == 32) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
        }
        // 16x16x32 form: element r of lane (l16, g16) in tile (i, j) is output row i*16 + l16 and
        // output column j*16 + g16*4 + r (weights are the row operand, as above)
        constexpr int TM16 = WTM / 16, TN16 = WTN / 16;
        f32x4 acc16[MI == 16 ? TM16 : 1][MI == 16 ? TN16 : 1];
        if constexpr (MI == 16) {
#pragma unroll
            for (int i = 0; i < TM16; ++i)
#pragma unroll
                for (int j = 0; j < TN16; ++j)
#pragma unroll
                    for (int r = 0; r < 4; ++r) acc16[i][j][r] = 0.f;
        }
        const int l16 = lane & 15, g16 = lane >> 4;

        // fragment read addresses (bytes inside a stage): row = base + l32, piece kk*2+half
        const int a_row = wm * WTM + l32;
        const int b_row = wn * WTN + l32;
        // 32-row sub-tiles of this wavefront that hold at least one valid row; the others
        // (past the end of a ragged M-tile) are neither read nor multiplied
        const int rows_w = mt.rows - wm * WTM;
        const int tm_valid = rows_w <= 0 ? 0 : (rows_w >= WTM ? TM : (rows_w + 31) / 32);
        const int sw = swz<CPR>(l32);  // rows differ by multiples of 32 -> same swizzle
        constexpr int KK = BK / 16;

        // The K loop exists twice: FULL (every 32-row sub-tile of this wavefront is valid,
        // no conditions inside the loop) and ragged (sub-tiles i >= tm_valid are skipped).
        // Both run the same sequence of barriers, so wavefronts of one workgroup may take
        // different versions.
        const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)smem;
        auto k_loop = [&](auto full_tag) {
            constexpr bool FULL = decltype(full_tag)::value;
            constexpr int ROW_BYTES = CPR * 16;
            bf16x8 af[2][TM], bfr[2][TN];
            auto load_frags = [&](int kt, int kk, int buf) {
                const unsigned stage = lds_base + (kt % NSTAGE) * STAGE_BYTES;
                const unsigned piece = (unsigned)(((kk * 2 + half) ^ sw) * 16);
                static_for<TM>([&](auto I) {
                    constexpr int i = decltype(I)::value;
                    if (FULL || i < tm_valid)
                        lds_read_b128<i * 32 * ROW_BYTES>(af[buf][i], stage + a_row * ROW_BYTES + piece);
                });
                static_for<TN>([&](auto J) {
                    constexpr int j = decltype(J)::value;
                    lds_read_b128<j * 32 * ROW_BYTES>(bfr[buf][j], stage + A_BYTES + b_row * ROW_BYTES + piece);
                });
            };
            auto frags_landed = [&](int buf) {
#pragma unroll
                for (int i = 0; i < TM; ++i) lds_landed(af[buf][i]);
#pragma unroll
                for (int j = 0; j < TN; ++j) lds_landed(bfr[buf][j]);
            };
            // The loop is software-pipelined across the k-tile barrier.  Fragments are
            // double-buffered in registers; the LDS reads of step kk+1 are issued ahead of the
            // MFMAs of step kk, which wait only for their own fragments.  The barrier that
            // hands over k-tile kt+1 sits before the LAST step of k-tile kt: after it the
            // wavefront reads the first fragments of k-tile kt+1 and refills the stage that
            // k-tile kt occupied (all of its fragments are in registers by then), and the
            // MFMAs of the last step cover both.
            if ((!SKIP_TAIL_LOADS || mt.rows == BM) && KT >= NSTAGE)
                wait_vmcnt<LPT*(NSTAGE - 1)>();  // k-tile 0 landed, the others may be in flight
            else
                wait_vmcnt<0>();
            __builtin_amdgcn_s_barrier();
            load_frags(0, 0, 0);
            for (int kt = 0; kt < KT; ++kt) {
#pragma unroll
                for (int kk = 0; kk < KK; ++kk) {
                    if (kk + 1 < KK) {
                        load_frags(kt, kk + 1, (kk + 1) & 1);
                        if (FULL)
                            lds_wait<TM + TN>();
                        else
                            lds_wait<0>();
                    } else {
                        lds_wait<0>();  // every fragment of k-tile kt is in registers
                        if (kt + 1 < KT) {
                            // this wavefront's pieces of k-tile kt+1 have landed; the barrier
                            // extends that to every wavefront's pieces and says all of them are
                            // done with k-tile kt's stage
                            if (KT - 2 - kt >= NSTAGE - 2)
                                wait_vmcnt<LPT*(NSTAGE - 2)>();
                            else
                                wait_vmcnt<0>();
                            __builtin_amdgcn_s_barrier();
                            load_frags(kt + 1, 0, 0);
                            if (kt + NSTAGE < KT) issue_loads(kt + NSTAGE, kt % NSTAGE);
                        }
                    }
                    frags_landed(kk & 1);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int i = 0; i < TM; ++i)
                        if (FULL || i < tm_valid) {
#pragma unroll
                            for (int j = 0; j < TN; ++j)
                                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[kk & 1][j], af[kk & 1][i],
                                                                                    acc[i][j], 0, 0, 0);
                        }
                    __builtin_amdgcn_sched_barrier(0);
                }
                // The first fragments of the next k-tile were requested before the last
                // step's MFMAs; they have landed by now.  Settling them here means no
                // register that the LDS is still writing is live across the loop edge,
                // where the compiler may place copies.
                lds_wait<0>();
                frags_landed(0);
            }
        };
        // Alternating schedule.  The wavefronts form two groups (wm = 0, 1; wavefronts w and
        // w + 4 share a SIMD) that run the same sequence of half-k-tile steps
        //     memory(s): LDS -> register reads of the step's fragments (and, on the first half
        //                of a k-tile, the global -> LDS refill of the stage freed one k-tile ago)
        //     barrier
        //     compute(s): the step's MFMAs, nothing else
        //     barrier
        // one barrier apart, so that while one group computes the other is in its memory
        // phase.  Loads of k-tile j + 1 go out in memory(2j) and are waited for in the phase
        // before any wavefront reads them (the end of step 2j + 1).
        auto k_loop_alt = [&](auto full_tag) {
            constexpr bool FULL = decltype(full_tag)::value;
            constexpr int ROW_BYTES = CPR * 16;
            static_assert(SCHED != kSchedAlternate || (NSTAGE == 2 && BK == 64 && WGM == 2),
                          "the alternating schedule is written for two stages of 64 and two row groups");
            bf16x8 af[2][TM], bfr[2][TN];
            auto load_frags = [&](int kt, int kk, int buf) {
                const unsigned stage = lds_base + (kt & 1) * STAGE_BYTES;
                const unsigned piece = (unsigned)(((kk * 2 + half) ^ sw) * 16);
                static_for<TM>([&](auto I) {
                    constexpr int i = decltype(I)::value;
                    if (FULL || i < tm_valid)
                        lds_read_b128<i * 32 * ROW_BYTES>(af[buf][i], stage + a_row * ROW_BYTES + piece);
                });
                static_for<TN>([&](auto J) {
                    constexpr int j = decltype(J)::value;
                    lds_read_b128<j * 32 * ROW_BYTES>(bfr[buf][j], stage + A_BYTES + b_row * ROW_BYTES + piece);
                });
            };
            auto step = [&](int j, auto half_tag) {
                constexpr int h = decltype(half_tag)::value;
                // memory phase
                if (h == 0 && j >= 1 && j + 1 < KT) issue_loads(j + 1, (j + 1) & 1);
                load_frags(j, 2 * h, 0);
                load_frags(j, 2 * h + 1, 1);
                if (h == 1 && wm == 1) wait_vmcnt<0>();  // this wavefront's pieces of k-tile j + 1
                lds_wait<0>();
#pragma unroll
                for (int b = 0; b < 2; ++b) {
#pragma unroll
                    for (int i = 0; i < TM; ++i) lds_landed(af[b][i]);
#pragma unroll
                    for (int jj = 0; jj < TN; ++jj) lds_landed(bfr[b][jj]);
                }
                __builtin_amdgcn_sched_barrier(0);
                __builtin_amdgcn_s_barrier();
                // compute phase
                __builtin_amdgcn_s_setprio(1);
#pragma unroll
                for (int b = 0; b < 2; ++b)
#pragma unroll
                    for (int i = 0; i < TM; ++i)
                        if (FULL || i < tm_valid) {
#pragma unroll
                            for (int jj = 0; jj < TN; ++jj)
                                acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[b][jj], af[b][i], acc[i][jj], 0,
                                                                                     0, 0);
                        }
                __builtin_amdgcn_s_setprio(0);
                if (h == 1 && wm == 0) wait_vmcnt<0>();
                __builtin_amdgcn_sched_barrier(0);
                __builtin_amdgcn_s_barrier();
            };
            if ((!SKIP_TAIL_LOADS || mt.rows == BM) && KT >= 2)
                wait_vmcnt<LPT>();  // k-tile 0 landed, k-tile 1 may be in flight
            else
                wait_vmcnt<0>();
            __builtin_amdgcn_s_barrier();
            if (wm == 1) __builtin_amdgcn_s_barrier();  // the second group runs one phase behind
            for (int j = 0; j < KT; ++j) {
                step(j, std::integral_constant<int, 0>{});
                step(j, std::integral_constant<int, 1>{});
            }
            if (wm == 0) __builtin_amdgcn_s_barrier();  // same number of barriers for both groups
        };
        // Fine schedule, for one wavefront per SIMD (4 wavefronts, 128x128 each).  With nobody
        // else on the SIMD to fill a gap, the matrix pipe only stays busy if the wavefront never
        // spends more than one MFMA's time (32 cycles) on anything else.  So every LDS read and
        // every global->LDS load is placed between two MFMAs: step (kt, kk) runs its 16 MFMAs
        // and hangs the 8 fragment reads of the next step behind the first 8 of them; the last
        // step of a k-tile starts with the hand-over (own loads of k-tile kt+1 landed, barrier),
        // reads the first fragments of k-tile kt+1 and hangs the 16 loads of k-tile kt+2, into
        // the stage k-tile kt just left, behind its 16 MFMAs.
        auto k_loop_fine = [&](auto full_tag) {
            constexpr bool FULL = decltype(full_tag)::value;
            constexpr int ROW_BYTES = CPR * 16;
            static_assert(SCHED != kSchedFine || (NSTAGE == 2 && BK == 64 && TM * TN == 2 * IAW && IAW == IBW),
                          "the fine schedule hangs one load behind every second MFMA of two steps");
            bf16x8 af[2][TM], bfr[2][TN];
            // read r of the TM + TN fragment reads of step (kt, kk), into buffer buf
            auto read_frag = [&](auto R, int kt, int kk, int buf) {
                constexpr int r = decltype(R)::value;
                const unsigned stage = lds_base + (kt & 1) * STAGE_BYTES;
                const unsigned piece = (unsigned)(((kk * 2 + half) ^ sw) * 16);
                if constexpr (r < TM) {
                    if (FULL || r < tm_valid)
                        lds_read_b128<r * 32 * ROW_BYTES>(af[buf][r], stage + a_row * ROW_BYTES + piece);
                } else {
                    lds_read_b128<(r - TM) * 32 * ROW_BYTES>(bfr[buf][r - TM],
                                                              stage + A_BYTES + b_row * ROW_BYTES + piece);
                }
            };
            auto frags_landed = [&](int buf) {
#pragma unroll
                for (int i = 0; i < TM; ++i) lds_landed(af[buf][i]);
#pragma unroll
                for (int j = 0; j < TN; ++j) lds_landed(bfr[buf][j]);
            };
            // load l of the IAW + IBW loads of this wavefront for k-tile kt (l < IAW: activations)
            auto issue_one_load = [&](auto L, int kt, int stage) {
                constexpr int l = decltype(L)::value;
                unsigned char* sA = smem + stage * STAGE_BYTES;
                if constexpr (l < IAW) {
                    const unsigned char* base = (const unsigned char*)Ab + (size_t)(kt * (BK * 2));
                    if (!SKIP_TAIL_LOADS || (wave + l * NW) * ROWS_PER_LOAD < mt.rows)
                        __builtin_amdgcn_global_load_lds(
                            (const __attribute__((address_space(1))) void*)(base + (size_t)offA_b[l]),
                            (__attribute__((address_space(3))) void*)(sA + (wave + l * NW) * 1024), 16, 0, 0);
                } else {
                    const unsigned char* base = (const unsigned char*)Bb + (size_t)(kt * (BK * 2));
                    __builtin_amdgcn_global_load_lds(
                        (const __attribute__((address_space(1))) void*)(base + (size_t)offB_b[l - IAW]),
                        (__attribute__((address_space(3))) void*)(sA + A_BYTES + (wave + (l - IAW) * NW) * 1024), 16,
                        0, 0);
                }
            };
            // One step.  NEXT: fragments of the following step are read (false only for the very
            // last step of the tile).  LOADS, on the last step of k-tile kt: the weight loads of
            // k-tile kt + 2 go out here; on the first step: the activation loads of k-tile kt + 1
            // (both into the stage that the hand-over before them has freed; the weights, which
            // come from further away, get the longer lead).  One load behind every second MFMA.
            auto step = [&](int kt, auto kk_tag, auto next_tag, auto loads_tag) {
                constexpr int kk = decltype(kk_tag)::value;
                constexpr bool NEXT = decltype(next_tag)::value, LOADS = decltype(loads_tag)::value;
                constexpr bool LAST = kk == KK - 1;
                constexpr int cur = kk & 1, nxt = cur ^ 1;
                if constexpr (LAST && NEXT) {
                    wait_vmcnt<0>();               // this wavefront's pieces of k-tile kt + 1
                    __builtin_amdgcn_s_barrier();  // everybody's, and everybody has read all of k-tile kt
                }
                static_for<TM * TN>([&](auto M) {
                    constexpr int m = decltype(M)::value;
                    constexpr int i = m / TN, j = m % TN;
                    if (FULL || i < tm_valid)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[cur][j], af[cur][i], acc[i][j], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                    if constexpr (NEXT && m < TM + TN) read_frag(M, LAST ? kt + 1 : kt, LAST ? 0 : kk + 1, nxt);
                    if constexpr (LOADS && m % 2 == 1) {
                        if constexpr (LAST)
                            issue_one_load(std::integral_constant<int, IAW + m / 2>{}, kt + 2, kt & 1);
                        else
                            issue_one_load(std::integral_constant<int, m / 2>{}, kt + 1, (kt + 1) & 1);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                });
                if constexpr (NEXT) {
                    lds_wait<0>();
                    frags_landed(nxt);
                }
            };
            // a_loads: k-tile kt + 1's activations are still to be loaded (not so for kt = 0: the
            // prologue has loaded k-tiles 0 and 1 whole); b_loads: k-tile kt + 2 exists
            auto k_tile = [&](int kt, auto a_loads, auto b_loads) {
                step(kt, std::integral_constant<int, 0>{}, std::true_type{}, a_loads);
                static_for<KK - 2>([&](auto S) {
                    step(kt, std::integral_constant<int, decltype(S)::value + 1>{}, std::true_type{}, std::false_type{});
                });
                step(kt, std::integral_constant<int, KK - 1>{}, std::true_type{}, b_loads);
            };
            if ((!SKIP_TAIL_LOADS || mt.rows == BM) && KT >= NSTAGE)
                wait_vmcnt<LPT*(NSTAGE - 1)>();  // k-tile 0 landed, k-tile 1 may be in flight
            else
                wait_vmcnt<0>();
            __builtin_amdgcn_s_barrier();
            static_for<TM + TN>([&](auto R) { read_frag(R, 0, 0, 0); });
            lds_wait<0>();
            frags_landed(0);
            int kt = 0;
            if (KT > 2) {
                k_tile(0, std::false_type{}, std::true_type{});
                for (kt = 1; kt + 2 < KT; ++kt) k_tile(kt, std::true_type{}, std::true_type{});
                k_tile(kt, std::true_type{}, std::false_type{});  // kt = KT - 2
                ++kt;
            } else if (KT == 2) {
                k_tile(0, std::false_type{}, std::false_type{});
                kt = 1;
            }
            static_for<KK - 1>([&](auto S) { step(kt, S, std::true_type{}, std::false_type{}); });
            step(kt, std::integral_constant<int, KK - 1>{}, std::false_type{}, std::false_type{});
        };
        // K loop of the 16x16x32 form.  A step is 32 deep: TM16 activation fragments (16 rows
        // each) and TN16 weight fragments, TM16 * TN16 MFMAs, taken row of tiles by row of tiles.
        // The weight fragments are double-buffered; an activation fragment is free once its row
        // of tiles has been issued, so its register is refilled for the next step right behind
        // that row.  LDS reads complete in issue order (weights of a step first, then its
        // activation fragments 0, 1, ...), which fixes how many may still be in flight before
        // each row.  The hand-over to the next k-tile (own loads landed, barrier, refill of the
        // stage just left) opens a k-tile's last step, when every fragment of that k-tile is in
        // a register; the loads of the refill go out one or two per row of tiles.
        auto k_loop16 = [&](auto full_tag) {
            constexpr bool FULL = decltype(full_tag)::value;
            constexpr int ROW_BYTES = CPR * 16;
            constexpr int KS = BK / 32;
            constexpr int HAND = 0;  // rows of tiles issued before the hand-over (0 and 1 measured alike, 2 to 4 a little slower)
            static_assert(MI != 16 || (CPR == 8 && KS == 2 && SCHED == kSchedInterleaved && TM16 + TN16 <= 12),
                          "the 16x16x32 loop is written for 64-deep k-tiles and the interleaved schedule");
            const int rows_w16 = mt.rows - wm * WTM;
            const int tmv16 = rows_w16 <= 0 ? 0 : (rows_w16 >= WTM ? TM16 : (rows_w16 + 15) / 16);
            const int sw16 = swz<CPR>(l16);  // rows differ by multiples of 16 -> same swizzle
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
            // load l of this wavefront's LPT loads of k-tile kt (activations first), one instruction
            auto issue_load_n = [&](auto L, int kt, int stage) {
                constexpr int l = decltype(L)::value;
                unsigned char* sA = smem + stage * STAGE_BYTES;
                if constexpr (l < IAW) {
                    const unsigned char* base = (const unsigned char*)Ab + (size_t)(kt * (BK * 2));
                    if (!SKIP_TAIL_LOADS || (wave + l * NW) * ROWS_PER_LOAD < mt.rows)
                        __builtin_amdgcn_global_load_lds(
                            (const __attribute__((address_space(1))) void*)(base + (size_t)offA_b[l]),
                            (__attribute__((address_space(3))) void*)(sA + (wave + l * NW) * 1024), 16, 0, 0);
                } else {
                    const unsigned char* base = (const unsigned char*)Bb + (size_t)(kt * (BK * 2));
                    __builtin_amdgcn_global_load_lds(
                        (const __attribute__((address_space(1))) void*)(base + (size_t)offB_b[l - IAW]),
                        (__attribute__((address_space(3))) void*)(sA + A_BYTES + (wave + (l - IAW) * NW) * 1024), 16,
                        0, 0);
                }
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
                    if constexpr (HANDOVER && i == HAND) {
                        // every fragment of k-tile kt is in a register (waited for on entry); this
                        // wavefront's pieces of k-tile kt + 1 have landed; the barrier extends both
                        // to every wavefront, so the stage of k-tile kt can be refilled
                        if (KT - 2 - kt >= NSTAGE - 2)
                            wait_vmcnt<LPT*(NSTAGE - 2)>();
                        else
                            wait_vmcnt<0>();
                        __builtin_amdgcn_s_barrier();
                        read_b_all(nxt, np);
                        static_for<HAND>([&](auto P) { read_a(P, np); });
                    }
                    if constexpr (i > 0 && NEXT && !HANDOVER)
                        lds_wait<TM16 - 1 + TN16>();  // activation fragment i has landed
                    row_mfmas(I, cur);
                    if constexpr (NEXT && (!HANDOVER || i >= HAND)) read_a(I, np);
                    if constexpr (HANDOVER && i >= HAND) {
                        // the refill of the stage k-tile kt has left: this wavefront's loads of
                        // k-tile kt + NSTAGE, dealt over the rows of tiles behind the hand-over so
                        // that a load waiting for the CU's one address unit holds up a few MFMAs of
                        // this wavefront, not the SIMD (its other wavefront keeps issuing)
                        constexpr int R = TM16 - HAND, q = i - HAND;
                        constexpr int l0 = q * LPT / R, l1 = (q + 1) * LPT / R;
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
        if constexpr (MI == 16) {
            if (mt.rows - wm * WTM >= WTM)
                k_loop16(std::true_type{});
            else
                k_loop16(std::false_type{});
        } else if constexpr (SCHED == kSchedFine) {
            if (tm_valid == TM)
                k_loop_fine(std::true_type{});
            else
                k_loop_fine(std::false_type{});
        } else if constexpr (SCHED == kSchedAlternate) {
            if (tm_valid == TM)
                k_loop_alt(std::true_type{});
            else
                k_loop_alt(std::false_type{});
        } else {
            if (tm_valid == TM)
                k_loop(std::true_type{});
            else
                k_loop(std::false_type{});
        }
        // every wavefront has read next_tile (the K loop holds a barrier)
        if (tid == 0) next_tile = settle_claim(ahead_q, ahead_i);

        // epilogue: 4 consecutive columns per lane and accumulator group -> 8-byte stores
        const int col_w = (SWIGLU ? (n0 + wn * WTN) / 2 : (n0 + wn * WTN)) + half * 4;
        const int n_out = SWIGLU ? N / 2 : N;
        constexpr int TNO = SWIGLU ? TN / 2 : TN;  // 32-column tiles of output per wavefront
        if constexpr (MI == 16) {
            // 4 consecutive columns per lane and tile -> 8-byte stores (16 bytes of fp32 partial sums)
            const int n_out16 = SWIGLU ? N / 2 : N;
            const int col0 = (SWIGLU ? (n0 + wn * WTN) / 2 : (n0 + wn * WTN));
            constexpr int TNO16 = SWIGLU ? TN16 / 2 : TN16;  // 16-column tiles of output per wavefront
            static_assert(!SWIGLU || TN16 % 4 == 0, "gate and up tiles pair up inside 64 packed columns");
            float* slab = nullptr;
            if constexpr (EPI == kEpiNone)
                if (mt.part >= 0) slab = partials + (size_t)mt.part * kPartRows * N;
#pragma unroll
            for (int i = 0; i < TM16; ++i) {
                const int row = wm * WTM + i * 16 + l16;
                if (row < mt.rows) {
                    bf16_t* crow = C + (size_t)(mt.row0 + row) * ldc + col0 + g16 * 4;
#pragma unroll
                    for (int jo = 0; jo < TNO16; ++jo) {
                        // output tile jo: packed tiles (jo/2)*4 + jo%2 (gate) and + 2 (up) with SwiGLU
                        const int jg = SWIGLU ? (jo / 2) * 4 + (jo % 2) : jo;
                        if (col0 + jo * 16 < n_out16) {
                            float v[4];
#pragma unroll
                            for (int c = 0; c < 4; ++c) {
                                if (SWIGLU)
                                    v[c] = silu_f(acc16[i][jg][c]) * acc16[i][jg + 2][c];
                                else if (EPI == kEpiRelu)
                                    v[c] = fmaxf(acc16[i][jg][c], 0.f);
                                else
                                    v[c] = acc16[i][jg][c];
                            }
                            if (slab) {
                                float4 o;
                                o.x = v[0];
                                o.y = v[1];
                                o.z = v[2];
                                o.w = v[3];
                                *(float4*)(slab + (size_t)row * N + col0 + jo * 16 + g16 * 4) = o;
                            } else {
                                uint2 o;
                                o.x = pack_bf16x2(v[0], v[1]);
                                o.y = pack_bf16x2(v[2], v[3]);
                                *(uint2*)(crow + jo * 16) = o;
                            }
                        }
                    }
                }
            }
            continue;
        }
        if constexpr (EPI == kEpiNone) {
            if (mt.part >= 0) {
                // part of K only: the fp32 sums go to this entry's slab, 16 bytes per lane and group
                float* slab = partials + (size_t)mt.part * kPartRows * N;
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    const int row = wm * WTM + i * 32 + l32;
                    if (row < mt.rows) {
                        float* prow = slab + (size_t)row * N + col_w;
#pragma unroll
                        for (int jo = 0; jo < TN; ++jo) {
                            if (col_w - half * 4 + jo * 32 < N) {
#pragma unroll
                                for (int g = 0; g < 4; ++g) {
                                    float4 o;
                                    o.x = acc[i][jo][g * 4 + 0];
                                    o.y = acc[i][jo][g * 4 + 1];
                                    o.z = acc[i][jo][g * 4 + 2];
                                    o.w = acc[i][jo][g * 4 + 3];
                                    *(float4*)(prow + jo * 32 + g * 8) = o;
                                }
                            }
                        }
                    }
                }
                continue;
            }
        }
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row = wm * WTM + i * 32 + l32;
            if (row < mt.rows) {
                bf16_t* crow = C + (size_t)(mt.row0 + row) * ldc + col_w;
#pragma unroll
                for (int jo = 0; jo < TNO; ++jo) {
                    if (col_w - half * 4 + jo * 32 < n_out) {  // whole 32-column tile in range (n_out % 32 == 0)
#pragma unroll
                        for (int g = 0; g < 4; ++g) {
                            float v[4];
#pragma unroll
                            for (int c = 0; c < 4; ++c) {
                                if (SWIGLU)
                                    v[c] = silu_f(acc[i][2 * jo][g * 4 + c]) * acc[i][2 * jo + 1][g * 4 + c];
                                else if (EPI == kEpiRelu)
                                    v[c] = fmaxf(acc[i][jo][g * 4 + c], 0.f);
                                else
                                    v[c] = acc[i][jo][g * 4 + c];
                            }
                            uint2 o;
                            o.x = pack_bf16x2(v[0], v[1]);
                            o.y = pack_bf16x2(v[2], v[3]);
                            *(uint2*)(crow + jo * 32 + g * 8) = o;
                        }
                    }
                }
            }
        }
    }
}

// Adds up the two fp32 slabs of every ragged tile whose K range was split and writes the
// rows as bf16: y[row0 + r] = P[2t][r] + P[2t + 1][r].  blockIdx.x = ragged tile,
// blockIdx.y strides over its rows; n_tiles[2] = number of such tiles.
__global__ __launch_bounds__(256) void add_partials_kernel(const float* __restrict__ partials,
                                                            const TailInfo* __restrict__ tails,
                                                            const int32_t* __restrict__ n_tiles,
                                                            bf16_t* __restrict__ C, int ldc, int N) {
    const int t = blockIdx.x;
    if (t >= n_tiles[2]) return;
    const TailInfo ti = tails[t];
    const float* p0 = partials + (size_t)(2 * t) * kPartRows * N;
    const float* p1 = p0 + (size_t)kPartRows * N;
    const int n4 = N / 4;
    for (int r = blockIdx.y; r < ti.rows; r += gridDim.y) {
        const float4* a = (const float4*)(p0 + (size_t)r * N);
        const float4* b = (const float4*)(p1 + (size_t)r * N);
        uint2* out = (uint2*)(C + (size_t)(ti.row0 + r) * ldc);
        for (int c = threadIdx.x; c < n4; c += blockDim.x) {
            const float4 u = a[c], v = b[c];
            uint2 o;
            o.x = pack_bf16x2(u.x + v.x, u.y + v.y);
            o.y = pack_bf16x2(u.z + v.z, u.w + v.w);
            out[c] = o;
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
                                                                const int32_t* __restrict__ n_mtiles_ptr, int N,
                                                                int K, const int32_t* __restrict__ gather_rows,
                                                                int gather_div, int relu) {
    constexpr int BM = 64, BN = 64, BK = 16;
    __shared__ float sA[BK][BM + 4];
    __shared__ float sB1[BK][BN + 4];
    __shared__ float sB3[SWIGLU ? BK : 1][BN + 4];
    const int n_mtiles = n_mtiles_ptr[0];
    const int n_ntiles = (N + BN - 1) / BN;
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;  // 16 x 16 threads, 4x4 outputs each
    for (int tile = blockIdx.x; tile < n_mtiles * n_ntiles; tile += gridDim.x) {
        const MTile mt = mtiles[tile / n_ntiles];
        const int n0 = (tile % n_ntiles) * BN;
        const float* b1 = B1 + (size_t)mt.expert * b_stride;
        const float* b3 = SWIGLU ? B3 + (size_t)mt.expert * b_stride : nullptr;
        float acc1[4][4] = {}, acc3[4][4] = {};
        for (int k0 = 0; k0 < K; k0 += BK) {
            __syncthreads();
            for (int i = tid; i < BM * BK; i += 256) {
                const int r = i / BK, c = i % BK;
                const int rr = r < mt.rows ? r : mt.rows - 1;
                const int src = gather_rows ? gather_rows[mt.row0 + rr] / gather_div : mt.row0 + rr;
                sA[c][r] = (k0 + c < K) ? A[(size_t)src * lda + k0 + c] : 0.f;
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
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int row = ty * 4 + i, col = n0 + tx * 4 + j;
                if (row < mt.rows && col < N) {
                    float v = acc1[i][j];
                    if (SWIGLU) v = v / (1.0f + expf(-v)) * acc3[i][j];
                    else if (relu) v = fmaxf(v, 0.f);
                    C[(size_t)(mt.row0 + row) * ldc + col] = v;
                }
            }
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
struct FfnWs {
    void* h;          // [A, ffn] hidden activations
    MTile* tiles1;    // M-tiles for GEMM-1
    MTile* tiles2;    // M-tiles for GEMM-2
    int32_t* counts;  // [0..1], [2..4]: number of M-tiles and of full-height M-tiles in tiles1, tiles2
                      // (tiles2 also: number of ragged tiles listed in two halves of K)
    int32_t* queues;  // [0..7], [8..15]: per-XCD claim counters of GEMM-1, GEMM-2
    TailInfo* tails;  // ragged tiles of the second product when their K range is split, else null
    float* partials;  // their fp32 slabs: [2 * nseg][kPartRows][d]
    int capacity;
};

constexpr int kMinBM = 64;

static int env_int(const char* name, int dflt) {
    const char* s = getenv(name);
    return (s && *s) ? atoi(s) : dflt;
}

// The bf16 kernels work on a hidden width padded to a multiple of 64: the packed weights
// carry zero columns (W1, W3) and zero rows (W2) for the padding, so the padded hidden
// activations are exact zeros and add nothing to the second product.
static inline int padded_ffn(int ffn, int dtype) {
    return dtype == MOE_DTYPE_BF16 ? (int)align_up((size_t)ffn, 64) : ffn;
}
constexpr int kGemmGrid = 256;  // persistent workgroups: 8 XCDs x 32

// The ragged tiles of the second product are computed as two halves of K (see the table
// builder) when the product has few tiles per workgroup, so that the uneven end of the launch
// matters, and the fp32 slabs are no larger than the hidden activations.  Decided from the sizes the
// workspace is laid out for, so that the layout and the call agree.
static bool split_tails(int64_t A, int d, int ffn, int nseg, int dtype) {
    if (dtype != MOE_DTYPE_BF16 || A < 1) return false;
    const int mode = env_int("MOEGPS_FFN_SPLIT_TAILS", 1);  // 0: never, 2: whenever the kernels can (for tests)
    if (mode == 0) return false;
    const int fp = padded_ffn(ffn, dtype);
    if (fp < 128) return false;
    if (mode == 2) return true;
    const int64_t est_tiles = (A / 256 + (nseg + 1) / 2) * ceil_div(d, 256);
    if (est_tiles > 4 * kGemmGrid) return false;
    const size_t slabs = (size_t)2 * nseg * kPartRows * d * sizeof(float);
    return slabs <= (size_t)A * fp * dtype_size(dtype);  // at most the size of the hidden activations
}

static size_t ffn_ws_layout(int64_t A, int d, int ffn, int nseg, int dtype, char* base, FfnWs* ws) {
    size_t off = 0;
    auto take = [&](size_t bytes) {
        void* p = base ? (void*)(base + off) : nullptr;
        off += align_up(bytes, 256);
        return p;
    };
    FfnWs w;
    w.capacity = (int)(ceil_div64(A > 0 ? A : 1, kMinBM) + 2 * nseg);
    w.h = take((size_t)(A > 0 ? A : 1) * padded_ffn(ffn, dtype) * dtype_size(dtype));
    w.tiles1 = (MTile*)take((size_t)w.capacity * sizeof(MTile));
    w.tiles2 = (MTile*)take((size_t)w.capacity * sizeof(MTile));
    w.counts = (int32_t*)take(256);
    w.queues = w.counts ? w.counts + 8 : nullptr;
    w.tails = nullptr;
    w.partials = nullptr;
    if (split_tails(A, d, ffn, nseg, dtype)) {
        w.tails = (TailInfo*)take((size_t)nseg * sizeof(TailInfo));
        w.partials = (float*)take((size_t)2 * nseg * kPartRows * d * sizeof(float));
    }
    if (ws) *ws = w;
    return off;
}

struct GemmVariant {
    int bm, bn, bk;
    size_t lds;
    int threads;
    void (*kern)(const bf16_t*, int, const bf16_t*, size_t, bf16_t*, int, const MTile*, const int32_t*, int32_t*, int,
                 int, int, const int32_t*, int, float*);
};

template <int BM, int BN, int BK, int WGM, int WGN, int NSTAGE, int EPI, int SCHED = kSchedInterleaved, int MI = 32>
static GemmVariant make_variant() {
    GemmVariant v;
    v.bm = BM;
    v.bn = BN;
    v.bk = BK;
    v.lds = (size_t)NSTAGE * (BM + BN) * BK * 2;
    v.threads = WGM * WGN * 64;
    v.kern = grouped_gemm_bf16_kernel<BM, BN, BK, WGM, WGN, NSTAGE, EPI, SCHED, MI>;
    return v;
}

// tile shapes built into the library, by index; the defaults are 9, 10 and 6 (see the rule in
// grouped_ffn_impl), the others are kept for comparison and run by the tests
static const GemmVariant kGemm1[] = {
    make_variant<128, 256, 64, 2, 2, 3, kEpiSwiglu>(),
    make_variant<256, 256, 64, 2, 2, 2, kEpiSwiglu>(),
    make_variant<128, 512, 32, 1, 4, 3, kEpiSwiglu>(),
    make_variant<256, 256, 64, 2, 4, 2, kEpiSwiglu>(),
    make_variant<64, 256, 64, 1, 4, 3, kEpiSwiglu>(),
    make_variant<256, 256, 32, 2, 4, 4, kEpiSwiglu>(),
    make_variant<128, 256, 64, 2, 4, 3, kEpiSwiglu>(),
    make_variant<256, 256, 64, 2, 4, 2, kEpiSwiglu, kSchedAlternate>(),
    make_variant<256, 256, 64, 2, 2, 2, kEpiSwiglu, kSchedFine>(),
    make_variant<256, 256, 64, 2, 4, 2, kEpiSwiglu, kSchedInterleaved, 16>(),
    make_variant<128, 256, 64, 2, 4, 3, kEpiSwiglu, kSchedInterleaved, 16>(),
};
static const GemmVariant kGemm2[] = {
    make_variant<128, 256, 64, 2, 2, 3, kEpiNone>(),
    make_variant<256, 256, 64, 2, 2, 2, kEpiNone>(),
    make_variant<128, 512, 32, 1, 4, 3, kEpiNone>(),
    make_variant<256, 256, 64, 2, 4, 2, kEpiNone>(),
    make_variant<64, 256, 64, 1, 4, 3, kEpiNone>(),
    make_variant<256, 256, 32, 2, 4, 4, kEpiNone>(),
    make_variant<128, 256, 64, 2, 4, 3, kEpiNone>(),
    make_variant<256, 256, 64, 2, 4, 2, kEpiNone, kSchedAlternate>(),
    make_variant<256, 256, 64, 2, 2, 2, kEpiNone, kSchedFine>(),
    make_variant<256, 256, 64, 2, 4, 2, kEpiNone, kSchedInterleaved, 16>(),
    make_variant<128, 256, 64, 2, 4, 3, kEpiNone, kSchedInterleaved, 16>(),
};
constexpr int kNumVariants = sizeof(kGemm1) / sizeof(kGemm1[0]);
// first product of the ReLU form of the FFN (default tile shape only)
static const GemmVariant kGemm1Relu = make_variant<256, 256, 64, 2, 4, 2, kEpiRelu, kSchedInterleaved, 16>();

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
                            bf16_t* C, int ldc, const MTile* tiles, const int32_t* n_tiles, int32_t* queues, int N,
                            int K, int group_n, const int32_t* gather_rows, int gather_div, float* partials,
                            hipStream_t st) {
    hipError_t e = hipFuncSetAttribute((const void*)v.kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)v.lds);
    if (e != hipSuccess) {
        set_last_hip_error(e);
        return MOE_ERR_HIP;
    }
    // 32 workgroups for each of the 8 XCDs; they claim tiles from `queues` (cleared by the table builder)
    hipLaunchKernelGGL(v.kern, dim3(kGemmGrid), dim3(v.threads), v.lds, st, A, lda, Bp, b_stride, C, ldc, tiles,
                       n_tiles, queues, N, K, group_n, gather_rows, gather_div, partials);
    return check_launch();
}

}  // namespace moegps

extern "C" size_t moe_packed_weights_bytes(int E, int d, int ffn, int dtype) {
    if (E < 1 || d < 1 || ffn < 1) return 0;
    return (size_t)3 * E * d * moegps::padded_ffn(ffn, dtype) * moegps::dtype_size(dtype);
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
    const size_t ep = (size_t)d * fp;       // and padded
    bf16_t* p1 = (bf16_t*)packed;           // [E][n1*fp][d]; gate/up interleaved by 32 columns when n1 = 2
    bf16_t* p2 = p1 + n1 * E * ep;          // [E][d][fp]
    // W1 (, W3): in[k = d][n = ffn] -> out[n'][d], zero rows for n >= ffn
    dim3 g13(fp / 32, d / 32, E);
    hipLaunchKernelGGL(pack_transpose_kernel, g13, dim3(256), 0, st, (const bf16_t*)W1, p1, d, ffn, d, fp, es,
                       n1 * ep, W3 ? 1 : 0, 0);
    int rc = check_launch();
    if (rc != MOE_OK) return rc;
    if (W3) {
        hipLaunchKernelGGL(pack_transpose_kernel, g13, dim3(256), 0, st, (const bf16_t*)W3, p1, d, ffn, d, fp, es,
                           2 * ep, 1, 1);
        if ((rc = check_launch()) != MOE_OK) return rc;
    }
    // W2: in[k = ffn][n = d] -> out[n = d][k = fp], zero for k >= ffn
    dim3 g2(d / 32, fp / 32, E);
    hipLaunchKernelGGL(pack_transpose_kernel, g2, dim3(256), 0, st, (const bf16_t*)W2, p2, ffn, d, fp, d, es, ep, 0,
                       0);
    return check_launch();
}
}  // namespace moegps

extern "C" int moe_pack_weights(const void* W1, const void* W3, const void* W2, int dtype, int E, int d, int ffn,
                                void* packed, void* stream) {
    if (!W3) return MOE_ERR_INVALID_ARG;
    return moegps::pack_weights_impl(W1, W3, W2, dtype, E, d, ffn, packed, stream);
}

extern "C" size_t moe_packed_weights_relu_bytes(int E, int d, int ffn, int dtype) {
    if (E < 1 || d < 1 || ffn < 1) return 0;
    return (size_t)2 * E * d * moegps::padded_ffn(ffn, dtype) * moegps::dtype_size(dtype);
}

extern "C" int moe_pack_weights_relu(const void* W1, const void* W2, int dtype, int E, int d, int ffn, void* packed,
                                     void* stream) {
    return moegps::pack_weights_impl(W1, nullptr, W2, dtype, E, d, ffn, packed, stream);
}

extern "C" size_t moe_grouped_ffn_workspace_bytes(int64_t A, int d, int ffn, int nseg, int dtype) {
    using namespace moegps;
    if (A < 0 || d < 1 || ffn < 1 || nseg < 1) return 0;
    return ffn_ws_layout(A, d, ffn, nseg, dtype, nullptr, nullptr);
}

namespace moegps {
// x_perm rows are read directly (gather_rows == nullptr) or row r is x_perm[gather_rows[r] / gather_div]
static int grouped_ffn_impl(int relu, const void* x_perm, const int32_t* gather_rows, int gather_div, int dtype, int64_t A,
                            int d, int ffn, int E, const int32_t* seg_offsets, const int32_t* slot_expert, int nseg,
                            int seg_begin, int seg_end, const void* packed, void* y_perm, void* workspace,
                            size_t workspace_bytes, void* stream) {
    if (dtype != MOE_DTYPE_F32 && dtype != MOE_DTYPE_BF16) return MOE_ERR_INVALID_ARG;
    if (A < 0 || d < 1 || ffn < 1 || E < 1 || nseg < 1) return MOE_ERR_INVALID_ARG;
    if (seg_begin < 0 || seg_end > nseg || seg_begin > seg_end) return MOE_ERR_INVALID_ARG;
    if (nseg > MOE_MAX_SEGMENTS || A >= (1ll << 31)) return MOE_ERR_UNSUPPORTED;
    if (dtype == MOE_DTYPE_BF16 && d % 64 != 0) return MOE_ERR_UNSUPPORTED;
    if (dtype == MOE_DTYPE_F32 && (d % 4 != 0 || ffn % 4 != 0)) return MOE_ERR_UNSUPPORTED;
    if ((int64_t)256 * (d > ffn + 63 ? d : ffn + 63) >= (1ll << 31)) return MOE_ERR_UNSUPPORTED;  // 32-bit tile offsets
    if (!seg_offsets || !slot_expert || !packed || !workspace) return MOE_ERR_INVALID_ARG;
    if (A > 0 && (!x_perm || !y_perm)) return MOE_ERR_INVALID_ARG;
    FfnWs ws;
    const size_t need = ffn_ws_layout(A, d, ffn, nseg, dtype, (char*)workspace, &ws);
    if (workspace_bytes < need) return MOE_ERR_WORKSPACE_TOO_SMALL;
    if (A == 0 || seg_begin == seg_end) return MOE_OK;
    hipStream_t st = (hipStream_t)stream;
    const size_t per = (size_t)E * d * ffn;
    int rc;

    if (dtype == MOE_DTYPE_F32) {
        hipLaunchKernelGGL(build_mtiles_kernel, dim3(1), dim3(1024), 0, st, seg_offsets, slot_expert, seg_begin,
                           seg_end, E, 64, ws.tiles1, ws.capacity, ws.counts, (int32_t*)nullptr, 0, 0,
                           (TailInfo*)nullptr);
        if ((rc = check_launch()) != MOE_OK) return rc;
        const float* w1 = (const float*)packed;
        const float* w3 = w1 + per;
        const float* w2 = relu ? w3 : w3 + per;
        const int grid = 4 * num_cus();
        if (relu)
            hipLaunchKernelGGL((grouped_gemm_f32_kernel<false>), dim3(grid), dim3(256), 0, st, (const float*)x_perm, d,
                               w1, (const float*)nullptr, (size_t)d * ffn, (float*)ws.h, ffn, ws.tiles1, ws.counts,
                               ffn, d, gather_rows, gather_div, 1);
        else
            hipLaunchKernelGGL((grouped_gemm_f32_kernel<true>), dim3(grid), dim3(256), 0, st, (const float*)x_perm, d,
                               w1, w3, (size_t)d * ffn, (float*)ws.h, ffn, ws.tiles1, ws.counts, ffn, d, gather_rows,
                               gather_div, 0);
        if ((rc = check_launch()) != MOE_OK) return rc;
        hipLaunchKernelGGL((grouped_gemm_f32_kernel<false>), dim3(grid), dim3(256), 0, st, (const float*)ws.h, ffn,
                           w2, (const float*)nullptr, (size_t)d * ffn, (float*)y_perm, d, ws.tiles1, ws.counts, d,
                           ffn, (const int32_t*)nullptr, 1, 0);
        return check_launch();
    }

    // Tile shape per product: 256x256 (index 9) unless the product has too few such tiles to
    // keep 256 workgroups busy for two rounds, then 128x256 with three stages (index 10); both
    // with the 16x16x32 matrix instruction.  The tile count is only known on the device; the
    // host estimates it from the row count.
    auto pick = [&](const char* env_name, int n_cols) {
        const int v = env_int(env_name, -1);
        if (v >= 0) return v < kNumVariants ? v : 0;
        const int64_t est_mtiles = A / 256 + (seg_end - seg_begin + 1) / 2;
        // segments of a few rows each (decode): every tile is a sliver; the low 32x32x16 tile,
        // which skips the reads of rows that are not there, handles those fastest
        if (A < (int64_t)64 * (seg_end - seg_begin)) return 6;
        return est_mtiles * ceil_div(n_cols, 256) > 2 * kGemmGrid ? 9 : 10;
    };
    const int v1 = pick("MOEGPS_FFN_TILE1", (relu ? 1 : 2) * padded_ffn(ffn, dtype));
    const int v2 = pick("MOEGPS_FFN_TILE2", d);
    // N-tiles walked side by side under one run of M-tiles: all of them when the output is
    // narrow (at most 16 tiles), else 8 (measured best on the Mixtral-shaped gate/up product)
    const int group_env = env_int("MOEGPS_FFN_GROUP_N", 0);
    auto group_for = [&](int n_cols, int bn) {
        if (group_env > 0) return group_env;
        const int n_ntiles = ceil_div(n_cols, bn);
        return n_ntiles <= 16 ? n_ntiles : 8;
    };
    const GemmVariant& g1 = relu ? kGemm1Relu : kGemm1[v1];
    const GemmVariant& g2 = kGemm2[v2];
    hipLaunchKernelGGL(build_mtiles_kernel, dim3(1), dim3(1024), 0, st, seg_offsets, slot_expert, seg_begin, seg_end,
                       E, g1.bm, ws.tiles1, ws.capacity, ws.counts, ws.queues, 16, 0, (TailInfo*)nullptr);
    if ((rc = check_launch()) != MOE_OK) return rc;
    const MTile* tiles2 = ws.tiles1;
    const int32_t* count2 = ws.counts;
    const int fp = padded_ffn(ffn, dtype);  // hidden width the kernels see
    const bool split = ws.partials != nullptr && g2.bm <= kPartRows && fp / g2.bk >= 2;
    // the second product walks its own M-tiles only if its tile height differs or it splits ragged tiles
    if (g2.bm != g1.bm || split) {
        hipLaunchKernelGGL(build_mtiles_kernel, dim3(1), dim3(1024), 0, st, seg_offsets, slot_expert, seg_begin,
                           seg_end, E, g2.bm, ws.tiles2, ws.capacity, ws.counts + 2, (int32_t*)nullptr, 0,
                           split ? fp / g2.bk : 0, ws.tails);
        if ((rc = check_launch()) != MOE_OK) return rc;
        tiles2 = ws.tiles2;
        count2 = ws.counts + 2;
    }
    const int n1 = relu ? 1 : 2;  // matrices in the first product
    const bf16_t* p13 = (const bf16_t*)packed;
    const bf16_t* p2 = p13 + (size_t)n1 * E * d * fp;
    const bool timed = g_time_armed;
    g_time_armed = false;
    if (timed) (void)hipEventRecord(g_time_events[0], st);
    rc = launch_gemm_bf16(g1, (const bf16_t*)x_perm, d, p13, (size_t)n1 * d * fp, (bf16_t*)ws.h, fp, ws.tiles1,
                          ws.counts, ws.queues, n1 * fp, d, group_for(n1 * fp, g1.bn), gather_rows, gather_div,
                          nullptr, st);
    if (timed) (void)hipEventRecord(g_time_events[1], st);
    if (rc != MOE_OK) return rc;
    if (timed) (void)hipEventRecord(g_time_events[2], st);
    rc = launch_gemm_bf16(g2, (const bf16_t*)ws.h, fp, p2, (size_t)d * fp, (bf16_t*)y_perm, d, tiles2, count2,
                          ws.queues + 8, d, fp, group_for(d, g2.bn), nullptr, 1, ws.partials, st);
    if (rc == MOE_OK && split) {
        hipLaunchKernelGGL(add_partials_kernel, dim3(seg_end - seg_begin, 32), dim3(256), 0, st, ws.partials,
                           ws.tails, count2, (bf16_t*)y_perm, d, d);
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
    return moegps::grouped_ffn_impl(0, x_perm, nullptr, 1, dtype, A, d, ffn, E, seg_offsets, slot_expert, nseg,
                                    seg_begin, seg_end, packed, y_perm, workspace, workspace_bytes, stream);
}

extern "C" int moe_grouped_ffn_relu(const void* x_perm, int dtype, int64_t A, int d, int ffn, int E,
                                    const int32_t* seg_offsets, const int32_t* slot_expert, int nseg, int seg_begin,
                                    int seg_end, const void* packed, void* y_perm, void* workspace,
                                    size_t workspace_bytes, void* stream) {
    return moegps::grouped_ffn_impl(1, x_perm, nullptr, 1, dtype, A, d, ffn, E, seg_offsets, slot_expert, nseg,
                                    seg_begin, seg_end, packed, y_perm, workspace, workspace_bytes, stream);
}

extern "C" int moe_grouped_ffn_gather(const void* x, int dtype, int T, int k, const int32_t* assign_of_row, int d,
                                      int ffn, int E, const int32_t* seg_offsets, const int32_t* slot_expert,
                                      int nseg, int seg_begin, int seg_end, const void* packed, void* y_perm,
                                      void* workspace, size_t workspace_bytes, void* stream) {
    if (T < 0 || k < 1 || d < 1) return MOE_ERR_INVALID_ARG;
    if ((int64_t)T * d >= (1ll << 31)) return MOE_ERR_UNSUPPORTED;  // 32-bit element offsets into x
    if (T > 0 && !assign_of_row) return MOE_ERR_INVALID_ARG;
    return moegps::grouped_ffn_impl(0, x, assign_of_row, k, dtype, (int64_t)T * k, d, ffn, E, seg_offsets, slot_expert,
                                    nseg, seg_begin, seg_end, packed, y_perm, workspace, workspace_bytes, stream);
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
