// Exclusive prefix sum of up to 2048 ints held in LDS, by a 1024-thread workgroup.
#pragma once
#include "common.h"

namespace moegps {

// data[0..n) -> exclusive prefix sums in place, data[n] = total.  n <= 2048,
// blockDim.x == 1024, data has room for n+1 ints, wave_sum for 16 ints.
// Every thread of the workgroup must call it.
__device__ inline void block_exclusive_scan_2048(int* data, int n, int* wave_sum) {
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int i0 = 2 * tid, i1 = 2 * tid + 1;
    const int a0 = i0 < n ? data[i0] : 0;
    const int a1 = i1 < n ? data[i1] : 0;
    int incl = a0 + a1;
#pragma unroll
    for (int m = 1; m < kWave; m <<= 1) {
        const int o = __shfl_up(incl, m, kWave);
        if (lane >= m) incl += o;
    }
    if (lane == kWave - 1) wave_sum[tid / kWave] = incl;
    __syncthreads();
    int ws[16];  // all reads first: they overlap
#pragma unroll
    for (int ww = 0; ww < 16; ++ww) ws[ww] = wave_sum[ww];
    int wbase = 0, total = 0;
#pragma unroll
    for (int ww = 0; ww < 16; ++ww) {
        wbase += ww < tid / kWave ? ws[ww] : 0;
        total += ws[ww];
    }
    const int excl = wbase + incl - (a0 + a1);
    if (i0 < n) data[i0] = excl;
    if (i1 < n) data[i1] = excl + a0;
    if (tid == 0) data[n] = total;
    __syncthreads();
}

// The same for two arrays at once (one pass, one pair of barriers): wave_sum has room for 32 ints.
__device__ inline void block_exclusive_scan2_2048(int* da, int* db, int n, int* wave_sum) {
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int i0 = 2 * tid, i1 = 2 * tid + 1;
    const int a0 = i0 < n ? da[i0] : 0, a1 = i1 < n ? da[i1] : 0;
    const int b0 = i0 < n ? db[i0] : 0, b1 = i1 < n ? db[i1] : 0;
    int ia = a0 + a1, ib = b0 + b1;
#pragma unroll
    for (int m = 1; m < kWave; m <<= 1) {
        const int oa = __shfl_up(ia, m, kWave);
        const int ob = __shfl_up(ib, m, kWave);
        if (lane >= m) {
            ia += oa;
            ib += ob;
        }
    }
    if (lane == kWave - 1) {
        wave_sum[tid / kWave] = ia;
        wave_sum[16 + tid / kWave] = ib;
    }
    __syncthreads();
    int sa[16], sb[16];
#pragma unroll
    for (int ww = 0; ww < 16; ++ww) {
        sa[ww] = wave_sum[ww];
        sb[ww] = wave_sum[16 + ww];
    }
    int wa = 0, wb = 0, ta = 0, tb = 0;
#pragma unroll
    for (int ww = 0; ww < 16; ++ww) {
        wa += ww < tid / kWave ? sa[ww] : 0;
        wb += ww < tid / kWave ? sb[ww] : 0;
        ta += sa[ww];
        tb += sb[ww];
    }
    const int ea = wa + ia - (a0 + a1), eb = wb + ib - (b0 + b1);
    if (i0 < n) {
        da[i0] = ea;
        db[i0] = eb;
    }
    if (i1 < n) {
        da[i1] = ea + a0;
        db[i1] = eb + b0;
    }
    if (tid == 0) {
        da[n] = ta;
        db[n] = tb;
    }
    __syncthreads();
}

// sum of v over the 64 lanes of a wavefront (every lane active), in every lane
__device__ __forceinline__ int wave_sum_i32(int v) {
#pragma unroll
    for (int m = kWave / 2; m > 0; m >>= 1) v += __shfl_xor(v, m, kWave);
    return v;
}

}  // namespace moegps
