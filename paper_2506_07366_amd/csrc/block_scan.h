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
    int wbase = 0;
    for (int ww = 0; ww < tid / kWave; ++ww) wbase += wave_sum[ww];
    const int excl = wbase + incl - (a0 + a1);
    if (i0 < n) data[i0] = excl;
    if (i1 < n) data[i1] = excl + a0;
    if (tid == 0) {
        int total = 0;
        for (int ww = 0; ww < 16; ++ww) total += wave_sum[ww];
        data[n] = total;
    }
    __syncthreads();
}

}  // namespace moegps
