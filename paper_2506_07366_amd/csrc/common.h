// Shared host-side helpers of libmoegps (error recording, launch checks).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/moegps.h"

namespace moegps {

constexpr int kWave = 64;

void set_last_hip_error(hipError_t e);

// Records a failed launch; returns MOE_OK or MOE_ERR_HIP.
inline int check_launch() {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_last_hip_error(e);
        return MOE_ERR_HIP;
    }
    return MOE_OK;
}

// a >= 0, b > 0; no intermediate sum, so a may be as large as the type allows
__host__ __device__ inline int ceil_div(int a, int b) { return a / b + (a % b != 0 ? 1 : 0); }
__host__ __device__ inline int64_t ceil_div64(int64_t a, int64_t b) { return a / b + (a % b != 0 ? 1 : 0); }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline int dtype_size(int dtype) { return dtype == MOE_DTYPE_BF16 ? 2 : 4; }

}  // namespace moegps
