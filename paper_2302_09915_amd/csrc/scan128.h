// Workgroup-wide exclusive prefix sum over at most 128 integers held in LDS.
#pragma once

#include "internal.h"

namespace tamoe {

// Exclusive prefix sum of v[0..n) (n <= 128) into out[0..n], out[n] = total.  Called by every
// thread of the workgroup (at least 128 threads); tmp is 256 ints of LDS; v, out, tmp in LDS.
__device__ __forceinline__ void exclusive_scan_128(const int32_t* v, int32_t* out, int32_t* tmp, int n) {
    const int t = threadIdx.x;
    const int32_t mine = (t < n) ? v[t] : 0;
    if (t < 128) tmp[t] = mine;
    __syncthreads();
    int cur = 0;
#pragma unroll
    for (int s = 1; s < 128; s <<= 1) {
        if (t < 128) tmp[(cur ^ 1) * 128 + t] = tmp[cur * 128 + t] + (t >= s ? tmp[cur * 128 + t - s] : 0);
        __syncthreads();
        cur ^= 1;
    }
    if (t < n) {
        const int32_t incl = tmp[cur * 128 + t];
        out[t] = incl - mine;
        if (t == n - 1) out[n] = incl;
    }
    if (n == 0 && t == 0) out[0] = 0;
    __syncthreads();
}

}  // namespace tamoe
