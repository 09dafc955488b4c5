// Shared host-side helpers of the HIP sources (error bookkeeping, launch checks).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "graft.h"

namespace graft {

// Raw hipError_t of the last failed launch on this thread; defined in api.hip.
void set_last_hip_error(int32_t e);

// Checks the launch that was just enqueued; maps a failure to GRAFT_ERR_HIP.
inline int32_t check_launch() {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_last_hip_error(static_cast<int32_t>(e));
        return GRAFT_ERR_HIP;
    }
    return GRAFT_OK;
}

using u64 = unsigned long long;

__device__ __forceinline__ u64 shfl_xor_u64(u64 v, int lane_mask) {
    unsigned lo = static_cast<unsigned>(v), hi = static_cast<unsigned>(v >> 32);
    lo = __shfl_xor(lo, lane_mask);
    hi = __shfl_xor(hi, lane_mask);
    return (static_cast<u64>(hi) << 32) | lo;
}

// Maximum of a 64-bit key over one 64-lane wavefront (all lanes get it).
__device__ __forceinline__ u64 wave_max_u64(u64 v) {
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) {
        u64 o = shfl_xor_u64(v, s);
        v = o > v ? o : v;
    }
    return v;
}

}  // namespace graft
