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

// OR of a predicate over a workgroup of two wavefronts (the 128-thread kernels): each wavefront
// puts its ballot's verdict into its own LDS slot, one barrier, everyone reads both slots.  The
// library's __syncthreads_or costs several hundred cycles more, which these launch-latency-bound
// kernels notice.  `slots` is LDS, two words, not used for anything else until the next barrier;
// the barrier also orders every LDS write made before the call.
__device__ __forceinline__ bool workgroup_or_128(bool pred, int32_t* slots) {
    const bool wave_any = __builtin_amdgcn_ballot_w64(pred) != 0;
    if ((threadIdx.x & 63) == 0) slots[threadIdx.x >> 6] = wave_any ? 1 : 0;
    __syncthreads();
    return (slots[0] | slots[1]) != 0;
}

// v from the lane that the DPP control names (0xB1: lane ^ 1, 0x4E: lane ^ 2, 0x141: mirror
// within 8 lanes, 0x140: mirror within 16 lanes), both halves of the 64-bit value.
template <int DPP_CTRL>
__device__ __forceinline__ u64 dpp_u64(u64 v) {
    const int lo = static_cast<int>(static_cast<unsigned>(v)), hi = static_cast<int>(static_cast<unsigned>(v >> 32));
    const unsigned lo2 = static_cast<unsigned>(__builtin_amdgcn_update_dpp(lo, lo, DPP_CTRL, 0xf, 0xf, false));
    const unsigned hi2 = static_cast<unsigned>(__builtin_amdgcn_update_dpp(hi, hi, DPP_CTRL, 0xf, 0xf, false));
    return (static_cast<u64>(hi2) << 32) | lo2;
}

// Maximum of a 64-bit key over one 64-lane wavefront (all lanes get it).  Four DPP steps
// reduce each row of 16 lanes (register-to-register, no LDS crossbar); the gfx950 lane
// swaps then combine the rows: permlane16_swap(x, x) returns {rows 0,0,2,2} and
// {rows 1,1,3,3} of x, permlane32_swap(x, x) returns {low half twice} and {high half twice}.
__device__ __forceinline__ u64 wave_max_u64(u64 v) {
    u64 o;
    o = dpp_u64<0xB1>(v);  v = o > v ? o : v;
    o = dpp_u64<0x4E>(v);  v = o > v ? o : v;
    o = dpp_u64<0x141>(v); v = o > v ? o : v;
    o = dpp_u64<0x140>(v); v = o > v ? o : v;
    {
        const unsigned lo = static_cast<unsigned>(v), hi = static_cast<unsigned>(v >> 32);
        const auto rl = __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
        const auto rh = __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
        const u64 a = (static_cast<u64>(rh[0]) << 32) | rl[0], b = (static_cast<u64>(rh[1]) << 32) | rl[1];
        v = a > b ? a : b;
    }
    {
        const unsigned lo = static_cast<unsigned>(v), hi = static_cast<unsigned>(v >> 32);
        const auto rl = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
        const auto rh = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
        const u64 a = (static_cast<u64>(rh[0]) << 32) | rl[0], b = (static_cast<u64>(rh[1]) << 32) | rl[1];
        v = a > b ? a : b;
    }
    return v;
}

// Maximum of a float over one 64-lane wavefront (all lanes get it); same steps as above.
template <int DPP_CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
    const int b = __float_as_int(v);
    return __int_as_float(__builtin_amdgcn_update_dpp(b, b, DPP_CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float wave_max_f32(float v) {
    v = __builtin_fmaxf(v, dpp_f32<0xB1>(v));
    v = __builtin_fmaxf(v, dpp_f32<0x4E>(v));
    v = __builtin_fmaxf(v, dpp_f32<0x141>(v));
    v = __builtin_fmaxf(v, dpp_f32<0x140>(v));
    {
        const unsigned u = __float_as_uint(v);
        const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
        v = __builtin_fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
    }
    {
        const unsigned u = __float_as_uint(v);
        const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
        v = __builtin_fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
    }
    return v;
}

// Maximum over the four lanes l, l + 16, l + 32, l + 48 (the four 16-lane rows of a wavefront),
// all four get it: the two lane swaps of gfx950, no trip through the LDS crossbar.
__device__ __forceinline__ float rows_max_f32(float v) {
    {
        const unsigned u = __float_as_uint(v);
        const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
        v = __builtin_fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
    }
    {
        const unsigned u = __float_as_uint(v);
        const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
        v = __builtin_fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
    }
    return v;
}

}  // namespace graft
