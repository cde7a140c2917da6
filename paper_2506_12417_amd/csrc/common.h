// Shared host/device helpers of libmoe (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "moe.h"

// Records the calling thread's error text (printf-style) and returns `code`.
int moe_fail(int code, const char* fmt, ...);

#define MOE_REQUIRE(cond, code, ...)            \
    do {                                        \
        if (!(cond)) return moe_fail((code), __VA_ARGS__); \
    } while (0)

// After a kernel launch: turn a launch error into MOE_ERR_HIP.
#define MOE_CHECK_LAUNCH(what)                                                        \
    do {                                                                              \
        hipError_t e_ = hipGetLastError();                                            \
        if (e_ != hipSuccess) return moe_fail(MOE_ERR_HIP, "%s: %s", (what), hipGetErrorString(e_)); \
    } while (0)

#define MOE_CHECK_HIP(expr)                                                           \
    do {                                                                              \
        hipError_t e_ = (expr);                                                       \
        if (e_ != hipSuccess) return moe_fail(MOE_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

static inline size_t moe_elem_size(moe_dtype dt) { return dt == MOE_BF16 ? 2 : 4; }
static inline bool moe_dtype_ok(int dt) { return dt == MOE_F32 || dt == MOE_BF16; }

#define MOE_WAVE 64

// bfloat16 <-> float (bit level; round to nearest, ties to even; NaN kept quiet)
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

template <typename T> __device__ __forceinline__ float load_as_f32(const T* p);
template <> __device__ __forceinline__ float load_as_f32<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float load_as_f32<uint16_t>(const uint16_t* p) { return bf16_to_f32(*p); }

// Wave-wide unsigned min / max / sum at ALU speed (all 64 lanes must be active): four DPP steps
// reduce each row of 16 lanes (pairs, quads, half rows, rows), then the four row results are
// combined through SGPRs.  Every lane gets the result.
__device__ __forceinline__ unsigned moe_wave_min_u32(unsigned v) {
    unsigned t;
    t = __builtin_amdgcn_update_dpp(v, v, 0xB1, 0xf, 0xf, false); v = t < v ? t : v;    // quad_perm [1,0,3,2]
    t = __builtin_amdgcn_update_dpp(v, v, 0x4E, 0xf, 0xf, false); v = t < v ? t : v;    // quad_perm [2,3,0,1]
    t = __builtin_amdgcn_update_dpp(v, v, 0x141, 0xf, 0xf, false); v = t < v ? t : v;   // row_half_mirror
    t = __builtin_amdgcn_update_dpp(v, v, 0x140, 0xf, 0xf, false); v = t < v ? t : v;   // row_mirror
    unsigned a = __builtin_amdgcn_readlane(v, 0), b = __builtin_amdgcn_readlane(v, 16);
    unsigned c = __builtin_amdgcn_readlane(v, 32), d = __builtin_amdgcn_readlane(v, 48);
    a = a < b ? a : b;
    c = c < d ? c : d;
    return a < c ? a : c;
}
__device__ __forceinline__ unsigned moe_wave_max_u32(unsigned v) { return ~moe_wave_min_u32(~v); }
__device__ __forceinline__ unsigned moe_wave_sum_u32(unsigned v) {
    v += (unsigned)__builtin_amdgcn_update_dpp((int)v, (int)v, 0xB1, 0xf, 0xf, false);
    v += (unsigned)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x4E, 0xf, 0xf, false);
    v += (unsigned)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x141, 0xf, 0xf, false);
    v += (unsigned)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x140, 0xf, 0xf, false);
    return __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) + __builtin_amdgcn_readlane(v, 32) +
           __builtin_amdgcn_readlane(v, 48);
}
// max of non-negative floats (their bit patterns order like unsigned integers)
__device__ __forceinline__ float moe_wave_max_nonneg(float v) {
    return __uint_as_float(moe_wave_max_u32(__float_as_uint(v)));
}
