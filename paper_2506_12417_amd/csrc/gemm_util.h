// Device-side helpers shared by the 16-bit grouped GEMM kernels (ffn_bf16.hip, ffn_stream.hip).
#pragma once
#include "common.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
typedef __attribute__((address_space(3))) void lds_void_t;

// s_waitcnt on vmcnt only (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[15:14])
#define MOE_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 0xF) | (((n) >> 4) << 14) | (0x7 << 4) | (0xF << 8))
// s_waitcnt on lgkmcnt only
#define MOE_WAIT_LGKMCNT(n) __builtin_amdgcn_s_waitcnt(0xF | (0x3 << 14) | (0x7 << 4) | (((n) & 0xF) << 8))

__device__ __forceinline__ float silu_f(float z) { return z / (1.f + __expf(-z)); }

// raw buffer descriptor over [p, p + bytes): offsets beyond `bytes` read 0 / are not written
// (pointer and size are wave-uniform; readfirstlane tells the compiler so)
__device__ __forceinline__ int sgpr(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ const void* sgpr_ptr(const void* p) {
    const uint64_t u = (uint64_t)p;
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)u);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(u >> 32));
    return (const void*)(((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, unsigned bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(sgpr_ptr(p)), 0, sgpr((int)bytes), 0x00020000);
}

// take_ticket: lane 0 adds one to *ctr; the old value arrives some time later, like a load, in
// register v250.  read_ticket fetches it from there; the caller does so only after a vmcnt wait
// that covers the request.  Written as assembly with a fixed register, because the compiler would
// wait for the answer on the spot (draining the whole queue of operand loads in flight), and
// because a result register it knows of gets copied around before the answer is in it.  This is
// sound only in kernels whose own code never touches v250: the kernels that use it stay well
// below 250 registers, and a unit test compiles this file and checks that v250 appears in these
// two instructions only.
#define MOE_TICKET_REG "v250"
__device__ __forceinline__ void take_ticket(int32_t* ctr) {
    unsigned long long saved;
    asm volatile(
        "s_mov_b64 %0, exec\n\t"
        "s_mov_b64 exec, 1\n\t"
        "global_atomic_add " MOE_TICKET_REG ", %1, %2, %3 sc0\n\t"
        "s_mov_b64 exec, %0"
        : "=&s"(saved)
        : "v"(0), "v"(1), "s"(ctr)
        : "memory", MOE_TICKET_REG);
}
__device__ __forceinline__ int read_ticket() {
    int v;
    asm volatile("v_readfirstlane_b32 %0, " MOE_TICKET_REG : "=s"(v) : : MOE_TICKET_REG);
    return v;
}

}  // namespace
