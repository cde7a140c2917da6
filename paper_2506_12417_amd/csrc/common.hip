// Error text, version, workspace sizes and the threshold q (section 4.4, Eq. 4).
#include "common.h"
#include <cstdarg>
#include <cstdio>
#include <cmath>

static thread_local char g_err[512] = "";

int moe_fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

extern "C" const char* moe_last_error(void) { return g_err; }
extern "C" const char* moe_version(void) { return "libmoe 0.1 (gfx950)"; }

// Eq. 4: q > phi * d_type / (2 * beta)
extern "C" int moe_token_threshold(double phi, int d_type, double beta) {
    if (!(phi > 0.0) || !(beta > 0.0) || d_type < 1) return 1;
    double q = phi * (double)d_type / (2.0 * beta);
    if (q > 1e9) q = 1e9;
    int qi = (int)std::ceil(q);
    return qi < 1 ? 1 : qi;
}

// permute scratch: one histogram of E counters per block of PERMUTE_BLOCK_ITEMS assignments
extern "C" size_t moe_workspace_bytes(int op, int T, int d, int F, int E, int k, moe_dtype dt) {
    (void)d; (void)F; (void)dt;
    if (op == MOE_OP_PERMUTE) {
        if (T < 0 || k < 1 || E < 1) return 0;
        size_t A = (size_t)T * (size_t)k;
        size_t nb = (A + 1023) / 1024;
        if (nb == 0) nb = 1;
        return nb * (size_t)E * sizeof(int32_t);
    }
    return 0;
}

// ------------------------------------------------------------------------------------------
// moe_copy_bytes: a plain device-to-device copy, 16 bytes per lane, grid-stride.  It moves a
// known number of bytes through HBM, which makes it the reference for scaling hardware
// traffic counters (what the counter reports for this kernel vs. the bytes it really moved).
namespace {
__global__ __launch_bounds__(256) void copy_bytes_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}
}  // namespace

extern "C" int moe_copy_bytes(const void* src, void* dst, size_t bytes, void* stream) {
    MOE_REQUIRE(bytes % 16 == 0, MOE_ERR_UNSUPPORTED, "moe_copy_bytes: %zu bytes is not a multiple of 16", bytes);
    if (bytes == 0) return MOE_OK;
    MOE_REQUIRE(src && dst, MOE_ERR_ARG, "moe_copy_bytes: null pointer");
    MOE_REQUIRE((((uintptr_t)src | (uintptr_t)dst) & 15) == 0, MOE_ERR_UNSUPPORTED, "moe_copy_bytes: pointers must be 16-byte aligned");
    const size_t n16 = bytes / 16;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(copy_bytes_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, (const uint4*)src,
                       (uint4*)dst, n16);
    MOE_CHECK_LAUNCH("moe_copy_bytes");
    return MOE_OK;
}
