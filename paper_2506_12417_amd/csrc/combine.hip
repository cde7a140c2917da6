// moe_unpermute_combine: original token order restored, the k expert outputs of a token
// weighted by the router's values and summed (Alg. 1 step 6, "reconstruct"; section 2).
// One float4 of one output row per thread; j ascending, so the sum has a fixed order.
// HBM traffic: A*d*4 bytes read (+ T*d*4 for the shared expert), T*d*4 written.
#include "common.h"

namespace {
__global__ __launch_bounds__(256) void combine_kernel(const float4* __restrict__ y_perm,
                                                      const int32_t* __restrict__ inv_perm,
                                                      const float* __restrict__ gate_w,
                                                      const float4* __restrict__ shared, int T, int vpr, int k,
                                                      float4* __restrict__ y) {
    const size_t total = (size_t)T * vpr;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const int t = (int)(i / vpr), v = (int)(i - (size_t)t * vpr);
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int j = 0; j < k; ++j) {
            const float w = gate_w ? gate_w[(size_t)t * k + j] : 1.f;
            const float4 r = y_perm[(size_t)inv_perm[(size_t)t * k + j] * vpr + v];
            acc.x = fmaf(w, r.x, acc.x);
            acc.y = fmaf(w, r.y, acc.y);
            acc.z = fmaf(w, r.z, acc.z);
            acc.w = fmaf(w, r.w, acc.w);
        }
        if (shared) {
            const float4 s = shared[i];
            acc.x += s.x; acc.y += s.y; acc.z += s.z; acc.w += s.w;
        }
        y[i] = acc;
    }
}
}  // namespace

extern "C" int moe_unpermute_combine(const float* y_perm, const int32_t* inv_perm, const float* gate_w,
                                     const float* shared, int T, int d, int k, float* y, void* stream) {
    MOE_REQUIRE(T >= 0 && d >= 1 && k >= 1, MOE_ERR_ARG, "moe_unpermute_combine: T=%d d=%d k=%d", T, d, k);
    MOE_REQUIRE(d % 4 == 0, MOE_ERR_UNSUPPORTED, "moe_unpermute_combine: d=%d is not a multiple of 4", d);
    if (T == 0) return MOE_OK;
    MOE_REQUIRE(y_perm && inv_perm && y, MOE_ERR_ARG, "moe_unpermute_combine: null pointer");
    const int vpr = d / 4;
    size_t blocks = ((size_t)T * vpr + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(combine_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, (const float4*)y_perm,
                       inv_perm, gate_w, (const float4*)shared, T, vpr, k, (float4*)y);
    MOE_CHECK_LAUNCH("moe_unpermute_combine");
    return MOE_OK;
}
