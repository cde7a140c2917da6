// moe_pack_weights: the paper's W (K inputs x N outputs, section 4.4) rewritten output-major
// (N x K, contraction index contiguous), optionally with a second matrix interleaved in blocks
// of 32 output rows (SwiGLU gate / up).  A 32x32 LDS transpose; done once, outside the hot path.
// moe_pack_w_out: the same for W_out, whose bf16 values become IEEE half on the way (the second
// product of the FFN multiplies half by half).
// 16-bit FFN weights are also reordered inside every block of 32 output rows (PERM): packed row
// 16 h + j of a block holds output 2 j + h.  The 16x16x32 matrix instruction gives lane j of a
// wavefront column j of a 16-column sub-block; with this order the two sub-blocks of a 32-column
// block give a lane two adjacent outputs, which it stores as one pair.
#include "common.h"

namespace {
// bf16 bits -> IEEE half bits, nearest-even (exact for magnitudes 2^-14 .. 65504: half carries
// more significant bits than bf16; smaller values land on the half subnormals, spacing 2^-24)
__device__ __forceinline__ uint16_t bf16_to_half(uint16_t b) {
    const _Float16 h = (_Float16)__uint_as_float((uint32_t)b << 16);
    return __builtin_bit_cast(uint16_t, h);
}
template <typename T, bool TO_HALF = false, bool PERM = false>
__global__ __launch_bounds__(256) void pack_kernel(const T* __restrict__ wa, const T* __restrict__ wb, int K, int N,
                                                   T* __restrict__ out) {
    __shared__ T tile[32][33];
    const int m = blockIdx.z / (wb ? 2 : 1), which = wb ? blockIdx.z % 2 : 0;
    const T* src = (which ? wb : wa) + (size_t)m * K * N;
    const int n0 = blockIdx.x * 32, k0 = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
    for (int r = ty; r < 32; r += 8)
        if (k0 + r < K && n0 + tx < N) tile[r][tx] = src[(size_t)(k0 + r) * N + n0 + tx];
    __syncthreads();
    const int n_rows = wb ? 2 * N : N;
    T* dst = out + (size_t)m * n_rows * K;
    for (int r = ty; r < 32; r += 8) {
        const int n = n0 + r;
        if (n < N && k0 + tx < K) {
            const int c = PERM ? 16 * (n & 1) + ((n % 32) >> 1) : n % 32;
            const int prow = wb ? (n / 32) * 64 + which * 32 + c : (n / 32) * 32 + c;
            if constexpr (TO_HALF) dst[(size_t)prow * K + k0 + tx] = bf16_to_half(tile[tx][r]);
            else dst[(size_t)prow * K + k0 + tx] = tile[tx][r];
        }
    }
}
// squared column norms of W_g [d,E], fp32, rounded up a little: an upper bound for the router's error bound
template <typename T>
__global__ __launch_bounds__(256) void router_norm_kernel(const T* __restrict__ wg, int d, int E, float* __restrict__ norm2) {
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= E) return;
    float s = 0.f;
    for (int i = 0; i < d; ++i) {
        const float v = load_as_f32(wg + (size_t)i * E + e);
        s = fmaf(v, v, s);
    }
    norm2[e] = s * 1.002f;
}
}  // namespace

enum PackKind { PACK_W_IN, PACK_W_OUT, PACK_PLAIN };
static int pack_impl(PackKind kind, const void* w_a, const void* w_b, int n, int K, int N, moe_dtype dt, void* out,
                     void* stream) {
    MOE_REQUIRE(moe_dtype_ok(dt), MOE_ERR_UNSUPPORTED, "moe_pack_weights: dtype %d", (int)dt);
    MOE_REQUIRE(n >= 0 && K >= 1 && N >= 1, MOE_ERR_ARG, "moe_pack_weights: n=%d K=%d N=%d", n, K, N);
    MOE_REQUIRE(!w_b || N % 32 == 0, MOE_ERR_UNSUPPORTED, "moe_pack_weights: interleaving needs N %% 32 == 0 (N=%d)", N);
    if (n == 0) return MOE_OK;
    MOE_REQUIRE(kind == PACK_PLAIN || dt != MOE_BF16 || N % 32 == 0, MOE_ERR_UNSUPPORTED,
                "moe_pack_weights: bf16 weights are ordered in blocks of 32 outputs, N=%d is not a multiple of 32", N);
    MOE_REQUIRE(w_a && out, MOE_ERR_ARG, "moe_pack_weights: null pointer");
    MOE_REQUIRE((long long)n * (w_b ? 2 : 1) <= 65535, MOE_ERR_UNSUPPORTED, "moe_pack_weights: too many matrices");
    dim3 grid((N + 31) / 32, (K + 31) / 32, n * (w_b ? 2 : 1));
    MOE_REQUIRE(grid.y <= 65535, MOE_ERR_UNSUPPORTED, "moe_pack_weights: K too large");
    if (dt == MOE_BF16 && kind == PACK_W_OUT)
        hipLaunchKernelGGL((pack_kernel<uint16_t, true, true>), grid, dim3(256), 0, (hipStream_t)stream, (const uint16_t*)w_a,
                           (const uint16_t*)w_b, K, N, (uint16_t*)out);
    else if (dt == MOE_BF16 && kind == PACK_W_IN)
        hipLaunchKernelGGL((pack_kernel<uint16_t, false, true>), grid, dim3(256), 0, (hipStream_t)stream, (const uint16_t*)w_a,
                           (const uint16_t*)w_b, K, N, (uint16_t*)out);
    else if (dt == MOE_BF16)
        hipLaunchKernelGGL(pack_kernel<uint16_t>, grid, dim3(256), 0, (hipStream_t)stream, (const uint16_t*)w_a,
                           (const uint16_t*)w_b, K, N, (uint16_t*)out);
    else
        hipLaunchKernelGGL(pack_kernel<float>, grid, dim3(256), 0, (hipStream_t)stream, (const float*)w_a,
                           (const float*)w_b, K, N, (float*)out);
    MOE_CHECK_LAUNCH("moe_pack_weights");
    return MOE_OK;
}

extern "C" int moe_pack_weights(const void* w_a, const void* w_b, int n, int K, int N, moe_dtype dt, void* out,
                                void* stream) {
    return pack_impl(PACK_W_IN, w_a, w_b, n, K, N, dt, out, stream);
}

extern "C" int moe_pack_w_out(const void* w, int n, int F, int d, moe_dtype dt, void* out, void* stream) {
    return pack_impl(PACK_W_OUT, w, nullptr, n, F, d, dt, out, stream);
}

extern "C" int moe_pack_router(const void* w_gate, int d, int E, moe_dtype dt, void* w_gate_t, float* w_norm2,
                               void* stream) {
    MOE_REQUIRE(moe_dtype_ok(dt), MOE_ERR_UNSUPPORTED, "moe_pack_router: dtype %d", (int)dt);
    MOE_REQUIRE(d >= 1 && E >= 1, MOE_ERR_ARG, "moe_pack_router: d=%d E=%d", d, E);
    MOE_REQUIRE(w_gate && w_gate_t && w_norm2, MOE_ERR_ARG, "moe_pack_router: null pointer");
    const int rc = pack_impl(PACK_PLAIN, w_gate, nullptr, 1, d, E, dt, w_gate_t, stream);
    if (rc != MOE_OK) return rc;
    if (dt == MOE_BF16)
        hipLaunchKernelGGL(router_norm_kernel<uint16_t>, dim3((E + 255) / 256), dim3(256), 0, (hipStream_t)stream,
                           (const uint16_t*)w_gate, d, E, w_norm2);
    else
        hipLaunchKernelGGL(router_norm_kernel<float>, dim3((E + 255) / 256), dim3(256), 0, (hipStream_t)stream,
                           (const float*)w_gate, d, E, w_norm2);
    MOE_CHECK_LAUNCH("moe_pack_router");
    return MOE_OK;
}
