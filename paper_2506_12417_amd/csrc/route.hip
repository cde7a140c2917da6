// moe_route_topk: router logits, softmax, top-k selection (Alg. 1 step 1; section 2).
// This file: argument checks, and the fp32-input kernel (plain FMAs); bf16 inputs go to the MFMA
// kernel in route_mfma.hip, which follows the same scheme.
//
// One work-group takes 64 tokens.  The logits x.W_g are accumulated with fp32 FMAs in chunks of
// 32 terms; every chunk's partial sum is then added into an fp64 accumulator, so the only
// rounding that matters is the one inside a chunk: |error| <= 32u * |x_t| * |w_e| (u = 2^-24,
// Cauchy-Schwarz on the sum of |products|).  The top-k decision of a token is final when all
// its deciding gaps are wider than twice that bound; the few tokens that fail the test get
// their logits recomputed entirely in fp64 by their wavefront, so the selected experts and
// their order are those of exact arithmetic.  HBM traffic: x once, W_g once per work-group
// (L2-resident), k*(4+4) bytes out per token.
#include "common.h"
#include <climits>

namespace {

constexpr int TB = 64;    // tokens per work-group
constexpr int KC = 32;    // terms accumulated in fp32 before the partial sum goes to fp64
constexpr int NTH = 256;

template <typename V> __device__ __forceinline__ bool beats(V av, int ae, V bv, int be) {
    return av > bv || (av == bv && ae < be);
}
template <typename V> __device__ __forceinline__ void wave_best(V& v, int& e) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        V ov = __shfl_xor(v, off);
        int oe = __shfl_xor(e, off);
        if (beats(ov, oe, v, e)) { v = ov; e = oe; }
    }
}
template <typename V> __device__ __forceinline__ V wave_sum(V v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
    return v;
}
template <typename V> __device__ __forceinline__ V wave_max(V v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) { V o = __shfl_xor(v, off); v = o > v ? o : v; }
    return v;
}
template <typename V> __device__ __forceinline__ V neg_inf();
template <> __device__ __forceinline__ float neg_inf<float>() { return -__builtin_huge_valf(); }
template <> __device__ __forceinline__ double neg_inf<double>() { return -__builtin_huge_val(); }
__device__ __forceinline__ float exp_v(float z) { return __expf(z) ; }
__device__ __forceinline__ double exp_v(double z) { return exp(z); }

constexpr int MAXR = MOE_MAX_TOPK + 1;

// A wavefront holds one token's logits, lane l owning experts l, l+64, l+128, l+192.
// Picks the `rounds` largest (ties to the lower expert id), and the softmax denominator.
template <typename V>
__device__ __forceinline__ void select_topk(V (&v)[4], int lane, int E, int rounds,
                                            V (&sel_v)[MAXR], int (&sel_e)[MAXR], V& denom) {
    V m = neg_inf<V>();
#pragma unroll
    for (int j = 0; j < 4; ++j) if (lane + 64 * j < E) m = v[j] > m ? v[j] : m;
    m = wave_max(m);
    V s = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) if (lane + 64 * j < E) s += exp_v(v[j] - m);
    denom = wave_sum(s);
#pragma unroll
    for (int r = 0; r < MAXR; ++r) {
        if (r < rounds) {
            V bv = neg_inf<V>();
            int be = INT_MAX;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                int e = lane + 64 * j;
                if (e < E && beats(v[j], e, bv, be)) { bv = v[j]; be = e; }
            }
            wave_best(bv, be);
            sel_v[r] = bv;
            sel_e[r] = be;
#pragma unroll
            for (int j = 0; j < 4; ++j) if (lane + 64 * j == be) v[j] = neg_inf<V>();
        }
    }
}

template <typename V>
__device__ __forceinline__ void write_choice(const V (&sel_v)[MAXR], const int (&sel_e)[MAXR], V denom,
                                             int k, int renorm, int lane, int32_t* idx_row, float* w_row) {
    V p[MOE_MAX_TOPK];
    V tot = 0;
#pragma unroll
    for (int r = 0; r < MOE_MAX_TOPK; ++r) {
        if (r < k) { p[r] = exp_v(sel_v[r] - sel_v[0]) / denom; tot += p[r]; }
    }
#pragma unroll
    for (int r = 0; r < MOE_MAX_TOPK; ++r) {
        if (r < k && lane == r) {
            idx_row[r] = sel_e[r];
            w_row[r] = (float)(renorm ? p[r] / tot : p[r]);
        }
    }
}

template <typename XT, int NE>
__global__ __launch_bounds__(NTH) void route_kernel(const XT* __restrict__ x, const XT* __restrict__ wg,
                                                    const float* __restrict__ bias, int T, int d, int E,
                                                    int k, int renorm, int32_t* __restrict__ idx_out,
                                                    float* __restrict__ w_out, float* __restrict__ logits_out) {
    constexpr int EP = 16 * NE;
    extern __shared__ float smem[];
    float (*xs)[KC + 1] = reinterpret_cast<float (*)[KC + 1]>(smem);
    float (*ws)[EP] = reinterpret_cast<float (*)[EP]>(smem + TB * (KC + 1));
    float (*ls)[EP + 1] = reinterpret_cast<float (*)[EP + 1]>(smem + TB * (KC + 1) + KC * EP);
    float* xn2 = smem + TB * (KC + 1) + KC * EP + TB * (EP + 1);
    float* wn2 = xn2 + TB;

    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int t0 = blockIdx.x * TB;

    for (int i = tid; i < KC * EP; i += NTH) (&ws[0][0])[i] = 0.f;
    for (int i = tid; i < EP; i += NTH) wn2[i] = 0.f;
    __syncthreads();

    double acc64[4][NE];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < NE; ++j) acc64[i][j] = 0.0;
    float xsq = 0.f;

    const int s_tok = tid >> 2, s_kk = (tid & 3) * 8;
    const int s_t = t0 + s_tok;

    for (int k0 = 0; k0 < d; k0 += KC) {
        {   // x tile: 64 tokens x 32 terms, 8 consecutive terms per thread
            float v[8];
            if (s_t < T && k0 + s_kk < d) {
                const XT* p = x + (size_t)s_t * d + k0 + s_kk;
#pragma unroll
                for (int i = 0; i < 8; ++i) v[i] = load_as_f32<XT>(p + i);
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) v[i] = 0.f;
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) { xs[s_tok][s_kk + i] = v[i]; xsq = fmaf(v[i], v[i], xsq); }
        }
        for (int i = tid; i < KC * E; i += NTH) {   // W_g chunk: 32 rows x E
            int kk = i / E, e = i - kk * E;
            float v = (k0 + kk < d) ? load_as_f32<XT>(wg + (size_t)(k0 + kk) * E + e) : 0.f;
            ws[kk][e] = v;
            atomicAdd(&wn2[e], v * v);
        }
        __syncthreads();
        float acc[4][NE];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < NE; ++j) acc[i][j] = 0.f;
#pragma unroll 8
        for (int kk = 0; kk < KC; ++kk) {
            float xv[4], wv[NE];
#pragma unroll
            for (int i = 0; i < 4; ++i) xv[i] = xs[ty * 4 + i][kk];
#pragma unroll
            for (int j = 0; j < NE; ++j) wv[j] = ws[kk][tx + 16 * j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < NE; ++j) acc[i][j] = fmaf(xv[i], wv[j], acc[i][j]);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < NE; ++j) acc64[i][j] += (double)acc[i][j];
        __syncthreads();
    }

    xsq += __shfl_xor(xsq, 1);
    xsq += __shfl_xor(xsq, 2);
    if ((tid & 3) == 0) xn2[s_tok] = xsq;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int tok = ty * 4 + i, t = t0 + tok;
#pragma unroll
        for (int j = 0; j < NE; ++j) {
            int e = tx + 16 * j;
            if (e < E) {
                float l = (float)(acc64[i][j] + (bias ? (double)bias[e] : 0.0));
                ls[tok][e] = l;
                if (logits_out && t < T) logits_out[(size_t)t * E + e] = l;
            }
        }
    }
    __syncthreads();

    const int lane = tid & 63, wave = tid >> 6;
    float wmax2 = 0.f, bmax = 0.f;
    for (int e = lane; e < E; e += 64) {
        wmax2 = fmaxf(wmax2, wn2[e]);
        if (bias) bmax = fmaxf(bmax, fabsf(bias[e]));
    }
    const float wn_max = sqrtf(wave_max(wmax2)) * 1.0001f;
    bmax = wave_max(bmax);
    const int rounds = (k + 1 < E) ? k + 1 : E;
    const float u = 5.9604645e-8f;   // 2^-24

    for (int tt = 0; tt < TB / 4; ++tt) {
        const int tok = wave * (TB / 4) + tt, t = t0 + tok;
        if (t >= T) break;
        float v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = (lane + 64 * j < E) ? ls[tok][lane + 64 * j] : 0.f;
        float sel_v[MAXR];
        int sel_e[MAXR];
        float denom;
        select_topk<float>(v, lane, E, rounds, sel_v, sel_e, denom);
        // twice the bound on a logit's error: chunk rounding (KC terms, +2 for the conversions)
        // plus the final rounding of the logit itself to fp32
        const float xn = sqrtf(xn2[tok]) * 1.0001f;
        const float tau = 2.1f * u * ((KC + 3) * xn * wn_max + bmax);
        bool near = false;
#pragma unroll
        for (int r = 0; r + 1 < MAXR; ++r)
            if (r + 1 < rounds && sel_v[r] - sel_v[r + 1] < tau) near = true;
        if (!near) {
            write_choice<float>(sel_v, sel_e, denom, k, renorm, lane, idx_out + (size_t)t * k, w_out + (size_t)t * k);
        } else {
            // exact path: this token's logits in fp64, lane l owning experts l + 64 j
            double v64[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) v64[j] = (bias && lane + 64 * j < E) ? (double)bias[lane + 64 * j] : 0.0;
            const XT* xr = x + (size_t)t * d;
#pragma unroll 4
            for (int i = 0; i < d; ++i) {
                double xv = (double)load_as_f32<XT>(xr + i);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    int e = lane + 64 * j;
                    if (e < E) v64[j] = fma(xv, (double)load_as_f32<XT>(wg + (size_t)i * E + e), v64[j]);
                }
            }
            double sv[MAXR], dn;
            int se[MAXR];
            select_topk<double>(v64, lane, E, rounds, sv, se, dn);
            write_choice<double>(sv, se, dn, k, renorm, lane, idx_out + (size_t)t * k, w_out + (size_t)t * k);
        }
    }
}

template <typename XT, int NE>
int launch_route(const void* x, const void* wg, const float* bias, int T, int d, int E, int k, int renorm,
                 int32_t* idx, float* w, float* logits, hipStream_t st) {
    constexpr int EP = 16 * NE;
    size_t smem = sizeof(float) * (size_t)(TB * (KC + 1) + KC * EP + TB * (EP + 1) + TB + EP);
    auto kern = route_kernel<XT, NE>;
    if (smem > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return moe_fail(MOE_ERR_HIP, "route: shared memory attribute: %s", hipGetErrorString(e));
    }
    int grid = (T + TB - 1) / TB;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(NTH), smem, st, (const XT*)x, (const XT*)wg, bias, T, d, E, k,
                       renorm, idx, w, logits);
    MOE_CHECK_LAUNCH("moe_route_topk");
    return MOE_OK;
}

template <typename XT>
int dispatch_route(const void* x, const void* wg, const float* bias, int T, int d, int E, int k, int renorm,
                   int32_t* idx, float* w, float* logits, hipStream_t st) {
    if (E <= 16) return launch_route<XT, 1>(x, wg, bias, T, d, E, k, renorm, idx, w, logits, st);
    if (E <= 32) return launch_route<XT, 2>(x, wg, bias, T, d, E, k, renorm, idx, w, logits, st);
    if (E <= 64) return launch_route<XT, 4>(x, wg, bias, T, d, E, k, renorm, idx, w, logits, st);
    if (E <= 128) return launch_route<XT, 8>(x, wg, bias, T, d, E, k, renorm, idx, w, logits, st);
    return launch_route<XT, 16>(x, wg, bias, T, d, E, k, renorm, idx, w, logits, st);
}

}  // namespace

// bf16 inputs: the MFMA kernel of route_mfma.hip
int moe_route_bf16_mfma(const void* x, const void* wg, const float* bias, int T, int d, int E, int k, int renorm,
                        int32_t* idx, float* w, float* logits, hipStream_t st);

int moe_route_bf16_packed(const void* x, const void* wgt, const float* w_norm2, const float* bias, int T, int d, int E,
                          int k, int renorm, int32_t* idx, float* w, float* logits, hipStream_t st);

extern "C" int moe_route_topk_packed(const void* x, const void* w_gate_t, const float* w_norm2, const float* bias, int T,
                                     int d, int E, int k, int renorm, moe_dtype dt, int32_t* expert_idx, float* gate_w,
                                     float* logits_out, void* stream) {
    MOE_REQUIRE(dt == MOE_BF16, MOE_ERR_UNSUPPORTED, "moe_route_topk_packed: dtype %d (bf16 only)", (int)dt);
    MOE_REQUIRE(T >= 0 && d >= 1 && E >= 1, MOE_ERR_ARG, "moe_route_topk_packed: T=%d d=%d E=%d", T, d, E);
    MOE_REQUIRE(k >= 1 && k <= E, MOE_ERR_ARG, "moe_route_topk_packed: k=%d outside [1, E=%d]", k, E);
    MOE_REQUIRE(k <= MOE_MAX_TOPK, MOE_ERR_UNSUPPORTED, "moe_route_topk_packed: k=%d > %d", k, MOE_MAX_TOPK);
    MOE_REQUIRE(E <= MOE_MAX_EXPERTS, MOE_ERR_UNSUPPORTED, "moe_route_topk_packed: E=%d > %d", E, MOE_MAX_EXPERTS);
    MOE_REQUIRE(d % 64 == 0, MOE_ERR_UNSUPPORTED, "moe_route_topk_packed: d=%d is not a multiple of 64", d);
    MOE_REQUIRE((long long)d * MOE_MAX_EXPERTS * 2 < (1ll << 31), MOE_ERR_UNSUPPORTED, "moe_route_topk_packed: d=%d too large", d);
    if (T == 0) return MOE_OK;
    MOE_REQUIRE(x && w_gate_t && w_norm2 && expert_idx && gate_w, MOE_ERR_ARG, "moe_route_topk_packed: null pointer");
    return moe_route_bf16_packed(x, w_gate_t, w_norm2, bias, T, d, E, k, renorm, expert_idx, gate_w, logits_out,
                                 (hipStream_t)stream);
}

extern "C" int moe_route_topk(const void* x, const void* w_gate, const float* bias, int T, int d, int E, int k,
                              int renorm, moe_dtype dt, int32_t* expert_idx, float* gate_w, float* logits_out,
                              void* stream) {
    MOE_REQUIRE(moe_dtype_ok(dt), MOE_ERR_UNSUPPORTED, "moe_route_topk: dtype %d", (int)dt);
    MOE_REQUIRE(T >= 0 && d >= 1 && E >= 1, MOE_ERR_ARG, "moe_route_topk: T=%d d=%d E=%d", T, d, E);
    MOE_REQUIRE(k >= 1 && k <= E, MOE_ERR_ARG, "moe_route_topk: k=%d outside [1, E=%d]", k, E);
    MOE_REQUIRE(k <= MOE_MAX_TOPK, MOE_ERR_UNSUPPORTED, "moe_route_topk: k=%d > %d", k, MOE_MAX_TOPK);
    MOE_REQUIRE(E <= MOE_MAX_EXPERTS, MOE_ERR_UNSUPPORTED, "moe_route_topk: E=%d > %d", E, MOE_MAX_EXPERTS);
    MOE_REQUIRE(d % 8 == 0, MOE_ERR_UNSUPPORTED, "moe_route_topk: d=%d is not a multiple of 8", d);
    if (T == 0) return MOE_OK;
    MOE_REQUIRE(x && w_gate && expert_idx && gate_w, MOE_ERR_ARG, "moe_route_topk: null pointer");
    hipStream_t st = (hipStream_t)stream;
    if (dt == MOE_BF16)
        return moe_route_bf16_mfma(x, w_gate, bias, T, d, E, k, renorm, expert_idx, gate_w, logits_out, st);
    return dispatch_route<float>(x, w_gate, bias, T, d, E, k, renorm, expert_idx, gate_w, logits_out, st);
}
