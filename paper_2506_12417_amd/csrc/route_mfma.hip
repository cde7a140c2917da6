// moe_route_topk for bf16 inputs: the router product on the matrix cores (Alg. 1 step 1).
//
// One work-group takes TB tokens (64, or 32 when E > 128).  Logits x.W_g are accumulated by
// v_mfma_f32_32x32x16_bf16 in chunks of 32 terms (bf16 x bf16 products are exact in fp32); each
// chunk's fp32 result is added into fp64 accumulators, so only the rounding inside a chunk
// counts: |error| <= c * |x_t| * |w_e| with c = (2*32+6) * 2^-24 (two roundings per term allowed
// for, since the accumulation order inside the instruction is not specified).  A token whose
// deciding gaps are all wider than twice that bound keeps its fp32 selection; the others get the
// logits of every expert that could still reach the top k recomputed in fp64 by a wavefront, so
// expert indices and their order are those of exact arithmetic (ties to the lower index).
//
// W_g arrives as [d,E] (expert index contiguous); the MFMA wants the contraction index
// contiguous for both operands, so each chunk of W_g is transposed on its way into LDS.
// Selection: TPT = 256/TB threads scan one token's logits from LDS, keep a sorted top-(k+1)
// list in registers, and merge the lists with DPP exchanges inside their group of lanes.
#include "common.h"
#include <climits>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int NTH = 256;
constexpr int KC = 32;                 // terms per fp32 chunk (two MFMAs)
constexpr int PK = KC + 8;             // LDS pitch of a K-row in bf16 elements (80 B: conflict-free 16 B reads)
constexpr int MAXR = MOE_MAX_TOPK + 1;
constexpr float NEG_INF = -__builtin_huge_valf();

__device__ __forceinline__ bool beats(float av, int ae, float bv, int be) { return av > bv || (av == bv && ae < be); }
__device__ __forceinline__ bool beats(double av, int ae, double bv, int be) { return av > bv || (av == bv && ae < be); }

// exchange inside groups of 4 (steps 0,1) or 8 (step 2) neighbouring lanes
template <int STEP> __device__ __forceinline__ int dpp_xchg(int v) {
    if (STEP == 0) return __builtin_amdgcn_update_dpp(v, v, 0xB1, 0xf, 0xf, false);    // quad_perm [1,0,3,2]
    if (STEP == 1) return __builtin_amdgcn_update_dpp(v, v, 0x4E, 0xf, 0xf, false);    // quad_perm [2,3,0,1]
    return __builtin_amdgcn_update_dpp(v, v, 0x141, 0xf, 0xf, false);                  // row_half_mirror
}
template <int STEP> __device__ __forceinline__ float dpp_xchg(float v) {
    return __int_as_float(dpp_xchg<STEP>(__float_as_int(v)));
}
template <int TPT> __device__ __forceinline__ float group_max(float v) {
    v = fmaxf(v, dpp_xchg<0>(v));
    v = fmaxf(v, dpp_xchg<1>(v));
    if (TPT == 8) v = fmaxf(v, dpp_xchg<2>(v));
    return v;
}
// fixed pairing order, so every lane of the group gets the same bits
template <int TPT> __device__ __forceinline__ float group_sum(float v) {
    v += dpp_xchg<0>(v);
    v += dpp_xchg<1>(v);
    if (TPT == 8) v += dpp_xchg<2>(v);
    return v;
}
template <int TPT> __device__ __forceinline__ void group_best(float& v, int& e) {
    float ov; int oe;
    ov = dpp_xchg<0>(v); oe = dpp_xchg<0>(e); if (beats(ov, oe, v, e)) { v = ov; e = oe; }
    ov = dpp_xchg<1>(v); oe = dpp_xchg<1>(e); if (beats(ov, oe, v, e)) { v = ov; e = oe; }
    if (TPT == 8) { ov = dpp_xchg<2>(v); oe = dpp_xchg<2>(e); if (beats(ov, oe, v, e)) { v = ov; e = oe; } }
}

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
    return v;
}
__device__ __forceinline__ void wave_best_f64(double& v, int& e) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        double ov = __shfl_xor(v, off);
        int oe = __shfl_xor(e, off);
        if (beats(ov, oe, v, e)) { v = ov; e = oe; }
    }
}

// MT m-tiles of 32 tokens per work-group, NJ n-tiles of 32 experts per wavefront.
// wave w: m-tile w % MT, n-tiles w / MT + (4 / MT) * j.
template <int MT, int NJ>
__global__ __launch_bounds__(NTH) void route_mfma_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ wg,
                                                         const float* __restrict__ bias, int T, int d, int E, int k,
                                                         int renorm, int32_t* __restrict__ idx_out,
                                                         float* __restrict__ w_out, float* __restrict__ logits_out) {
    constexpr int TB = 32 * MT;
    constexpr int NW = 4 / MT;              // wavefronts along the expert axis
    constexpr int EP = 32 * NW * NJ;        // padded expert count
    constexpr int PL = EP + 4;              // pitch of a logit row (floats)
    constexpr int TPT = NTH / TB;           // threads per token in the selection
    __shared__ __attribute__((aligned(16))) uint16_t xs[TB * PK];
    __shared__ __attribute__((aligned(16))) uint16_t wsT[EP * PK];
    __shared__ float ls[TB * PL];
    __shared__ float xn2[TB], wn2[EP];
    __shared__ int flag_tok[TB];
    __shared__ float flag_thr[TB], flag_max[TB], flag_den[TB];
    __shared__ int n_flag;
    // the exact path's candidate lists reuse the W_g tile, which is dead by then (48*EP <= 80*EP bytes)
    double (*cand_v)[EP] = reinterpret_cast<double (*)[EP]>(wsT);
    int (*cand_e)[EP] = reinterpret_cast<int (*)[EP]>(wsT + 4 * EP * 4);
    constexpr int CJ = (EP + 63) / 64;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, lhi = lane >> 5;
    const int wm = wave % MT, wn0 = wave / MT;
    const int t0 = blockIdx.x * TB;

    for (int i = tid; i < EP; i += NTH) wn2[i] = 0.f;
    if (tid == 0) n_flag = 0;

    double acc64[NJ][16];
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc64[j][r] = 0.0;
    float xsq = 0.f;

    // x staging: one 16-byte piece (8 terms) of one token per thread and chunk
    const int s_tok = tid >> 2, s_kk = (tid & 3) * 8;
    const bool s_on = s_tok < TB;
    const int s_t = t0 + s_tok;
    __syncthreads();

    // Register staging, one chunk ahead: the loads of chunk c+1 are in flight while chunk c is
    // multiplied.  W_g piece u of a thread is element (kk, e) = ((tid + u*NTH) / EP, (tid + u*NTH) % EP).
    constexpr int WN = KC * EP / NTH;
    u32x4 xv = {0u, 0u, 0u, 0u};
    uint16_t wv[WN];
    auto load_chunk = [&](int k0) {
        xv = (u32x4){0u, 0u, 0u, 0u};
        if (s_on && s_t < T && k0 + s_kk < d) xv = *(const u32x4*)(x + (size_t)s_t * d + k0 + s_kk);
#pragma unroll
        for (int u2 = 0; u2 < WN; ++u2) {
            const int i = tid + u2 * NTH, kk = i / EP, e = i % EP;
            wv[u2] = (e < E && k0 + kk < d) ? wg[(size_t)(k0 + kk) * E + e] : (uint16_t)0;
        }
    };
    load_chunk(0);

    for (int k0 = 0; k0 < d; k0 += KC) {
        if (s_on) {
            *(u32x4*)(xs + s_tok * PK + s_kk) = xv;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float lo = __uint_as_float(xv[i] << 16), hi = __uint_as_float(xv[i] & 0xffff0000u);
                xsq = fmaf(lo, lo, xsq);
                xsq = fmaf(hi, hi, xsq);
            }
        }
#pragma unroll
        for (int u2 = 0; u2 < WN; ++u2) {             // W_g chunk, transposed into LDS
            const int i = tid + u2 * NTH, kk = i / EP, e = i % EP;
            wsT[e * PK + kk] = wv[u2];
        }
        __syncthreads();
        if (k0 + KC < d) load_chunk(k0 + KC);
        if (tid < E) {                                   // column norms, fixed order
            float s = wn2[tid];
#pragma unroll 8
            for (int kk = 0; kk < KC; ++kk) { float v = bf16_to_f32(wsT[tid * PK + kk]); s = fmaf(v, v, s); }
            wn2[tid] = s;
        }
        f32x16 acc[NJ];
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KC / 16; ++ks) {
            const bf16x8 a = *(const bf16x8*)(xs + (wm * 32 + l32) * PK + ks * 16 + lhi * 8);
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                const bf16x8 b = *(const bf16x8*)(wsT + ((wn0 + NW * j) * 32 + l32) * PK + ks * 16 + lhi * 8);
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
            }
        }
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc64[j][r] += (double)acc[j][r];
        __syncthreads();
    }

    // ---- logits to LDS (fp32), token norms
    if (s_on) {
        xsq += __shfl_xor(xsq, 1);
        xsq += __shfl_xor(xsq, 2);
        if ((tid & 3) == 0) xn2[s_tok] = xsq;
    }
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const int e = (wn0 + NW * j) * 32 + l32;
        const double be = (bias && e < E) ? (double)bias[e] : 0.0;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int tok = wm * 32 + 8 * (r >> 2) + 4 * lhi + (r & 3);
            const float l = (float)(acc64[j][r] + be);
            if (e < E) {
                ls[tok * PL + e] = l;
                if (logits_out && t0 + tok < T) logits_out[(size_t)(t0 + tok) * E + e] = l;
            }
        }
    }
    __syncthreads();

    float wmax2 = 0.f, bmax = 0.f;
    for (int e = 0; e < E; ++e) wmax2 = fmaxf(wmax2, wn2[e]);      // broadcast reads
    if (bias) for (int e = 0; e < E; ++e) bmax = fmaxf(bmax, fabsf(bias[e]));
    const float wn_max = sqrtf(wmax2) * 1.0001f;
    const int rounds = (k + 1 < E) ? k + 1 : E;
    const float u = 5.9604645e-8f;   // 2^-24

    // ---- selection: TPT threads per token, thread `sub` scans experts sub, sub+TPT, ...
    {
        const int tok = tid / TPT, sub = tid % TPT, t = t0 + tok;
        const float* row = ls + tok * PL;
        float lv[MAXR];
        int le[MAXR];
#pragma unroll
        for (int r = 0; r < MAXR; ++r) { lv[r] = NEG_INF; le[r] = INT_MAX; }
        float m = NEG_INF;
        for (int e = sub; e < E; e += TPT) {
            float v = row[e];
            int ve = e;
            m = fmaxf(m, v);
            if (beats(v, ve, lv[MAXR - 1], le[MAXR - 1])) {     // sorted insertion, static indices
#pragma unroll
                for (int r = 0; r < MAXR; ++r) {
                    if (beats(v, ve, lv[r], le[r])) {
                        float tv = lv[r]; int te = le[r];
                        lv[r] = v; le[r] = ve;
                        v = tv; ve = te;
                    }
                }
            }
        }
        m = group_max<TPT>(m);
        float s = 0.f;
        for (int e = sub; e < E; e += TPT) s += __expf(row[e] - m);
        const float denom = group_sum<TPT>(s);
        float sel_v[MAXR];
        int sel_e[MAXR];
#pragma unroll
        for (int r = 0; r < MAXR; ++r) {
            sel_v[r] = NEG_INF; sel_e[r] = INT_MAX;
            if (r < rounds) {
                float bv = lv[0];
                int be = le[0];
                group_best<TPT>(bv, be);
                sel_v[r] = bv;
                sel_e[r] = be;
                if (le[0] == be) {                               // the winner's owner pops its head
#pragma unroll
                    for (int i = 0; i + 1 < MAXR; ++i) { lv[i] = lv[i + 1]; le[i] = le[i + 1]; }
                    lv[MAXR - 1] = NEG_INF; le[MAXR - 1] = INT_MAX;
                }
            }
        }
        const float xn = sqrtf(xn2[tok]) * 1.0001f;
        const float tau = 2.1f * u * ((2 * KC + 6) * xn * wn_max + bmax);
        bool near = false;
#pragma unroll
        for (int r = 0; r + 1 < MAXR; ++r)
            if (r + 1 < rounds && sel_v[r] - sel_v[r + 1] < tau) near = true;
        if (t < T && sub == 0) {
            if (!near) {
                float p[MOE_MAX_TOPK], tot = 0.f;
#pragma unroll
                for (int r = 0; r < MOE_MAX_TOPK; ++r)
                    if (r < k) { p[r] = __expf(sel_v[r] - m) / denom; tot += p[r]; }
#pragma unroll
                for (int r = 0; r < MOE_MAX_TOPK; ++r)
                    if (r < k) {
                        idx_out[(size_t)t * k + r] = sel_e[r];
                        w_out[(size_t)t * k + r] = renorm ? p[r] / tot : p[r];
                    }
            } else {
                float last = sel_v[0];
#pragma unroll
                for (int r = 1; r < MAXR; ++r) if (r < rounds) last = sel_v[r];
                const int f = atomicAdd(&n_flag, 1);
                flag_tok[f] = tok;
                flag_thr[f] = last - tau;
                flag_max[f] = m;
                flag_den[f] = denom;
            }
        }
    }
    __syncthreads();

    // ---- exact path for the flagged tokens: one wavefront per token
    const int nf = n_flag;
    for (int f = wave; f < nf; f += 4) {
        const int tok = flag_tok[f], t = t0 + tok;
        const float thr = flag_thr[f];
        const uint16_t* xr = x + (size_t)t * d;
        int nc = 0;
        for (int e0 = 0; e0 < E; e0 += 64) {
            const int e = e0 + lane;
            unsigned long long mask = __ballot(e < E && ls[tok * PL + e] >= thr);
            while (mask) {
                const int ce = e0 + (int)__builtin_ctzll(mask);
                mask &= mask - 1;
                double part = 0.0;
                for (int i = lane; i < d; i += 64)
                    part = fma((double)bf16_to_f32(xr[i]), (double)bf16_to_f32(wg[(size_t)i * E + ce]), part);
                const double tot = wave_sum_f64(part) + (bias ? (double)bias[ce] : 0.0);
                if (lane == 0) { cand_v[wave][nc] = tot; cand_e[wave][nc] = ce; }
                ++nc;
            }
        }
        // candidates back to lanes (c = lane + 64 j), then k rounds of arg-best in fp64
        double cv[CJ];
        int ce_[CJ];
#pragma unroll
        for (int j = 0; j < CJ; ++j) {
            const int c = lane + 64 * j;
            cv[j] = c < nc ? cand_v[wave][c] : -__builtin_huge_val();
            ce_[j] = c < nc ? cand_e[wave][c] : INT_MAX;
        }
        const double m = (double)flag_max[f], den = (double)flag_den[f];
        double p[MOE_MAX_TOPK], tot = 0.0;
        int pe[MOE_MAX_TOPK];
#pragma unroll
        for (int r = 0; r < MOE_MAX_TOPK; ++r) {
            if (r < k) {
                double bv = -__builtin_huge_val();
                int be = INT_MAX;
#pragma unroll
                for (int j = 0; j < CJ; ++j)
                    if (beats(cv[j], ce_[j], bv, be)) { bv = cv[j]; be = ce_[j]; }
                wave_best_f64(bv, be);
#pragma unroll
                for (int j = 0; j < CJ; ++j)
                    if (ce_[j] == be) { cv[j] = -__builtin_huge_val(); ce_[j] = INT_MAX; }
                p[r] = exp(bv - m) / den;
                pe[r] = be;
                tot += p[r];
            }
        }
        if (lane == 0) {
#pragma unroll
            for (int r = 0; r < MOE_MAX_TOPK; ++r)
                if (r < k) {
                    idx_out[(size_t)t * k + r] = pe[r];
                    w_out[(size_t)t * k + r] = (float)(renorm ? p[r] / tot : p[r]);
                }
        }
    }
}

template <int MT, int NJ>
int launch(const void* x, const void* wg, const float* bias, int T, int d, int E, int k, int renorm, int32_t* idx,
           float* w, float* logits, hipStream_t st) {
    constexpr int TB = 32 * MT;
    hipLaunchKernelGGL((route_mfma_kernel<MT, NJ>), dim3((T + TB - 1) / TB), dim3(NTH), 0, st, (const uint16_t*)x,
                       (const uint16_t*)wg, bias, T, d, E, k, renorm, idx, w, logits);
    MOE_CHECK_LAUNCH("moe_route_topk");
    return MOE_OK;
}

}  // namespace

// bf16 path of moe_route_topk (arguments already validated by the caller)
int moe_route_bf16_mfma(const void* x, const void* wg, const float* bias, int T, int d, int E, int k, int renorm,
                        int32_t* idx, float* w, float* logits, hipStream_t st) {
    if (E <= 64) return launch<2, 1>(x, wg, bias, T, d, E, k, renorm, idx, w, logits, st);
    if (E <= 128) return launch<2, 2>(x, wg, bias, T, d, E, k, renorm, idx, w, logits, st);
    return launch<1, 2>(x, wg, bias, T, d, E, k, renorm, idx, w, logits, st);
}
