// moe_route_topk for bf16 inputs: the router product on the matrix cores (Alg. 1 step 1).
//
// One work-group takes TB tokens (64, or 32 when E > 128).  Logits x.W_g are accumulated by
// v_mfma_f32_32x32x16_bf16 in chunks of 64 terms (bf16 x bf16 products are exact in fp32); each
// chunk's fp32 result is added into fp64 accumulators, so only the rounding inside a chunk
// counts: |error| <= c * |x_t| * |w_e| with c = (2*64+6) * 2^-24 (two roundings per term allowed
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
#include <type_traits>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int NTH = 256;
constexpr int KC = 64;                 // terms per fp32 chunk (four MFMAs)
constexpr int KACC = 256;              // prepared-router kernel: terms per fp32 accumulation
constexpr int PK = KC + 8;             // LDS pitch of a K-row in bf16 elements (144 B: conflict-free 16 B reads)
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
    __shared__ float xn2[TB], part[NTH], red_w[4], red_b[4];
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

    if (tid == 0) n_flag = 0;

    double acc64[NJ][16];
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc64[j][r] = 0.0;

    // Register staging, one chunk ahead: the loads of chunk c+1 are in flight while chunk c is
    // multiplied.  x: piece p = tid + u*NTH is 8 terms of token p / 8 at k offset (p % 8) * 8.
    // W_g: piece u is element (kk, e) = ((tid + u*NTH) / EP, tid % EP) -- always the same column,
    // so the column's sum of squares is kept in a register.
    constexpr int XN = TB * (KC / 8) / NTH;
    constexpr int WN = KC * EP / NTH;
    u32x4 xv[XN];
    uint16_t wv[WN];
    float xsq[XN], wsq = 0.f;
#pragma unroll
    for (int u2 = 0; u2 < XN; ++u2) xsq[u2] = 0.f;
    const int w_e = tid % EP, w_kk0 = tid / EP;
    auto load_chunk = [&](int k0) {
#pragma unroll
        for (int u2 = 0; u2 < XN; ++u2) {
            const int p = tid + u2 * NTH, tok = p >> 3, kk = (p & 7) * 8;
            xv[u2] = (u32x4){0u, 0u, 0u, 0u};
            if (t0 + tok < T && k0 + kk < d) xv[u2] = *(const u32x4*)(x + (size_t)(t0 + tok) * d + k0 + kk);
        }
#pragma unroll
        for (int u2 = 0; u2 < WN; ++u2) {
            const int kk = w_kk0 + u2 * (NTH / EP);
            wv[u2] = (w_e < E && k0 + kk < d) ? wg[(size_t)(k0 + kk) * E + w_e] : (uint16_t)0;
        }
    };
    // Work-groups start at different chunks: all of them reading the same 16 KB of W_g at the same
    // moment would queue on a few L2 channels.
    const int n_chunks = (d + KC - 1) / KC;
    int chunk = blockIdx.x % n_chunks;
    load_chunk(chunk * KC);
    __syncthreads();

    for (int c = 0; c < n_chunks; ++c) {
#pragma unroll
        for (int u2 = 0; u2 < XN; ++u2) {
            const int p = tid + u2 * NTH, tok = p >> 3, kk = (p & 7) * 8;
            *(u32x4*)(xs + tok * PK + kk) = xv[u2];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float lo = __uint_as_float(xv[u2][i] << 16), hi = __uint_as_float(xv[u2][i] & 0xffff0000u);
                xsq[u2] = fmaf(lo, lo, xsq[u2]);
                xsq[u2] = fmaf(hi, hi, xsq[u2]);
            }
        }
#pragma unroll
        for (int u2 = 0; u2 < WN; ++u2) {             // W_g chunk, transposed into LDS
            wsT[w_e * PK + w_kk0 + u2 * (NTH / EP)] = wv[u2];
            const float v = bf16_to_f32(wv[u2]);
            wsq = fmaf(v, v, wsq);
        }
        __syncthreads();
        chunk = chunk + 1 == n_chunks ? 0 : chunk + 1;
        if (c + 1 < n_chunks) load_chunk(chunk * KC);
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

    // ---- logits to LDS (fp32), token and column norms
#pragma unroll
    for (int u2 = 0; u2 < XN; ++u2) {              // the 8 threads of a token row are neighbours
        float v = xsq[u2];
        v += dpp_xchg<0>(v);
        v += dpp_xchg<1>(v);
        v += dpp_xchg<2>(v);
        if ((tid & 7) == 0) xn2[(tid + u2 * NTH) >> 3] = v;
    }
    part[tid] = wsq;
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

    {   // largest column norm and largest |bias|, reduced in parallel
        float w2 = 0.f, bm = 0.f;
        if (tid < E) {
#pragma unroll
            for (int j = 0; j < NTH / EP; ++j) w2 += part[tid + j * EP];
            if (bias) bm = fabsf(bias[tid]);
        }
        w2 = moe_wave_max_nonneg(w2);
        bm = moe_wave_max_nonneg(bm);
        if (lane == 0) { red_w[wave] = w2; red_b[wave] = bm; }
    }
    __syncthreads();
    const float wmax2 = fmaxf(fmaxf(red_w[0], red_w[1]), fmaxf(red_w[2], red_w[3]));
    const float bmax = fmaxf(fmaxf(red_b[0], red_b[1]), fmaxf(red_b[2], red_b[3]));
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
                double psum = 0.0;
                for (int i0 = lane; i0 < d; i0 += 64 * 8) {      // 16 loads in flight per lane
                    float xa[8], wa[8];
#pragma unroll
                    for (int u2 = 0; u2 < 8; ++u2) {
                        const int i = i0 + 64 * u2;
                        xa[u2] = i < d ? bf16_to_f32(xr[i]) : 0.f;
                        wa[u2] = i < d ? bf16_to_f32(wg[(size_t)i * E + ce]) : 0.f;
                    }
#pragma unroll
                    for (int u2 = 0; u2 < 8; ++u2) psum = fma((double)xa[u2], (double)wa[u2], psum);
                }
                const double tot = wave_sum_f64(psum) + (bias ? (double)bias[ce] : 0.0);
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


// =========================================================================================
// Router with a prepared W_g (moe_pack_router): W_g^T [E,d], so the contraction index is
// contiguous for both operands.  Both are staged through LDS by global -> LDS loads of whole
// 128-byte lines (a stage = 64 * KSP contraction terms of the 32 tokens and of all experts; three or
// four stages in flight, one barrier per stage), and the MFMA fragments are read from there.
// (Fetching the fragments straight from global memory, 16 bytes per lane, touched 32 lines per
// load for 32 bytes each and left the kernel waiting on the vector cache: 20 us of its 34 on
// 16384 tokens x 768.)
//
// One work-group = 32 tokens.  Its wavefronts split the experts into blocks of 32 (NB blocks)
// and, when there are fewer than four blocks, also the contraction (KSP parts): wavefront
// (block, part) takes the 64-term chunks part, part+KSP, ... for its 32 experts.  A wavefront's
// fp32 MFMA accumulator collects up to KACC terms before it is added into fp64 sums (same error
// model as above, with KACC-term chunks); the KSP partial sums are added in a fixed order
// through LDS.  The staging ring shares its LDS with the buffers of the later phases.
typedef __attribute__((ext_vector_type(4))) unsigned int frag_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((address_space(3))) void lds_void_t;
constexpr int ROUTE_RING = 3;          // stages of the prepared-router kernel's staging ring
// s_waitcnt on vmcnt only (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[15:14])
#define MOE_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 0xF) | (((n) >> 4) << 14) | (0x7 << 4) | (0xF << 8))

// (the body is a __device__ function: buffer-descriptor types exist on the device side only)
template <int NB, int KSP, int RMAX>   // expert blocks, contraction parts, depth of the top list (>= k + 1)
__device__ __forceinline__ void route_packed_body(const uint16_t* __restrict__ x, const uint16_t* __restrict__ wgt,
                                                  const float* __restrict__ w_norm2, const float* __restrict__ bias,
                                                  int T, int d, int E, int k, int renorm, int32_t* __restrict__ idx_out,
                                                  float* __restrict__ w_out, float* __restrict__ logits_out) {
    constexpr int NWV = NB * KSP, NTHR = NWV * 64, TB = 32, TPT = 8, EPT = 32 * NB;
    constexpr int PL = EPT + 4;                      // pitch of a logit row (floats)
    constexpr int SLAB = KSP > 1 ? KSP * TB * EPT * 8 : 0;
    constexpr int CAND = NWV * (MOE_MAX_EXPERTS + 32) * 12;
    constexpr int REGION0 = SLAB > CAND ? SLAB : CAND;
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    // LDS: fp64 slabs [KSP][32][EPT] for the sum over the contraction parts (later the exact path's
    // candidate lists), the fp32 logits [32][PL], partial token norms, flags
    double* slab = reinterpret_cast<double*>(smem);
    float* ls = reinterpret_cast<float*>(smem + REGION0);
    float* xn2p = ls + TB * PL;                      // [KSP][32]
    int* flag_tok = reinterpret_cast<int*>(xn2p + KSP * TB);
    float* flag_thr = reinterpret_cast<float*>(flag_tok + TB);
    float* flag_max = flag_thr + TB;
    float* flag_den = flag_max + TB;
    float* red = flag_den + TB;                      // [2 * NWV]
    int* n_flag = reinterpret_cast<int*>(red + 2 * NWV);

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, lhi = lane >> 5;
    const int nbi = wave / KSP, ksi = wave % KSP;    // this wavefront's expert block and contraction part
    const int t0 = blockIdx.x * TB;
    const int n_chunks = d / KC;
    const int rows = T - t0 < TB ? T - t0 : TB;
    float xsq = 0.f;

    double acc64[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) acc64[r] = 0.0;
    f32x16 acc;
    int in_acc = 0;
    auto clear_acc = [&]() {
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
        in_acc = 0;
    };
    auto flush_acc = [&]() {
#pragma unroll
        for (int r = 0; r < 16; ++r) acc64[r] += (double)acc[r];
        clear_acc();
    };
    clear_acc();

    // ---- staging.  Stage s holds the chunks s*KSP ... s*KSP+KSP-1: for each, 32 token rows, then
    // for each EPT expert rows, every row one 128-byte line (64 terms) in eight 16-byte pieces,
    // piece p of row r at position p ^ ((r / 2) & 7) (conflict-free fragment reads).  A load moves
    // eight rows (lane = row * 8 + position); the loads of a stage are dealt to the wavefronts,
    // every wavefront issues the same number (LPW) per stage -- the surplus ones, and all loads
    // past the last stage, with an empty descriptor -- so the count of outstanding loads that
    // guarantees a stage is a constant.
    constexpr int SROWS = (TB + EPT) * KSP, NL = SROWS / 8, LPW = (NL + NWV - 1) / NWV;
    constexpr int STAGE = SROWS * 128;
    constexpr int RING = ROUTE_RING;
    static_assert(LPW * (RING - 1) < 64 && RING * STAGE + 1024 <= 150 * 1024, "staging ring");
    unsigned char* ring = smem;
    unsigned char* dump = smem + RING * STAGE;               // 1 KB where the surplus loads' zeros go
    const int n_stages = (n_chunks + KSP - 1) / KSP;
    const __amdgpu_buffer_rsrc_t rx =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(x + (size_t)t0 * d), 0, rows * d * 2, 0x00020000);
    const __amdgpu_buffer_rsrc_t rw =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(wgt), 0, E * d * 2, 0x00020000);
    const __amdgpu_buffer_rsrc_t rnull = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(x), 0, 0, 0x00020000);
    const int ld_r = lane >> 3, ld_p = lane & 7;
    auto issue_stage = [&](int st) {
        unsigned char* buf = ring + (st % RING) * STAGE;
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const int L = wave + i * NWV;                    // (wave-uniform)
            const int R = L * 8;                             // first stage row of this load
            const int sub = R / (TB + EPT);                  // chunk of the stage
            const int rr = R - sub * (TB + EPT);             // row inside the chunk: tokens, then experts
            const int c = st * KSP + sub;
            const bool live = L < NL && st < n_stages && c < n_chunks;
            const bool is_x = rr < TB;
            const int row = (is_x ? rr : rr - TB) + ld_r;    // token of the tile / expert
            const unsigned voff = (unsigned)row * (unsigned)d * 2u + (unsigned)((ld_p ^ (((rr + ld_r) >> 1) & 7)) << 4);
            lds_void_t* to = (lds_void_t*)(L < NL ? buf + R * 128 : dump);
            const unsigned soff = (unsigned)c * 128u;
            // (three calls under wave-uniform branches: a descriptor chosen by a conditional
            // expression is kept in memory by the compiler and reloaded, with a full wait, per load)
            if (live && is_x) __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, to, 16, voff, soff, 0, 0);
            else if (live) __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, to, 16, voff, soff, 0, 0);
            else __builtin_amdgcn_raw_ptr_buffer_load_lds(rnull, to, 16, voff, soff, 0, 0);
        }
    };
#pragma unroll
    for (int st = 0; st < RING - 1; ++st) issue_stage(st);
    const int frag_at = l32 * 128;
    const int frag_sw = (l32 >> 1) & 7;
    for (int st = 0; st < n_stages; ++st) {
        // stage st has landed once only the RING-2 younger stages are outstanding
        if (RING == 4) MOE_WAIT_VMCNT(2 * LPW);
        else if (RING == 3) MOE_WAIT_VMCNT(LPW);
        else MOE_WAIT_VMCNT(0);
        // ... for every wavefront after the barrier; and stage st-1 has been read by all.  (A bare
        // barrier: __syncthreads would first wait for every load in flight, the prefetched stages too.)
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("" ::: "memory");
        issue_stage(st + RING - 1);                          // into the buffer of stage st-1
        const int c = st * KSP + ksi;
        if (c < n_chunks) {
            const unsigned char* xb = ring + (st % RING) * STAGE + ksi * (TB + EPT) * 128;
            const unsigned char* wb_ = xb + (TB + nbi * 32) * 128;
            frag_t xa[KC / 16], wb[KC / 16];
#pragma unroll
            for (int ks = 0; ks < KC / 16; ++ks) {
                const int pos = ((ks * 2 + lhi) ^ frag_sw) << 4;
                xa[ks] = *(const frag_t*)(xb + frag_at + pos);
                wb[ks] = *(const frag_t*)(wb_ + frag_at + pos);
            }
#pragma unroll
            for (int ks = 0; ks < KC / 16; ++ks) {
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, xa[ks]),
                                                              __builtin_bit_cast(bf16x8, wb[ks]), acc, 0, 0, 0);
                if (nbi == 0) {                              // the token norms, once per contraction part
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const bf16x2 p2 = __builtin_bit_cast(bf16x2, xa[ks][i]);
                        xsq = __builtin_amdgcn_fdot2_f32_bf16(p2, p2, xsq, false);
                    }
                }
            }
            if (++in_acc == KACC / KC) flush_acc();
        }
    }
    if (in_acc) flush_acc();
    MOE_WAIT_VMCNT(0);                                       // (the trailing empty loads still target this LDS)
    __syncthreads();                                         // the ring's memory is reused below
    if (tid == 0) *n_flag = 0;

    // ---- logits.  acc64[r]: token 8*(r/4) + 4*lhi + r%4, expert nbi*32 + l32.
    if (KSP > 1) {                                   // the partial sums of the contraction parts, fixed order
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int tok = 8 * (r >> 2) + 4 * lhi + (r & 3);
            slab[(ksi * TB + tok) * EPT + nbi * 32 + l32] = acc64[r];
        }
        __syncthreads();
        for (int i = tid; i < TB * EPT; i += NTHR) {
            const int tok = i / EPT, e = i % EPT;
            if (e < E) {
                double v = slab[i];
#pragma unroll
                for (int p = 1; p < KSP; ++p) v += slab[p * TB * EPT + i];
                const float l = (float)(v + (bias ? (double)bias[e] : 0.0));
                ls[tok * PL + e] = l;
                if (logits_out && t0 + tok < T) logits_out[(size_t)(t0 + tok) * E + e] = l;
            }
        }
    } else {
        const int e = nbi * 32 + l32;
        const double be = (bias && e < E) ? (double)bias[e] : 0.0;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int tok = 8 * (r >> 2) + 4 * lhi + (r & 3);
            const float l = (float)(acc64[r] + be);
            if (e < E) {
                ls[tok * PL + e] = l;
                if (logits_out && t0 + tok < T) logits_out[(size_t)(t0 + tok) * E + e] = l;
            }
        }
    }
    // token norms: the two k-halves of a token sit in lanes l and l+32; the parts are added in a fixed order
    xsq += __shfl_xor(xsq, 32);
    if (nbi == 0 && lhi == 0) xn2p[ksi * TB + l32] = xsq;
    {   // largest column norm and largest |bias|
        float w2 = 0.f, bm = 0.f;
        for (int e = tid; e < E; e += NTHR) {
            w2 = fmaxf(w2, w_norm2[e]);
            if (bias) bm = fmaxf(bm, fabsf(bias[e]));
        }
        w2 = moe_wave_max_nonneg(w2);
        bm = moe_wave_max_nonneg(bm);
        if (lane == 0) { red[wave] = w2; red[NWV + wave] = bm; }
    }
    __syncthreads();
    float wmax2 = 0.f, bmax = 0.f;
#pragma unroll
    for (int w2 = 0; w2 < NWV; ++w2) { wmax2 = fmaxf(wmax2, red[w2]); bmax = fmaxf(bmax, red[NWV + w2]); }
    const float wn_max = sqrtf(wmax2) * 1.0001f;
    const int rounds = (k + 1 < E) ? k + 1 : E;
    const float u = 5.9604645e-8f;   // 2^-24

    // ---- selection: TPT threads per token (the first four wavefronts); thread `sub` takes the CPT
    // consecutive experts from sub * CPT on, fetched with four-float reads before the scan (a read
    // per expert inside the scan made it wait for LDS at every step)
    if (tid < TB * TPT) {
        constexpr int CPT = EPT / TPT;
        static_assert(CPT % 4 == 0 && PL % 4 == 0, "four-float reads of a logit row");
        const int tok = tid / TPT, sub = tid % TPT, t = t0 + tok;
        const float* row = ls + tok * PL;
        float mine[CPT];
#pragma unroll
        for (int j = 0; j < CPT; j += 4) {
            const float4 q = *reinterpret_cast<const float4*>(row + sub * CPT + j);
            mine[j] = q.x; mine[j + 1] = q.y; mine[j + 2] = q.z; mine[j + 3] = q.w;
        }
        float lv[RMAX];
        int le[RMAX];
#pragma unroll
        for (int r = 0; r < RMAX; ++r) { lv[r] = NEG_INF; le[r] = INT_MAX; }
        float m = NEG_INF;
#pragma unroll
        for (int j = 0; j < CPT; ++j) {
            int ve = sub * CPT + j;
            float v = ve < E ? mine[j] : NEG_INF;                // (columns past E hold nothing)
            mine[j] = v;
            m = fmaxf(m, v);
            if (ve < E && beats(v, ve, lv[RMAX - 1], le[RMAX - 1])) {     // sorted insertion, static indices
#pragma unroll
                for (int r = 0; r < RMAX; ++r) {
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
#pragma unroll
        for (int j = 0; j < CPT; ++j) s += sub * CPT + j < E ? __expf(mine[j] - m) : 0.f;
        const float denom = group_sum<TPT>(s);
        float sel_v[RMAX];
        int sel_e[RMAX];
#pragma unroll
        for (int r = 0; r < RMAX; ++r) {
            sel_v[r] = NEG_INF; sel_e[r] = INT_MAX;
            if (r < rounds) {
                float bv = lv[0];
                int be = le[0];
                group_best<TPT>(bv, be);
                sel_v[r] = bv;
                sel_e[r] = be;
                if (le[0] == be) {                               // the winner's owner pops its head
#pragma unroll
                    for (int i = 0; i + 1 < RMAX; ++i) { lv[i] = lv[i + 1]; le[i] = le[i + 1]; }
                    lv[RMAX - 1] = NEG_INF; le[RMAX - 1] = INT_MAX;
                }
            }
        }
        float xs2 = xn2p[tok];
#pragma unroll
        for (int p = 1; p < KSP; ++p) xs2 += xn2p[p * TB + tok];
        const float xn = sqrtf(xs2) * 1.0001f;
        const float tau = 2.1f * u * ((2 * KACC + 6) * xn * wn_max + bmax);
        bool near = false;
#pragma unroll
        for (int r = 0; r + 1 < RMAX; ++r)
            if (r + 1 < rounds && sel_v[r] - sel_v[r + 1] < tau) near = true;
        if (t < T && sub == 0) {
            if (!near) {
                float p[RMAX], tot = 0.f;
#pragma unroll
                for (int r = 0; r < RMAX; ++r)
                    if (r < k) { p[r] = __expf(sel_v[r] - m) / denom; tot += p[r]; }
#pragma unroll
                for (int r = 0; r < RMAX; ++r)
                    if (r < k) {
                        idx_out[(size_t)t * k + r] = sel_e[r];
                        w_out[(size_t)t * k + r] = renorm ? p[r] / tot : p[r];
                    }
            } else {
                float last = sel_v[0];
#pragma unroll
                for (int r = 1; r < RMAX; ++r) if (r < rounds) last = sel_v[r];
                const int f = atomicAdd(n_flag, 1);
                flag_tok[f] = tok;
                flag_thr[f] = last - tau;
                flag_max[f] = m;
                flag_den[f] = denom;
            }
        }
    }
    __syncthreads();

    // ---- exact path for the flagged tokens: one wavefront per token; every expert whose fp32
    // logit could still reach the top k is recomputed in fp64 (both operand rows are contiguous)
    double* cand_v = slab + wave * (MOE_MAX_EXPERTS + 32);                       // [NWV][288] doubles ...
    int* cand_e = reinterpret_cast<int*>(slab + NWV * (MOE_MAX_EXPERTS + 32)) + wave * (MOE_MAX_EXPERTS + 32);   // ... then ints
    constexpr int CJ = (MOE_MAX_EXPERTS + 63) / 64;
    const int nf = *n_flag;
    for (int f = wave; f < nf; f += NWV) {
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
                const uint16_t* wr = wgt + (size_t)ce * d;
                double psum = 0.0;
                for (int i0 = lane * 8; i0 < d; i0 += 64 * 8) {    // 8 terms per lane and step, 16-byte loads
                    const frag_t xv = *(const frag_t*)(xr + i0), wv = *(const frag_t*)(wr + i0);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        psum = fma((double)__uint_as_float(xv[i] << 16), (double)__uint_as_float(wv[i] << 16), psum);
                        psum = fma((double)__uint_as_float(xv[i] & 0xffff0000u), (double)__uint_as_float(wv[i] & 0xffff0000u), psum);
                    }
                }
                const double tot = wave_sum_f64(psum) + (bias ? (double)bias[ce] : 0.0);
                if (lane == 0) { cand_v[nc] = tot; cand_e[nc] = ce; }
                ++nc;
            }
        }
        double cv[CJ];
        int ce_[CJ];
#pragma unroll
        for (int j = 0; j < CJ; ++j) {
            const int c = lane + 64 * j;
            cv[j] = c < nc ? cand_v[c] : -__builtin_huge_val();
            ce_[j] = c < nc ? cand_e[c] : INT_MAX;
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

template <int NB, int KSP, int RMAX>
__global__ __launch_bounds__(NB * KSP * 64, 2) void route_packed_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ wgt,
                                                                        const float* __restrict__ w_norm2,
                                                                        const float* __restrict__ bias, int T, int d, int E, int k,
                                                                        int renorm, int32_t* __restrict__ idx_out,
                                                                        float* __restrict__ w_out, float* __restrict__ logits_out) {
    route_packed_body<NB, KSP, RMAX>(x, wgt, w_norm2, bias, T, d, E, k, renorm, idx_out, w_out, logits_out);
}

template <int NB, int KSP, int RMAX>
int launch_packed_r(const void* x, const void* wgt, const float* w_norm2, const float* bias, int T, int d, int E, int k,
                    int renorm, int32_t* idx, float* w, float* logits, hipStream_t st) {
    constexpr int NWV = NB * KSP, EPT = 32 * NB;
    constexpr size_t slab = KSP > 1 ? (size_t)KSP * 32 * EPT * 8 : 0, cand = (size_t)NWV * (MOE_MAX_EXPERTS + 32) * 12;
    const size_t later = (slab > cand ? slab : cand) + (size_t)32 * (EPT + 4) * 4 + KSP * 32 * 4 + 4 * 32 * 4 + 2 * NWV * 4 + 16;
    const size_t ring = (size_t)ROUTE_RING * (32 + EPT) * KSP * 128 + 1024;       // the staging ring and the later buffers share LDS
    const size_t smem = ring > later ? ring : later;
    auto kern = route_packed_kernel<NB, KSP, RMAX>;
    if (smem > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return moe_fail(MOE_ERR_HIP, "moe_route_topk_packed: shared memory attribute: %s", hipGetErrorString(e));
    }
    hipLaunchKernelGGL(kern, dim3((T + 31) / 32), dim3(NWV * 64), smem, st, (const uint16_t*)x, (const uint16_t*)wgt, w_norm2,
                       bias, T, d, E, k, renorm, idx, w, logits);
    MOE_CHECK_LAUNCH("moe_route_topk_packed");
    return MOE_OK;
}

template <int NB, int KSP>
int launch_packed(const void* x, const void* wgt, const float* w_norm2, const float* bias, int T, int d, int E, int k,
                  int renorm, int32_t* idx, float* w, float* logits, hipStream_t st) {
    // the depth of the per-thread top list follows k (a shorter list is less work per logit)
    if (k <= 1) return launch_packed_r<NB, KSP, 2>(x, wgt, w_norm2, bias, T, d, E, k, renorm, idx, w, logits, st);
    if (k <= 2) return launch_packed_r<NB, KSP, 3>(x, wgt, w_norm2, bias, T, d, E, k, renorm, idx, w, logits, st);
    if (k <= 4) return launch_packed_r<NB, KSP, 5>(x, wgt, w_norm2, bias, T, d, E, k, renorm, idx, w, logits, st);
    return launch_packed_r<NB, KSP, MAXR>(x, wgt, w_norm2, bias, T, d, E, k, renorm, idx, w, logits, st);
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
    // 32 tokens per work-group: twice the work-groups, so that two or three share a CU and hide
    // each other's load latency
    if (E <= 128) return launch<1, 1>(x, wg, bias, T, d, E, k, renorm, idx, w, logits, st);
    return launch<1, 2>(x, wg, bias, T, d, E, k, renorm, idx, w, logits, st);
}

// bf16 path of moe_route_topk_packed (arguments already validated by the caller)
int moe_route_bf16_packed(const void* x, const void* wgt, const float* w_norm2, const float* bias, int T, int d, int E,
                          int k, int renorm, int32_t* idx, float* w, float* logits, hipStream_t st) {
    if (E <= 32) return launch_packed<1, 4>(x, wgt, w_norm2, bias, T, d, E, k, renorm, idx, w, logits, st);
    if (E <= 64) return launch_packed<2, 2>(x, wgt, w_norm2, bias, T, d, E, k, renorm, idx, w, logits, st);
    if (E <= 128) return launch_packed<4, 1>(x, wgt, w_norm2, bias, T, d, E, k, renorm, idx, w, logits, st);
    return launch_packed<8, 1>(x, wgt, w_norm2, bias, T, d, E, k, renorm, idx, w, logits, st);
}
