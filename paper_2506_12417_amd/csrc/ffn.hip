// moe_grouped_ffn: the expert FFNs over rows grouped by expert (Alg. 1 step 5; section 2: two
// dense layers with an activation between; section 4.4: x W1 W2, no biases).
//
// Two grouped GEMMs, each one persistent launch driven by the tile table of moe_plan_tiles:
//   G1  H = act(x_perm . W_in^T)     (ReLU, or SiLU(gate)*up on interleaved gate/up rows)
//   G2  y_perm = H . W_out^T         (fp32 out)
// bf16 runs on the matrix cores (ffn_bf16.hip); this file holds the entry points and the fp32
// kernel, a plain FMA tile kernel used by the small fp32 configuration.
#include "common.h"
#include "ffn_kernels.h"

namespace {

constexpr int EPI_RELU = MOE_EPI_RELU, EPI_SWIGLU = MOE_EPI_SWIGLU, EPI_STORE = MOE_EPI_STORE;

struct WorkList {
    int bin_start, n_tiles, stride, first;
};
__device__ __forceinline__ WorkList work_list(const int32_t* __restrict__ hdr) {
    WorkList w;
    const int G = hdr[1];
    const int bin = blockIdx.x % G;
    w.first = blockIdx.x / G;
    w.stride = ((int)gridDim.x - bin + G - 1) / G;
    w.bin_start = hdr[4 + bin];
    w.n_tiles = hdr[4 + bin + 1] - w.bin_start;
    return w;
}

__device__ __forceinline__ float silu_f(float z) { return z / (1.f + __expf(-z)); }

// =============================================================================== fp32 / FMA
constexpr int FM = 64, FN = 64, FK = 16;

template <int EPI>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ a_mat, int K, int N,
                                                       const void* const* __restrict__ w_ptrs,
                                                       const moe_tile* __restrict__ tiles,
                                                       const int32_t* __restrict__ hdr, float* __restrict__ out,
                                                       int ld_out) {
    __shared__ float As[FK][FM + 4];
    __shared__ float Bs[FK][FN + 4];
    __shared__ float Cs[EPI == EPI_SWIGLU ? FM : 1][FN + 1];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int ld_row = tid >> 2, ld_k = (tid & 3) * 4;
    const int n_col_blocks = (N + FN - 1) / FN;

    const WorkList wl = work_list(hdr);
    const int n_items = wl.n_tiles * n_col_blocks;
    for (int item = wl.first; item < n_items; item += wl.stride) {
        const int cb = item / wl.n_tiles;
        const moe_tile tile = tiles[wl.bin_start + (item - cb * wl.n_tiles)];
        const int rc = tile.row_count;
        if (rc <= 0) continue;
        const int n0 = cb * FN;
        const float* __restrict__ wmat = (const float*)w_ptrs[tile.expert];
        const float* a_src = a_mat + (size_t)(tile.row_begin + (ld_row < rc ? ld_row : rc - 1)) * K;
        const float* b_src = wmat + (size_t)(n0 + ld_row < N ? n0 + ld_row : N - 1) * K;
        float acc[4][4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
        for (int k0 = 0; k0 < K; k0 += FK) {
            float4 av = make_float4(0.f, 0.f, 0.f, 0.f), bv = av;
            if (k0 + ld_k < K) {
                av = *(const float4*)(a_src + k0 + ld_k);
                bv = *(const float4*)(b_src + k0 + ld_k);
            }
            __syncthreads();
            As[ld_k + 0][ld_row] = av.x; As[ld_k + 1][ld_row] = av.y; As[ld_k + 2][ld_row] = av.z; As[ld_k + 3][ld_row] = av.w;
            Bs[ld_k + 0][ld_row] = bv.x; Bs[ld_k + 1][ld_row] = bv.y; Bs[ld_k + 2][ld_row] = bv.z; Bs[ld_k + 3][ld_row] = bv.w;
            __syncthreads();
#pragma unroll
            for (int kk = 0; kk < FK; ++kk) {
                float a[4], b[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
                for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
            }
        }
        if (EPI == EPI_SWIGLU) {
            __syncthreads();
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) Cs[ty * 4 + i][tx * 4 + j] = acc[i][j];
            __syncthreads();
            // packed columns [0,32) of the block are gate, [32,64) the matching up columns
            for (int i = tid; i < FM * 32; i += 256) {
                int row = i >> 5, c = i & 31;
                if (row < rc && n0 + c < N)
                    out[(size_t)(tile.row_begin + row) * ld_out + n0 / 2 + c] = silu_f(Cs[row][c]) * Cs[row][32 + c];
            }
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                int row = ty * 4 + i;
                if (row >= rc) continue;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    int col = n0 + tx * 4 + j;
                    if (col < N) {
                        float v = acc[i][j];
                        out[(size_t)(tile.row_begin + row) * ld_out + col] = (EPI == EPI_RELU) ? fmaxf(v, 0.f) : v;
                    }
                }
            }
        }
    }
}

constexpr int GRID_F32 = 512;

}  // namespace

extern "C" int moe_ffn_tile_m(moe_dtype dt) { return dt == MOE_BF16 ? 128 : FM; }

// bf16 has two tile heights: 256 rows pay off when the experts hold many rows each
extern "C" int moe_ffn_pick_tile_m(moe_dtype dt, int A, int E) {
    if (dt != MOE_BF16) return FM;
    return (E >= 1 && A / E >= 1024) ? 256 : 128;
}

// top1: step 6 folded into the second product (perm: output row of every row; gate_w may be null)
struct Top1 {
    const int32_t* perm = nullptr;
    const float* gate_w = nullptr;
    bool on = false;
};
// gather: step 4's row gather folded into the first product (x [x_rows, d]; row r is x[perm[r] / k])
struct Gather {
    const int32_t* perm = nullptr;
    int x_rows = 0, k = 1;
    bool on = false;
};

// which 16-bit kernels run the 128-row configuration: 0 the default (the LDS-ring kernels), 1 the
// LDS-ring kernels, 2 the register-streaming kernels wherever they cover the call
static int g_kernel_mode = 0;

extern "C" int moe_ffn_kernel_mode(int mode) {
    MOE_REQUIRE(mode >= -1 && mode <= 2, MOE_ERR_ARG, "moe_ffn_kernel_mode: mode %d", mode);
    const int before = g_kernel_mode;
    if (mode >= 0) g_kernel_mode = mode;
    return before;
}

static int grouped_ffn_impl(int phases, const void* x_perm, int A, int d, int F, int E, moe_act act, moe_dtype dt,
                            const void* const* w_in, const void* const* w_out, const moe_tile* tiles,
                            int32_t* plan_hdr, int tile_m, void* h_scratch, float* y_perm, void* stream,
                            const Top1& top1 = Top1(), const Gather& gather = Gather()) {
    MOE_REQUIRE(moe_dtype_ok(dt), MOE_ERR_UNSUPPORTED, "moe_grouped_ffn: dtype %d", (int)dt);
    MOE_REQUIRE(act == MOE_RELU || act == MOE_SWIGLU, MOE_ERR_UNSUPPORTED, "moe_grouped_ffn: activation %d", (int)act);
    MOE_REQUIRE(A >= 0 && d >= 1 && F >= 1 && E >= 1, MOE_ERR_ARG, "moe_grouped_ffn: A=%d d=%d F=%d E=%d", A, d, F, E);
    if (dt == MOE_BF16) {
        MOE_REQUIRE(tile_m == 128 || tile_m == 256, MOE_ERR_UNSUPPORTED, "moe_grouped_ffn: bf16 tile_m=%d, must be 128 or 256", tile_m);
        MOE_REQUIRE(d % 64 == 0 && F % 64 == 0, MOE_ERR_UNSUPPORTED, "moe_grouped_ffn: bf16 needs d and F multiples of 64 (d=%d F=%d)", d, F);
    } else {
        MOE_REQUIRE(tile_m == FM, MOE_ERR_UNSUPPORTED, "moe_grouped_ffn: fp32 tile_m=%d, the kernel's is %d", tile_m, FM);
        MOE_REQUIRE(d % 4 == 0 && F % 4 == 0 && (act != MOE_SWIGLU || F % 32 == 0), MOE_ERR_UNSUPPORTED,
                    "moe_grouped_ffn: fp32 needs d and F multiples of 4 (32 for SwiGLU) (d=%d F=%d)", d, F);
    }
    if (A == 0) return MOE_OK;
    MOE_REQUIRE(tiles && plan_hdr && h_scratch, MOE_ERR_ARG, "moe_grouped_ffn: null pointer");
    MOE_REQUIRE(!(phases & 1) || (x_perm && w_in), MOE_ERR_ARG, "moe_grouped_ffn: null pointer");
    MOE_REQUIRE(!(phases & 2) || (y_perm && w_out), MOE_ERR_ARG, "moe_grouped_ffn: null pointer");
    hipStream_t st = (hipStream_t)stream;
    const int n1 = act == MOE_SWIGLU ? 2 * F : F;
    int rc;
    if (dt == MOE_BF16) {
        // Work items are (tile, column block), handed to the work-groups as they become free.
        // Wide column blocks read an activation tile fewer times; only when there would not be
        // two items per CU does a GEMM take narrower ones.  The number of tiles is known on the
        // device only; this is its expected value.
        const long long tiles_est = (A + tile_m - 1) / tile_m + E / 2;
        auto narrow = [&](int N) { return tile_m == 128 && tiles_est * ((N + 255) / 256) < 2 * MOE_GEMM_GRID; };
        // The kernels that stream the weights into registers (ffn_stream.hip) run on request only
        // (moe_ffn_kernel_mode 2): on the workloads measured so far the LDS-ring kernels are faster.
        // They take items of 128 weight rows, two work-groups per CU, unless there are four wide
        // items per CU.
        const bool few_rows = tile_m == 128 && g_kernel_mode == 2;
        auto stream = [&](int epi, int K) { return few_rows && moe_gemm_stream_supports(epi, K); };
        auto stream_narrow = [&](int N) { return tiles_est * ((N + 255) / 256) < 4 * MOE_GEMM_GRID; };
        // 256-row tiles (many rows per expert: the arithmetic-bound case) go to the four-wavefront
        // kernels of ffn_wide.hip unless the LDS-ring kernels are asked for (moe_ffn_kernel_mode 1).
        auto wide = [&](int epi, int K) { return tile_m == 256 && g_kernel_mode != 1 && moe_gemm_wide_supports(epi, K); };
        if (phases & 1) {
            const int epi = act == MOE_SWIGLU ? MOE_EPI_SWIGLU : MOE_EPI_RELU;
            if (gather.on && stream(epi, d))
                rc = moe_launch_gemm_stream_gather(stream_narrow(n1), x_perm, gather.x_rows, d, n1, w_in, tiles, plan_hdr,
                                                   h_scratch, F, st, gather.perm, gather.k);
            else if (gather.on && tile_m == 256)
                // (fused_impl has checked that the four-wavefront kernels are in use and cover d)
                rc = moe_launch_gemm_wide_gather(epi, x_perm, gather.x_rows, d, n1, w_in, tiles, plan_hdr, h_scratch, F, st,
                                                 gather.perm, gather.k);
            else if (gather.on)
                rc = moe_launch_gemm_bf16_gather(epi, x_perm, gather.x_rows, d, n1,
                                                 w_in, tiles, plan_hdr, h_scratch, F, st, gather.perm, gather.k);
            else if (stream(epi, d))
                rc = moe_launch_gemm_stream(epi, stream_narrow(n1), x_perm, d, n1, w_in, tiles, plan_hdr, h_scratch, F, st);
            else if (wide(epi, d))
                rc = moe_launch_gemm_wide(epi, x_perm, d, n1, w_in, tiles, plan_hdr, h_scratch, F, st);
            else
                rc = moe_launch_gemm_bf16(epi, tile_m, narrow(n1), x_perm, d, n1,
                                          w_in, tiles, plan_hdr, h_scratch, F, st);
            if (rc != MOE_OK) return rc;
        }
        if (phases & 2) {
            const int epi = top1.on ? MOE_EPI_SCATTER : MOE_EPI_STORE;
            if (stream(epi, F))
                rc = moe_launch_gemm_stream(epi, stream_narrow(d), h_scratch, F, d, w_out, tiles, plan_hdr, (void*)y_perm, d, st,
                                            top1.perm, top1.gate_w, top1.on ? A : 0);
            else if (wide(epi, F))
                rc = moe_launch_gemm_wide(epi, h_scratch, F, d, w_out, tiles, plan_hdr, (void*)y_perm, d, st, top1.perm,
                                          top1.gate_w, top1.on ? A : 0);
            else if (top1.on)
                rc = moe_launch_gemm_bf16(MOE_EPI_SCATTER, tile_m, narrow(d), h_scratch, F, d, w_out, tiles, plan_hdr,
                                          (void*)y_perm, d, st, top1.perm, top1.gate_w, A);
            else
                rc = moe_launch_gemm_bf16(MOE_EPI_STORE, tile_m, narrow(d), h_scratch, F, d, w_out, tiles, plan_hdr,
                                          (void*)y_perm, d, st);
            if (rc != MOE_OK) return rc;
        }
    } else {
        if (phases & 1) {
            if (act == MOE_SWIGLU)
                hipLaunchKernelGGL(gemm_f32_kernel<EPI_SWIGLU>, dim3(GRID_F32), dim3(256), 0, st, (const float*)x_perm, d,
                                   n1, w_in, tiles, plan_hdr, (float*)h_scratch, F);
            else
                hipLaunchKernelGGL(gemm_f32_kernel<EPI_RELU>, dim3(GRID_F32), dim3(256), 0, st, (const float*)x_perm, d,
                                   n1, w_in, tiles, plan_hdr, (float*)h_scratch, F);
            MOE_CHECK_LAUNCH("moe_grouped_ffn/G1");
        }
        if (phases & 2) {
            hipLaunchKernelGGL(gemm_f32_kernel<EPI_STORE>, dim3(GRID_F32), dim3(256), 0, st, (const float*)h_scratch, F,
                               d, w_out, tiles, plan_hdr, y_perm, d);
            MOE_CHECK_LAUNCH("moe_grouped_ffn/G2");
        }
    }
    return MOE_OK;
}

extern "C" int moe_grouped_ffn(const void* x_perm, int A, int d, int F, int E, moe_act act, moe_dtype dt,
                               const void* const* w_in, const void* const* w_out, const moe_tile* tiles,
                               int32_t* plan_hdr, int tile_m, void* h_scratch, float* y_perm, void* stream) {
    return grouped_ffn_impl(3, x_perm, A, d, F, E, act, dt, w_in, w_out, tiles, plan_hdr, tile_m, h_scratch, y_perm, stream);
}

extern "C" int moe_grouped_ffn_phase(int phase, const void* x_perm, int A, int d, int F, int E, moe_act act,
                                     moe_dtype dt, const void* const* w_in, const void* const* w_out,
                                     const moe_tile* tiles, int32_t* plan_hdr, int tile_m, void* h_scratch,
                                     float* y_perm, void* stream) {
    MOE_REQUIRE(phase == 1 || phase == 2, MOE_ERR_ARG, "moe_grouped_ffn_phase: phase %d", phase);
    return grouped_ffn_impl(phase, x_perm, A, d, F, E, act, dt, w_in, w_out, tiles, plan_hdr, tile_m, h_scratch, y_perm, stream);
}

static int top1_impl(int phases, const void* x_perm, int T, int d, int F, int E, moe_act act, moe_dtype dt,
                     const void* const* w_in, const void* const* w_out, const moe_tile* tiles, int32_t* plan_hdr,
                     int tile_m, void* h_scratch, const int32_t* perm, const float* gate_w, float* y, void* stream) {
    MOE_REQUIRE(dt == MOE_BF16, MOE_ERR_UNSUPPORTED, "moe_grouped_ffn_top1: MOE_BF16 only (dtype %d)", (int)dt);
    MOE_REQUIRE(F >= 512, MOE_ERR_UNSUPPORTED, "moe_grouped_ffn_top1: needs F >= 512 (F=%d)", F);
    MOE_REQUIRE(T == 0 || !(phases & 2) || (perm && y), MOE_ERR_ARG, "moe_grouped_ffn_top1: null pointer");
    MOE_REQUIRE((long long)T * d * 4 < (1ll << 31), MOE_ERR_UNSUPPORTED, "moe_grouped_ffn_top1: y must be smaller than 2 GiB (T=%d d=%d)", T, d);
    Top1 t;
    t.perm = perm;
    t.gate_w = gate_w;
    t.on = true;
    return grouped_ffn_impl(phases, x_perm, T, d, F, E, act, dt, w_in, w_out, tiles, plan_hdr, tile_m, h_scratch, y, stream, t);
}

extern "C" int moe_grouped_ffn_top1(const void* x_perm, int T, int d, int F, int E, moe_act act, moe_dtype dt,
                                    const void* const* w_in, const void* const* w_out, const moe_tile* tiles,
                                    int32_t* plan_hdr, int tile_m, void* h_scratch, const int32_t* perm,
                                    const float* gate_w, float* y, void* stream) {
    return top1_impl(3, x_perm, T, d, F, E, act, dt, w_in, w_out, tiles, plan_hdr, tile_m, h_scratch, perm, gate_w, y, stream);
}

extern "C" int moe_grouped_ffn_top1_phase(int phase, const void* x_perm, int T, int d, int F, int E, moe_act act,
                                          moe_dtype dt, const void* const* w_in, const void* const* w_out,
                                          const moe_tile* tiles, int32_t* plan_hdr, int tile_m, void* h_scratch,
                                          const int32_t* perm, const float* gate_w, float* y, void* stream) {
    MOE_REQUIRE(phase == 1 || phase == 2, MOE_ERR_ARG, "moe_grouped_ffn_top1_phase: phase %d", phase);
    return top1_impl(phase, x_perm, T, d, F, E, act, dt, w_in, w_out, tiles, plan_hdr, tile_m, h_scratch, perm, gate_w, y, stream);
}

static int fused_impl(int phases, const void* x, int T, int d, int F, int E, int k, moe_act act, moe_dtype dt,
                      const void* const* w_in, const void* const* w_out, const moe_tile* tiles, int32_t* plan_hdr,
                      int tile_m, void* h_scratch, const int32_t* perm, const float* gate_w, float* y_out, void* stream) {
    MOE_REQUIRE(dt == MOE_BF16, MOE_ERR_UNSUPPORTED, "moe_grouped_ffn_fused: MOE_BF16 only (dtype %d)", (int)dt);
    MOE_REQUIRE(T >= 0 && k >= 1, MOE_ERR_ARG, "moe_grouped_ffn_fused: T=%d k=%d", T, k);
    MOE_REQUIRE((long long)T * k < (1ll << 30), MOE_ERR_UNSUPPORTED, "moe_grouped_ffn_fused: T*k too large");
    MOE_REQUIRE(tile_m == 128 || tile_m == 256, MOE_ERR_UNSUPPORTED, "moe_grouped_ffn_fused: bf16 tile_m=%d, must be 128 or 256", tile_m);
    MOE_REQUIRE(tile_m == 128 || (g_kernel_mode != 1 && moe_gemm_wide_supports(MOE_EPI_RELU, d)), MOE_ERR_UNSUPPORTED,
                "moe_grouped_ffn_fused: with 256-row tiles the row gather is done by the four-wavefront kernels only "
                "(moe_ffn_kernel_mode %d, d=%d)", g_kernel_mode, d);
    MOE_REQUIRE(d >= 256, MOE_ERR_UNSUPPORTED, "moe_grouped_ffn_fused: needs d >= 256 (d=%d)", d);
    MOE_REQUIRE((long long)T * d * 2 < (1ll << 32), MOE_ERR_UNSUPPORTED, "moe_grouped_ffn_fused: x must be smaller than 4 GiB (T=%d d=%d)", T, d);
    MOE_REQUIRE(T == 0 || perm, MOE_ERR_ARG, "moe_grouped_ffn_fused: null pointer");
    Gather g;
    g.perm = perm;
    g.x_rows = T;
    g.k = k;
    g.on = true;
    if (k == 1) {
        MOE_REQUIRE(F >= 512, MOE_ERR_UNSUPPORTED, "moe_grouped_ffn_fused: top-1 needs F >= 512 (F=%d)", F);
        MOE_REQUIRE(T == 0 || !(phases & 2) || y_out, MOE_ERR_ARG, "moe_grouped_ffn_fused: null pointer");
        MOE_REQUIRE((long long)T * d * 4 < (1ll << 31), MOE_ERR_UNSUPPORTED, "moe_grouped_ffn_fused: y must be smaller than 2 GiB (T=%d d=%d)", T, d);
        Top1 t;
        t.perm = perm;
        t.gate_w = gate_w;
        t.on = true;
        return grouped_ffn_impl(phases, x, T, d, F, E, act, dt, w_in, w_out, tiles, plan_hdr, tile_m, h_scratch, y_out, stream, t, g);
    }
    return grouped_ffn_impl(phases, x, T * k, d, F, E, act, dt, w_in, w_out, tiles, plan_hdr, tile_m, h_scratch, y_out, stream, Top1(), g);
}

extern "C" int moe_grouped_ffn_fused(const void* x, int T, int d, int F, int E, int k, moe_act act, moe_dtype dt,
                                     const void* const* w_in, const void* const* w_out, const moe_tile* tiles,
                                     int32_t* plan_hdr, int tile_m, void* h_scratch, const int32_t* perm,
                                     const float* gate_w, float* y_out, void* stream) {
    return fused_impl(3, x, T, d, F, E, k, act, dt, w_in, w_out, tiles, plan_hdr, tile_m, h_scratch, perm, gate_w, y_out, stream);
}

extern "C" int moe_grouped_ffn_fused_phase(int phase, const void* x, int T, int d, int F, int E, int k, moe_act act,
                                           moe_dtype dt, const void* const* w_in, const void* const* w_out,
                                           const moe_tile* tiles, int32_t* plan_hdr, int tile_m, void* h_scratch,
                                           const int32_t* perm, const float* gate_w, float* y_out, void* stream) {
    MOE_REQUIRE(phase == 1 || phase == 2, MOE_ERR_ARG, "moe_grouped_ffn_fused_phase: phase %d", phase);
    return fused_impl(phase, x, T, d, F, E, k, act, dt, w_in, w_out, tiles, plan_hdr, tile_m, h_scratch, perm, gate_w, y_out, stream);
}
