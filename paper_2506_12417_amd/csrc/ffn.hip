// moe_grouped_ffn: the expert FFNs over rows grouped by expert (Alg. 1 step 5; section 2: two
// dense layers with an activation between; section 4.4: x W1 W2, no biases).
//
// Two grouped GEMMs, each one persistent launch driven by the tile table of moe_plan_tiles:
//   G1  H = act(x_perm . W_in^T)     (ReLU, or SiLU(gate)*up on interleaved gate/up rows)
//   G2  y_perm = H . W_out^T         (fp32 out)
// Work-group b serves bin b % n_bins -- work-groups are dealt round-robin to the 8 XCDs, so a
// bin's tiles, and with them an expert's weights, stay inside one XCD's L2.  Inside a bin the
// work items (tile, column block) are taken column-block-major with a fixed stride, so the
// work-groups of an XCD sweep the same weight columns over consecutive row tiles.
//
// bf16: 128x128 output tile per work-group, K step 64, 4 wavefronts in 2x2, each 64x64 as 2x2
// v_mfma_f32_32x32x16_bf16 blocks; operands staged through double-buffered LDS with a padded
// row pitch (144 B) that keeps the 16-byte operand reads conflict-free; global loads of the next
// K step are in flight while the current one is multiplied.  fp32: a plain FMA tile kernel.
#include "common.h"

namespace {

enum { EPI_RELU = 0, EPI_SWIGLU = 1, EPI_STORE = 2 };

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

// =============================================================================== bf16 / MFMA
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;   // one 16-byte load/store

constexpr int BM = 128, BN = 128, BK = 64, PITCH = BK + 8;   // PITCH in bf16 elements (144 B)
constexpr int STAGE_ELEMS = (BM + BN) * PITCH;
constexpr size_t GEMM_SMEM = 2 * STAGE_ELEMS * sizeof(uint16_t);

template <int EPI>
__global__ __launch_bounds__(256, 2) void gemm_bf16_kernel(const uint16_t* __restrict__ a_mat, int K, int N,
                                                           const void* const* __restrict__ w_ptrs,
                                                           const moe_tile* __restrict__ tiles,
                                                           const int32_t* __restrict__ hdr, void* __restrict__ out,
                                                           int ld_out) {
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, lhi = lane >> 5;
    const int ld_row = tid >> 3, ld_kv = (tid & 7) * 8;
    const int n_col_blocks = (N + BN - 1) / BN;
    const int KT = K / BK;

    const WorkList wl = work_list(hdr);
    const int n_items = wl.n_tiles * n_col_blocks;
    for (int item = wl.first; item < n_items; item += wl.stride) {
        const int cb = item / wl.n_tiles;
        const moe_tile tile = tiles[wl.bin_start + (item - cb * wl.n_tiles)];
        const int rc = tile.row_count;
        if (rc <= 0) continue;
        const int n0 = cb * BN;
        const uint16_t* __restrict__ wmat = (const uint16_t*)w_ptrs[tile.expert];

        const uint16_t* a_src[4];
        const uint16_t* b_src[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int r = ld_row + 32 * i;
            int ar = r < rc ? r : rc - 1;
            int br = n0 + r < N ? n0 + r : N - 1;
            a_src[i] = a_mat + (size_t)(tile.row_begin + ar) * K + ld_kv;
            b_src[i] = wmat + (size_t)br * K + ld_kv;
        }
        u32x4 a_reg[4], b_reg[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            a_reg[i] = *(const u32x4*)(a_src[i]);
            b_reg[i] = *(const u32x4*)(b_src[i]);
        }
        f32x16 acc[2][2];
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

        __syncthreads();   // the previous item's last reads of stage 0 are done
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            *(u32x4*)(lds + (ld_row + 32 * i) * PITCH + ld_kv) = a_reg[i];
            *(u32x4*)(lds + (BM + ld_row + 32 * i) * PITCH + ld_kv) = b_reg[i];
        }
        __syncthreads();

        const bool m_on0 = wm * 64 < rc, m_on1 = wm * 64 + 32 < rc;
        for (int kt = 0; kt < KT; ++kt) {
            const uint16_t* st = lds + (kt & 1) * STAGE_ELEMS;
            if (kt + 1 < KT) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    a_reg[i] = *(const u32x4*)(a_src[i] + (size_t)(kt + 1) * BK);
                    b_reg[i] = *(const u32x4*)(b_src[i] + (size_t)(kt + 1) * BK);
                }
            }
            if (m_on0) {
#pragma unroll
                for (int ks = 0; ks < BK / 16; ++ks) {
                    bf16x8 af[2], bf[2];
#pragma unroll
                    for (int mi = 0; mi < 2; ++mi)
                        af[mi] = *(const bf16x8*)(st + (wm * 64 + mi * 32 + l32) * PITCH + ks * 16 + lhi * 8);
#pragma unroll
                    for (int ni = 0; ni < 2; ++ni)
                        bf[ni] = *(const bf16x8*)(st + (BM + wn * 64 + ni * 32 + l32) * PITCH + ks * 16 + lhi * 8);
#pragma unroll
                    for (int mi = 0; mi < 2; ++mi) {
                        if (mi == 0 || m_on1) {
#pragma unroll
                            for (int ni = 0; ni < 2; ++ni)
                                acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mi], bf[ni], acc[mi][ni], 0, 0, 0);
                        }
                    }
                }
            }
            if (kt + 1 < KT) {
                uint16_t* dst = lds + ((kt + 1) & 1) * STAGE_ELEMS;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    *(u32x4*)(dst + (ld_row + 32 * i) * PITCH + ld_kv) = a_reg[i];
                    *(u32x4*)(dst + (BM + ld_row + 32 * i) * PITCH + ld_kv) = b_reg[i];
                }
            }
            __syncthreads();
        }

        // ---- epilogue.  acc[mi][ni][r]: row 8*(r/4) + 4*lhi + r%4, column l32 of the 32x32 block
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = wm * 64 + mi * 32 + 8 * (r >> 2) + 4 * lhi + (r & 3);
                if (row >= rc) continue;
                const size_t grow = (size_t)(tile.row_begin + row);
                if (EPI == EPI_SWIGLU) {
                    const int col = (n0 + wn * 64) / 2 + l32;   // rows [0,32) of the 64 are gate, [32,64) up
                    if (n0 + wn * 64 < N) {
                        float h = silu_f(acc[mi][0][r]) * acc[mi][1][r];
                        ((uint16_t*)out)[grow * ld_out + col] = f32_to_bf16(h);
                    }
                } else {
#pragma unroll
                    for (int ni = 0; ni < 2; ++ni) {
                        const int col = n0 + wn * 64 + ni * 32 + l32;
                        if (col < N) {
                            if (EPI == EPI_RELU)
                                ((uint16_t*)out)[grow * ld_out + col] = f32_to_bf16(fmaxf(acc[mi][ni][r], 0.f));
                            else
                                ((float*)out)[grow * ld_out + col] = acc[mi][ni][r];
                        }
                    }
                }
            }
        }
    }
}

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

template <typename Kern>
int set_smem(Kern kern, size_t bytes) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) return moe_fail(MOE_ERR_HIP, "moe_grouped_ffn: shared memory attribute: %s", hipGetErrorString(e));
    return MOE_OK;
}

constexpr int GRID_BF16 = 512;   // 2 work-groups per CU, 64 per XCD
constexpr int GRID_F32 = 512;

}  // namespace

extern "C" int moe_ffn_tile_m(moe_dtype dt) { return dt == MOE_BF16 ? BM : FM; }

static int grouped_ffn_impl(int phases, const void* x_perm, int A, int d, int F, int E, moe_act act, moe_dtype dt,
                            const void* const* w_in, const void* const* w_out, const moe_tile* tiles,
                            const int32_t* plan_hdr, int tile_m, void* h_scratch, float* y_perm, void* stream) {
    MOE_REQUIRE(moe_dtype_ok(dt), MOE_ERR_UNSUPPORTED, "moe_grouped_ffn: dtype %d", (int)dt);
    MOE_REQUIRE(act == MOE_RELU || act == MOE_SWIGLU, MOE_ERR_UNSUPPORTED, "moe_grouped_ffn: activation %d", (int)act);
    MOE_REQUIRE(A >= 0 && d >= 1 && F >= 1 && E >= 1, MOE_ERR_ARG, "moe_grouped_ffn: A=%d d=%d F=%d E=%d", A, d, F, E);
    MOE_REQUIRE(tile_m == moe_ffn_tile_m(dt), MOE_ERR_UNSUPPORTED, "moe_grouped_ffn: tile_m=%d, the kernel's is %d", tile_m, moe_ffn_tile_m(dt));
    if (dt == MOE_BF16)
        MOE_REQUIRE(d % 64 == 0 && F % 64 == 0, MOE_ERR_UNSUPPORTED, "moe_grouped_ffn: bf16 needs d and F multiples of 64 (d=%d F=%d)", d, F);
    else
        MOE_REQUIRE(d % 4 == 0 && F % 4 == 0 && (act != MOE_SWIGLU || F % 32 == 0), MOE_ERR_UNSUPPORTED,
                    "moe_grouped_ffn: fp32 needs d and F multiples of 4 (32 for SwiGLU) (d=%d F=%d)", d, F);
    if (A == 0) return MOE_OK;
    MOE_REQUIRE(tiles && plan_hdr && h_scratch, MOE_ERR_ARG, "moe_grouped_ffn: null pointer");
    MOE_REQUIRE(!(phases & 1) || (x_perm && w_in), MOE_ERR_ARG, "moe_grouped_ffn: null pointer");
    MOE_REQUIRE(!(phases & 2) || (y_perm && w_out), MOE_ERR_ARG, "moe_grouped_ffn: null pointer");
    hipStream_t st = (hipStream_t)stream;
    const int n1 = act == MOE_SWIGLU ? 2 * F : F;
    int rc;
    if (dt == MOE_BF16) {
        if (phases & 1) {
            if (act == MOE_SWIGLU) {
                if ((rc = set_smem(gemm_bf16_kernel<EPI_SWIGLU>, GEMM_SMEM)) != MOE_OK) return rc;
                hipLaunchKernelGGL(gemm_bf16_kernel<EPI_SWIGLU>, dim3(GRID_BF16), dim3(256), GEMM_SMEM, st,
                                   (const uint16_t*)x_perm, d, n1, w_in, tiles, plan_hdr, h_scratch, F);
            } else {
                if ((rc = set_smem(gemm_bf16_kernel<EPI_RELU>, GEMM_SMEM)) != MOE_OK) return rc;
                hipLaunchKernelGGL(gemm_bf16_kernel<EPI_RELU>, dim3(GRID_BF16), dim3(256), GEMM_SMEM, st,
                                   (const uint16_t*)x_perm, d, n1, w_in, tiles, plan_hdr, h_scratch, F);
            }
            MOE_CHECK_LAUNCH("moe_grouped_ffn/G1");
        }
        if (phases & 2) {
            if ((rc = set_smem(gemm_bf16_kernel<EPI_STORE>, GEMM_SMEM)) != MOE_OK) return rc;
            hipLaunchKernelGGL(gemm_bf16_kernel<EPI_STORE>, dim3(GRID_BF16), dim3(256), GEMM_SMEM, st,
                               (const uint16_t*)h_scratch, F, d, w_out, tiles, plan_hdr, (void*)y_perm, d);
            MOE_CHECK_LAUNCH("moe_grouped_ffn/G2");
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
                               const int32_t* plan_hdr, int tile_m, void* h_scratch, float* y_perm, void* stream) {
    return grouped_ffn_impl(3, x_perm, A, d, F, E, act, dt, w_in, w_out, tiles, plan_hdr, tile_m, h_scratch, y_perm, stream);
}

extern "C" int moe_grouped_ffn_phase(int phase, const void* x_perm, int A, int d, int F, int E, moe_act act,
                                     moe_dtype dt, const void* const* w_in, const void* const* w_out,
                                     const moe_tile* tiles, const int32_t* plan_hdr, int tile_m, void* h_scratch,
                                     float* y_perm, void* stream) {
    MOE_REQUIRE(phase == 1 || phase == 2, MOE_ERR_ARG, "moe_grouped_ffn_phase: phase %d", phase);
    return grouped_ffn_impl(phase, x_perm, A, d, F, E, act, dt, w_in, w_out, tiles, plan_hdr, tile_m, h_scratch, y_perm, stream);
}
