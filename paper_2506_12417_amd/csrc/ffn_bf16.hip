// Grouped bf16 GEMM on the matrix cores: one of the two products of an expert FFN
// (section 4.4: x W1 W2) over rows grouped by expert, driven by the tile table.
//
//   out[r, n] = epilogue( sum_k a[r, k] * w_e[n, k] )      r in a tile of expert e
//
// Persistent launch, one work-group (4 wavefronts, 2 x 2) per CU.  Work-group b serves bin
// b % n_bins: work-groups are dealt round-robin to the 8 XCDs, so a bin's tiles -- and with them
// an expert's weights -- stay inside one XCD's L2.  Inside a bin the work items (tile, column
// block) are taken column-block-major with a fixed stride.
//
// Two shapes of the same kernel:
//   BM=128, BN=256  wavefront tile  64 x 128 (2 x 4 MFMA blocks)  -- experts with few rows
//   BM=256, BN=256  wavefront tile 128 x 128 (4 x 4 MFMA blocks)  -- many rows per expert
// A wavefront tile that large keeps the LDS operand traffic (one 16-byte read feeds 2 to 4
// v_mfma_f32_32x32x16_bf16) below the LDS bandwidth.
//
// Operands go global -> LDS directly (global_load_lds_dwordx4: each lane fetches 16 bytes, a
// wavefront fills 1 KB of LDS in lane order) into a ring of stages, so several K-steps of loads
// are in flight while one is multiplied; the stage barrier is a bare s_barrier, since a fence
// would drain the loads still in flight.  LDS layout of an operand tile: row r holds BK bf16
// (PPR pieces of 16 bytes), piece p stored at position p ^ swz(r); the swizzle is chosen so
// that the MFMA operand reads of 16 consecutive rows touch all 64 banks once, and it is applied
// on the global side (which piece a lane fetches).  Inside a K-step the operand reads of the
// next 16-wide slice are issued before the MFMAs of the current one.
#include "common.h"
#include "ffn_kernels.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) const void gbl_void_t;

// s_waitcnt on vmcnt only (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[15:14])
#define MOE_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 0xF) | (((n) >> 4) << 14) | (0x7 << 4) | (0xF << 8))

__device__ __forceinline__ float silu_f(float z) { return z / (1.f + __expf(-z)); }

template <int BM, int BN, int BK, int RING>
struct Cfg {
    static constexpr int PPR = BK / 8;                    // 16-byte pieces per row
    static constexpr int ROW_BYTES = BK * 2;
    static constexpr int WRAP = 256 / ROW_BYTES;          // rows per 256 bytes (one sweep of the banks)
    static constexpr int A_BYTES = BM * ROW_BYTES, B_BYTES = BN * ROW_BYTES;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int NA = BM * PPR / 256, NB = BN * PPR / 256;   // loads per thread and stage
    static constexpr int WTM = BM / 2, WTN = BN / 2;      // wavefront tile
    static constexpr int MI = WTM / 32, NI = WTN / 32;
    static constexpr size_t SMEM = (size_t)RING * STAGE_BYTES;
    __device__ static __forceinline__ int swz(int r) { return (r / WRAP) & (PPR - 1); }
};

template <int EPI, int BM, int BN, int BK, int RING>
__global__ __launch_bounds__(256, 1) void gemm_bf16_kernel(const uint16_t* __restrict__ a_mat, int K, int N,
                                                           const void* const* __restrict__ w_ptrs,
                                                           const moe_tile* __restrict__ tiles,
                                                           const int32_t* __restrict__ hdr, void* __restrict__ out,
                                                           int ld_out) {
    using C = Cfg<BM, BN, BK, RING>;
    extern __shared__ __attribute__((aligned(1024))) unsigned char ring[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, lhi = lane >> 5;
    const int n_col_blocks = (N + BN - 1) / BN;
    const int KT = K / BK;

    // the bin's work list
    const int G = hdr[1];
    const int bin = blockIdx.x % G;
    const int stride = ((int)gridDim.x - bin + G - 1) / G;
    const int bin_start = hdr[4 + bin];
    const int n_tiles = hdr[4 + bin + 1] - bin_start;
    const int n_items = n_tiles * n_col_blocks;

    for (int item = blockIdx.x / G; item < n_items; item += stride) {
        const int cb = item / n_tiles;
        const moe_tile tile = tiles[bin_start + (item - cb * n_tiles)];
        const int rc = tile.row_count;
        if (rc <= 0) continue;
        const int n0 = cb * BN;
        const uint16_t* __restrict__ wmat = (const uint16_t*)w_ptrs[tile.expert];

        // loader role: piece id = i*256 + tid -> row id / PPR, position id % PPR of the operand tile
        const uint16_t* a_src[C::NA];
        const uint16_t* b_src[C::NB];
#pragma unroll
        for (int i = 0; i < C::NA; ++i) {
            const int id = i * 256 + tid, r = id / C::PPR, kv = (id % C::PPR) ^ C::swz(r);
            a_src[i] = a_mat + (size_t)(tile.row_begin + (r < rc ? r : rc - 1)) * K + kv * 8;
        }
#pragma unroll
        for (int i = 0; i < C::NB; ++i) {
            const int id = i * 256 + tid, r = id / C::PPR, kv = (id % C::PPR) ^ C::swz(r);
            b_src[i] = wmat + (size_t)(n0 + r < N ? n0 + r : N - 1) * K + kv * 8;
        }
        auto issue = [&](int kt) {
            unsigned char* st = ring + (kt % RING) * C::STAGE_BYTES + wave * 1024;
#pragma unroll
            for (int i = 0; i < C::NA; ++i)
                __builtin_amdgcn_global_load_lds((gbl_void_t*)(a_src[i] + (size_t)kt * BK), (lds_void_t*)(st + i * 4096), 16, 0, 0);
#pragma unroll
            for (int i = 0; i < C::NB; ++i)
                __builtin_amdgcn_global_load_lds((gbl_void_t*)(b_src[i] + (size_t)kt * BK),
                                                 (lds_void_t*)(st + C::A_BYTES + i * 4096), 16, 0, 0);
        };

        f32x16 acc[C::MI][C::NI];
#pragma unroll
        for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

        // operand read offsets of this lane (bytes, without the piece position)
        int a_off[C::MI], a_swz[C::MI], b_off[C::NI], b_swz[C::NI];
#pragma unroll
        for (int mi = 0; mi < C::MI; ++mi) {
            const int r = wm * C::WTM + mi * 32 + l32;
            a_off[mi] = r * C::ROW_BYTES;
            a_swz[mi] = C::swz(r);
        }
#pragma unroll
        for (int ni = 0; ni < C::NI; ++ni) {
            const int r = wn * C::WTN + ni * 32 + l32;
            b_off[ni] = C::A_BYTES + r * C::ROW_BYTES;
            b_swz[ni] = C::swz(r);
        }
        // 32-row blocks of this wavefront that hold real rows (wave-uniform)
        int mi_on = (rc - wm * C::WTM + 31) / 32;
        mi_on = mi_on < 0 ? 0 : (mi_on > C::MI ? C::MI : mi_on);

        __syncthreads();                                       // the previous item's LDS reads are done
#pragma unroll
        for (int s = 0; s < RING - 1; ++s)
            if (s < KT) issue(s);

        constexpr int LPS = C::NA + C::NB;                     // loads per thread and stage
        for (int kt = 0; kt < KT; ++kt) {
            // stage kt has landed once only the younger stages' loads are outstanding
            const int younger = KT - 1 - kt < RING - 2 ? KT - 1 - kt : RING - 2;
            if (RING >= 4 && younger >= 2) MOE_WAIT_VMCNT(2 * LPS);
            else if (RING >= 3 && younger == 1) MOE_WAIT_VMCNT(LPS);
            else MOE_WAIT_VMCNT(0);
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            if (kt + RING - 1 < KT) issue(kt + RING - 1);      // refills the stage consumed at kt-1
            const unsigned char* st = ring + (kt % RING) * C::STAGE_BYTES;
            if (mi_on > 0) {
                bf16x8 af[2][C::MI], bf[2][C::NI];
                auto fetch = [&](int ks, int buf) {
                    const int kv = ks * 2 + lhi;
#pragma unroll
                    for (int mi = 0; mi < C::MI; ++mi)
                        if (mi < mi_on) af[buf][mi] = *(const bf16x8*)(st + a_off[mi] + ((kv ^ a_swz[mi]) << 4));
#pragma unroll
                    for (int ni = 0; ni < C::NI; ++ni)
                        bf[buf][ni] = *(const bf16x8*)(st + b_off[ni] + ((kv ^ b_swz[ni]) << 4));
                };
                fetch(0, 0);
#pragma unroll
                for (int ks = 0; ks < BK / 16; ++ks) {
                    if (ks + 1 < BK / 16) fetch(ks + 1, (ks + 1) & 1);
#pragma unroll
                    for (int mi = 0; mi < C::MI; ++mi) {
                        if (mi < mi_on) {
#pragma unroll
                            for (int ni = 0; ni < C::NI; ++ni)
                                acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks & 1][mi], bf[ks & 1][ni],
                                                                                     acc[mi][ni], 0, 0, 0);
                        }
                    }
                }
            }
        }

        // ---- epilogue.  acc[mi][ni][r]: row 8*(r/4) + 4*lhi + r%4, column l32 of the 32x32 block
#pragma unroll
        for (int mi = 0; mi < C::MI; ++mi) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = wm * C::WTM + mi * 32 + 8 * (r >> 2) + 4 * lhi + (r & 3);
                if (row >= rc) continue;
                const size_t grow = (size_t)(tile.row_begin + row);
                if (EPI == MOE_EPI_SWIGLU) {
                    // packed weight rows alternate in blocks of 32: gate, up, gate, up, ...
#pragma unroll
                    for (int ni = 0; ni < C::NI; ni += 2) {
                        const int pc = n0 + wn * C::WTN + ni * 32;          // packed column of the gate block
                        if (pc < N) {
                            const float h = silu_f(acc[mi][ni][r]) * acc[mi][ni + 1][r];
                            ((uint16_t*)out)[grow * ld_out + pc / 2 + l32] = f32_to_bf16(h);
                        }
                    }
                } else {
#pragma unroll
                    for (int ni = 0; ni < C::NI; ++ni) {
                        const int col = n0 + wn * C::WTN + ni * 32 + l32;
                        if (col < N) {
                            if (EPI == MOE_EPI_RELU)
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

template <int EPI, int BM, int BN, int BK, int RING>
int launch(const void* a, int K, int N, const void* const* w, const moe_tile* tiles, const int32_t* hdr, void* out,
           int ld_out, hipStream_t st) {
    using C = Cfg<BM, BN, BK, RING>;
    static_assert(C::SMEM <= 160 * 1024, "LDS ring too large");
    auto kern = gemm_bf16_kernel<EPI, BM, BN, BK, RING>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)C::SMEM);
    if (e != hipSuccess) return moe_fail(MOE_ERR_HIP, "moe_grouped_ffn: shared memory attribute: %s", hipGetErrorString(e));
    hipLaunchKernelGGL(kern, dim3(MOE_GEMM_GRID), dim3(256), C::SMEM, st, (const uint16_t*)a, K, N, w, tiles, hdr, out,
                       ld_out);
    MOE_CHECK_LAUNCH("moe_grouped_ffn (bf16 GEMM)");
    return MOE_OK;
}

template <int EPI>
int launch_tile(int tile_m, const void* a, int K, int N, const void* const* w, const moe_tile* tiles,
                const int32_t* hdr, void* out, int ld_out, hipStream_t st) {
    if (tile_m == 256) return launch<EPI, 256, 256, 32, 4>(a, K, N, w, tiles, hdr, out, ld_out, st);
    return launch<EPI, 128, 256, 64, 3>(a, K, N, w, tiles, hdr, out, ld_out, st);
}

}  // namespace

int moe_launch_gemm_bf16(int epi, int tile_m, const void* a, int K, int N, const void* const* w,
                         const moe_tile* tiles, const int32_t* hdr, void* out, int ld_out, hipStream_t st) {
    if (epi == MOE_EPI_RELU) return launch_tile<MOE_EPI_RELU>(tile_m, a, K, N, w, tiles, hdr, out, ld_out, st);
    if (epi == MOE_EPI_SWIGLU) return launch_tile<MOE_EPI_SWIGLU>(tile_m, a, K, N, w, tiles, hdr, out, ld_out, st);
    return launch_tile<MOE_EPI_STORE>(tile_m, a, K, N, w, tiles, hdr, out, ld_out, st);
}
