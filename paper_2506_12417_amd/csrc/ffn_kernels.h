// Internal interface between the FFN entry points (ffn.hip) and the bf16 MFMA kernels (ffn_bf16.hip).
#pragma once
#include "common.h"

enum { MOE_EPI_RELU = 0, MOE_EPI_SWIGLU = 1, MOE_EPI_STORE = 2, MOE_EPI_SCATTER = 3 };

// persistent grid: one work-group per CU (256 CUs; 32 per XCD, dealt round-robin)
constexpr int MOE_GEMM_GRID = 256;

// out = epilogue(a . w_e^T) over the tile table.  epi: RELU / SWIGLU write half, STORE writes fp32,
// SCATTER writes fp32 row r to out[row_token[r]] times row_gate[row_token[r]] (row_gate may be null;
// out has out_rows rows).
// tile_m: 128 or 256 (the tile height the table was planned with).  narrow: with tile_m = 128,
// use column blocks of 128 instead of 256 outputs (ignored for SWIGLU).
int moe_launch_gemm_bf16(int epi, int tile_m, int narrow, const void* a, int K, int N, const void* const* w,
                         const moe_tile* tiles, int32_t* hdr, void* out, int ld_out, hipStream_t st,
                         const int32_t* row_token = nullptr, const float* row_gate = nullptr, int out_rows = 0);

// The first product with the row gather folded in (128-row tiles, RELU or SWIGLU; K / 64 >= 4):
// row r of the table's row space is row row_src[r] / src_div of x [x_rows, K].
int moe_launch_gemm_bf16_gather(int epi, const void* x, int x_rows, int K, int N, const void* const* w,
                                const moe_tile* tiles, int32_t* hdr, void* out, int ld_out, hipStream_t st,
                                const int32_t* row_src, int src_div);

// The same products by the kernels of ffn_stream.hip (128-row tiles; weights streamed global ->
// registers: for experts that hold few rows each, where a product's time is the fetch of its
// weights).  Same results, bit for bit.  narrow: items of 128 instead of 256 weight rows, two
// work-groups per CU.  moe_gemm_stream_supports: whether those kernels cover (epilogue, K).
bool moe_gemm_stream_supports(int epi, int K);
int moe_launch_gemm_stream(int epi, int narrow, const void* a, int K, int N, const void* const* w, const moe_tile* tiles,
                           int32_t* hdr, void* out, int ld_out, hipStream_t st, const int32_t* row_token = nullptr,
                           const float* row_gate = nullptr, int out_rows = 0);
int moe_launch_gemm_stream_gather(int narrow, const void* x, int x_rows, int K, int N, const void* const* w,
                                  const moe_tile* tiles, int32_t* hdr, void* out, int ld_out, hipStream_t st,
                                  const int32_t* row_src, int src_div);

// The same products for 256-row tiles by the kernels of ffn_wide.hip (four wavefronts of 128 x 128
// per work-group instead of eight of 128 x 64: less LDS traffic per multiply-add, which is what the
// power-bound case pays for).  Same results, bit for bit; all four epilogues, and the first
// product with the row gather folded in (arguments as for the launchers above).
bool moe_gemm_wide_supports(int epi, int K);
int moe_launch_gemm_wide(int epi, const void* a, int K, int N, const void* const* w, const moe_tile* tiles,
                         const int32_t* hdr, void* out, int ld_out, hipStream_t st, const int32_t* row_token = nullptr,
                         const float* row_gate = nullptr, int out_rows = 0);
int moe_launch_gemm_wide_gather(int epi, const void* x, int x_rows, int K, int N, const void* const* w,
                                const moe_tile* tiles, const int32_t* hdr, void* out, int ld_out, hipStream_t st,
                                const int32_t* row_src, int src_div);

// MOE_OK if the current device is the GPU the persistent launches are laid out for (256 compute
// units in 8 XCDs), else MOE_ERR_UNSUPPORTED.
int moe_check_gemm_device();
