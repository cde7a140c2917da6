// Grouped 16-bit GEMM for 256-row tiles by FOUR wavefronts, each holding a 128 x 128 block of the
// 256 x 256 output tile (section 4.4: x W1 W2 over rows grouped by expert, driven by the tile
// table).  Same products, same operand layouts, same results bit for bit as the kernels of
// ffn_bf16.hip; what differs is where the energy goes.
//
// Where rows per expert are many the matrix cores run against the chip's power limit, so the
// time of a product follows the energy spent per multiply-add, not the issue slots.  An output
// tile shared by eight wavefronts of 128 x 64 reads 192 KB of operand fragments from LDS per 64
// terms of the contraction; four wavefronts of 128 x 128 read 128 KB, execute half as many
// barriers and half as many instructions around the matrix instructions.  The price is the
// register file: the 128 x 128 block is 256 accumulator registers per lane, which leaves one
// wavefront per SIMD -- so a wavefront overlaps its own memory work with its own matrix
// instructions instead of alternating with a partner.
//
// Schedule.  The contraction advances in stages of 32 terms (one matrix-instruction slice; a
// stage is 16 KB of rows + 16 KB of weight rows).  The LDS ring holds RING = 4 stages.  In step
// s a wavefront
//   * multiplies the fragments of stage s, which are in registers (64 matrix instructions),
//   * reads the fragments of stage s + 1 from LDS into the other half of its fragment registers,
//   * issues its share of the loads of stage s + RING into the buffer stage s has left,
// the three interleaved instruction by instruction, and one work-group barrier ends the step
// (everyone has read stage s + 1, everyone's part of stage s + 2 has landed).  Loads therefore
// have between two and three steps to arrive.  A work-group's items form one stream of stages:
// the loads cross item boundaries, and past the last item they go on with empty descriptors.
// An item's results are converted and stored between its last step and the next item's first.
// As in ffn_bf16.hip the first product can fetch its rows from x through the sort's permutation
// (Alg. 1's step 4 done by the operand loads) and, for top-1 routing, the second can write every
// row to its token's place times its gate value (step 6 done by the epilogue).
//
// The code is written as plain functions over explicit state (no lambdas that capture other
// lambdas): a closure is an object in memory that holds pointers, a chain of them is only
// dissolved by the compiler when every store through such a pointer can be told apart from
// the closures themselves, and when that fails the whole state of the kernel lives in scratch
// memory behind flat loads.
#include <type_traits>
#include "common.h"
#include "ffn_kernels.h"
#include "gemm_util.h"

namespace {

struct WCfg {
    static constexpr int BM = 256, BN = 256, BK = 32, RING = 4;
    static constexpr int NW = 4, NTH = NW * 64;
    static constexpr int PPR = BK / 8;                    // 16-byte pieces per row
    static constexpr int ROW_BYTES = BK * 2;
    static constexpr int WRAP = 256 / ROW_BYTES;          // rows per 256 bytes (one sweep of the banks)
    static constexpr int A_BYTES = BM * ROW_BYTES, B_BYTES = BN * ROW_BYTES;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int NA = A_BYTES / (NTH * 16), NB = B_BYTES / (NTH * 16);   // loads per thread and stage
    static constexpr int LPS = NA + NB;
    static constexpr int ROWS_PER_PASS = NTH / PPR;
    static constexpr int MI = 4, NI = 4;                  // 32 x 32 blocks of a wavefront's 128 x 128
    static constexpr int RING_BYTES = RING * STAGE_BYTES;
    static constexpr int MAX_BLK_TILES = 3068;            // tiles of a bin the block table can hold
    static constexpr int ROWINFO_BYTES = 2 * 2 * BM * 4;  // (token, gate) of a tile's rows, for two items
    static constexpr size_t SMEM = (size_t)RING_BYTES + (size_t)MAX_BLK_TILES * 4 + 16 + ROWINFO_BYTES;
    static constexpr int WAIT_BASE = (RING - 2) * LPS;    // loads younger than the stage a step waits for
    static_assert(ROWS_PER_PASS % (WRAP * PPR) == 0 && 16 % (WRAP * PPR) == 0, "swizzle period");
    static_assert(WAIT_BASE + 47 <= 63 && RING >= 3, "vmcnt range");
    static_assert(SMEM <= 160 * 1024, "LDS ring too large");
    static_assert(MI == NI, "one fragment array shape for both operands");
    __device__ static __forceinline__ int swz(int r) { return (r / WRAP) & (PPR - 1); }
};
using C = WCfg;

typedef bf16x8 FragSet[2][C::MI][2];    // [A, B][32-row block][16-row half]
typedef f32x4 Acc[C::MI][C::NI][2][2];

// What a launch and a work-group are given (wave-uniform, constant after set-up).
struct Geo {
    const uint16_t* a_mat;
    const void* const* w_ptrs;
    const moe_tile* tiles;
    const uint32_t* blk;       // LDS: first tile and tile count of the block each tile of the bin belongs to
    int K, N, KT, n_col_blocks, bin_start, n_tiles, n_items, stride;
    bool by_block;
    // gather (first product): row r of the table's row space is row row_token[r] / a_div of a_mat,
    // which has out_rows rows.  scatter (second product, top-1): row r goes to row row_token[r] of
    // the output (out_rows rows), times row_gate[that row] (1 if null).
    const int32_t* row_token;
    const float* row_gate;
    int out_rows, a_div;
    int* rinfo;                // LDS: per-row tables of two items, [parity][tokens | gates][BM]
};

// item -> (tile of the bin, column block): block after block of the bin's table, column-block-major
// inside a block (the work-groups of an XCD then share an expert's weights and a tile's rows
// through L2)
__device__ __forceinline__ void locate(const Geo& g, int it, int& tile_idx, int& cb) {
    if (g.by_block) {
        const uint32_t u = (uint32_t)sgpr((int)g.blk[it / g.n_col_blocks]);
        const int f = (int)(u & 0xffffu), sz = (int)(u >> 16);
        const int local = it - f * g.n_col_blocks;
        cb = local / sz;
        tile_idx = f + (local - cb * sz);
    } else {
        cb = it / g.n_tiles;
        tile_idx = it - cb * g.n_tiles;
    }
}

// The loader's place in the stream of stages.
struct Loader {
    __amdgpu_buffer_rsrc_t ra, rb;   // the item's rows and its block of weight rows (exactly: the range check does the clipping)
    int item, kt, buf;
    int seq;                         // gather: how many items the loader has turned to before this one
    unsigned voff_a[WCfg::NA];       // gather: byte offsets of the source rows of this lane's NA passes
};

// Gather: the source rows of an item's rows wait in LDS (rinfo[parity of the item's sequence
// number]): every wavefront fetches 64 of them there with one global -> LDS load, one item
// ahead.  Alg. 1's step 4 (the rows of x brought into expert order) is then done by the operand
// loads themselves, whose per-lane addresses are free to choose.
__device__ __forceinline__ void fetch_rows(const Geo& g, int par, int it, int wave, int lane) {
    int cb, ti;
    locate(g, it, ti, cb);
    const moe_tile t = g.tiles[g.bin_start + ti];
    const int rc = t.row_count < C::BM ? t.row_count : C::BM;
    const __amdgpu_buffer_rsrc_t rt = make_rsrc(g.row_token + t.row_begin, (unsigned)(rc > 0 ? rc : 0) * 4u);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rt, (lds_void_t*)(g.rinfo + par * 2 * C::BM + wave * 64), 4,
                                             (unsigned)(wave * 64 + lane) * 4u, 0, 0, 0);
}

template <bool GATHER>
__device__ __forceinline__ void load_item(const Geo& g, Loader& L, int it, int wave, int lane, int ld_row, unsigned ld_piece) {
    int cb, ti;
    locate(g, it, ti, cb);
    const moe_tile t = g.tiles[g.bin_start + ti];
    const int rc = t.row_count < C::BM ? t.row_count : C::BM;
    const int n0 = cb * C::BN;
    const int nr = g.N - n0 < C::BN ? g.N - n0 : C::BN;
    const uint16_t* wmat = (const uint16_t*)g.w_ptrs[t.expert];
    if constexpr (GATHER) {
        L.ra = make_rsrc(g.a_mat, (unsigned)g.out_rows * (unsigned)g.K * 2u);
        const int par = L.seq & 1;
#pragma unroll
        for (int q = 0; q < C::NA; ++q) {
            const int row = q * C::ROWS_PER_PASS + ld_row;
            unsigned src = (unsigned)g.rinfo[par * 2 * C::BM + row];
            if (g.a_div != 1) src /= (unsigned)g.a_div;
            // (a row past the tile's end gets an offset beyond the matrix: the range check reads zeros)
            L.voff_a[q] = row < rc ? src * (unsigned)g.K * 2u + ld_piece : 0xFFFFFFF0u;
        }
        // the rows of the item after this one (its table was read one item ago)
        if (it + g.stride < g.n_items) fetch_rows(g, par ^ 1, it + g.stride, wave, lane);
        ++L.seq;
    } else {
        L.ra = make_rsrc(g.a_mat + (size_t)t.row_begin * g.K, (unsigned)(rc > 0 ? rc : 0) * (unsigned)g.K * 2u);
    }
    L.rb = make_rsrc(wmat + (size_t)n0 * g.K, (unsigned)nr * (unsigned)g.K * 2u);
}

// Load q of a stage (the A passes first, then the B passes).  Piece id = i * NTH + tid of an operand
// tile: row id / PPR, position id % PPR, the piece fetched there is position ^ swz(row).  The row
// part of an address sits in the per-lane offset (only that one is range-checked); pass i lies a
// wave-uniform distance further down.
template <bool GATHER>
__device__ __forceinline__ void issue_load(const Loader& L, unsigned char* ring, int wave, unsigned ld_voff0,
                                           unsigned ld_pass, int q) {
    unsigned char* st = ring + L.buf * C::STAGE_BYTES + wave * 1024;
    const unsigned k_off = (unsigned)L.kt * (C::BK * 2);
    if (q < C::NA)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(L.ra, (lds_void_t*)(st + q * (C::NW * 1024)), 16,
                                                 GATHER ? L.voff_a[q < C::NA ? q : 0] : ld_voff0 + (unsigned)q * ld_pass, k_off, 0, 0);
    else
        __builtin_amdgcn_raw_ptr_buffer_load_lds(L.rb, (lds_void_t*)(st + C::A_BYTES + (q - C::NA) * (C::NW * 1024)), 16,
                                                 ld_voff0 + (unsigned)(q - C::NA) * ld_pass, k_off, 0, 0);
}

// after the last load of a stage
template <bool GATHER>
__device__ __forceinline__ void issue_done(const Geo& g, Loader& L, int wave, int lane, int ld_row, unsigned ld_piece) {
    L.buf = L.buf + 1 == C::RING ? 0 : L.buf + 1;
    if (++L.kt == g.KT) {
        L.kt = 0;
        if (L.item < g.n_items) L.item += g.stride;
        if (L.item < g.n_items) {
            load_item<GATHER>(g, L, L.item, wave, lane, ld_row, ld_piece);
        } else {
            // past the last item: empty descriptors (nothing is fetched), the schedule and the
            // count of outstanding loads stay those of the steady state
            L.ra = make_rsrc(g.a_mat, 0u);
            L.rb = L.ra;
        }
    }
}

// Fragment read j (0..15) of a stage into set S: the B fragments first.  Lane (l16, lq) supplies
// row l16 of a 16-row block, terms 8 lq .. 8 lq + 7 of the stage's 32: piece lq of the row, stored at
// position lq ^ swz(row); the swizzle repeats every 16 rows.
template <int S>
__device__ __forceinline__ void read_frag(FragSet (&fr)[2], const unsigned char* ring, int j, unsigned a_at, unsigned b_at) {
    if (j < 2 * C::NI)
        fr[S][1][j >> 1][j & 1] = *(const bf16x8*)(ring + b_at + ((j >> 1) * 32 + (j & 1) * 16) * C::ROW_BYTES);
    else
        fr[S][0][(j - 2 * C::NI) >> 1][j & 1] =
            *(const bf16x8*)(ring + a_at + (((j - 2 * C::NI) >> 1) * 64 + (j & 1) * 16) * C::ROW_BYTES);
}

template <int S, bool HALF_IN>
__device__ __forceinline__ void mfma(Acc& acc, const FragSet (&fr)[2], int mi, int a, int ni, int b) {
    if constexpr (HALF_IN)
        acc[mi][ni][a][b] = __builtin_amdgcn_mfma_f32_16x16x32_f16(
            __builtin_bit_cast(f16x8, fr[S][0][mi][a]), __builtin_bit_cast(f16x8, fr[S][1][ni][b]), acc[mi][ni][a][b], 0, 0, 0);
    else
        acc[mi][ni][a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fr[S][0][mi][a], fr[S][1][ni][b], acc[mi][ni][a][b], 0, 0, 0);
}

__device__ __forceinline__ void zero_acc(Acc& acc) {
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
            for (int ab = 0; ab < 4; ++ab)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[mi][ni][ab >> 1][ab & 1][r] = 0.f;
}

// (nothing may move across: neither memory operations nor matrix-core work)
__device__ __forceinline__ void wg_barrier() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("" ::: "memory");
}

// The stage two steps ahead has landed once only the stages issued after it are outstanding
// (loads complete in issue order).  Stores count like loads: for the two steps after an item
// has been stored, its store instructions (at least `n` of them) are younger than the stage
// waited for too.
struct StoreCredit {
    int left, n;
};
__device__ __forceinline__ void wait_landed(StoreCredit& sc) {
    if (sc.left > 0) {
        --sc.left;
        if (sc.n >= 47) MOE_WAIT_VMCNT(C::WAIT_BASE + 47);
        else if (sc.n >= 32) MOE_WAIT_VMCNT(C::WAIT_BASE + 32);
        else if (sc.n >= 16) MOE_WAIT_VMCNT(C::WAIT_BASE + 16);
        else MOE_WAIT_VMCNT(C::WAIT_BASE);
    } else {
        MOE_WAIT_VMCNT(C::WAIT_BASE);
    }
}

// What a lane needs to find its fragments and its loads.
struct Lane {
    int wave, lane, a_rd0, b_delta, ld_row;
    unsigned ld_voff0, ld_pass, ld_piece;
};

// One step: multiply set S (stage s), read stage s + 1 from buffer rd_buf into the other set,
// issue the loads of stage s + RING.  Sixteen groups of four matrix instructions; the reads go
// with the first twelve groups (their data is due at the next step's start), a load with every
// other group: the path that takes the loads accepts one per wavefront every few tens of
// cycles, so they are spread over the whole step.
template <int S, bool FULL, bool HALF_IN, bool GATHER>
__device__ __forceinline__ void step(const Geo& g, Loader& L, const Lane& ln, unsigned char* ring, Acc& acc,
                                     FragSet (&fr)[2], int& rd_buf, StoreCredit& sc, int mi_on) {
    const unsigned a_at = (unsigned)(rd_buf * C::STAGE_BYTES) + (unsigned)ln.a_rd0;
    const unsigned b_at = a_at + (unsigned)ln.b_delta;
#pragma unroll
    for (int t = 0; t < 16; ++t) {
        const int mi = t >> 2, a = (t >> 1) & 1, n2 = (t & 1) * 2;
        if (FULL || mi < mi_on) {
            mfma<S, HALF_IN>(acc, fr, mi, a, n2, 0);
            mfma<S, HALF_IN>(acc, fr, mi, a, n2, 1);
            mfma<S, HALF_IN>(acc, fr, mi, a, n2 + 1, 0);
            mfma<S, HALF_IN>(acc, fr, mi, a, n2 + 1, 1);
        }
        if (t < 4) {
            read_frag<S ^ 1>(fr, ring, 2 * t, a_at, b_at);
            read_frag<S ^ 1>(fr, ring, 2 * t + 1, a_at, b_at);
        } else if (t < 12) {
            read_frag<S ^ 1>(fr, ring, t + 4, a_at, b_at);
        }
        if (t & 1) issue_load<GATHER>(L, ring, ln.wave, ln.ld_voff0, ln.ld_pass, t >> 1);
        __builtin_amdgcn_sched_barrier(0);
    }
    issue_done<GATHER>(g, L, ln.wave, ln.lane, ln.ld_row, ln.ld_piece);
    rd_buf = rd_buf + 1 == C::RING ? 0 : rd_buf + 1;
    MOE_WAIT_LGKMCNT(0);
    wait_landed(sc);
    wg_barrier();
}

template <bool HALF_IN>
__device__ __forceinline__ void store_pair(__amdgpu_buffer_rsrc_t ro, float lo, float hi, unsigned voff, unsigned soff) {
    if (HALF_IN) {
        u32x2 v = {__float_as_uint(lo), __float_as_uint(hi)};
        __builtin_amdgcn_raw_buffer_store_b64(v, ro, voff, soff, 0);
    } else {
        // hidden activations saturate at the largest half value instead of becoming infinite
        const f32x2 f = {__builtin_amdgcn_fmed3f(lo, -65504.f, 65504.f), __builtin_amdgcn_fmed3f(hi, -65504.f, 65504.f)};
        const f16x2 b = __builtin_convertvector(f, f16x2);            // nearest-even
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, b), ro, voff, soff, 0);
    }
}

// Epilogue of one item.  acc[mi][ni][a][b][r]: row 16 a + 4 lq + r of the 32x32 block and packed
// weight row 16 b + l16 of its 32, which is output column 2 l16 + b (the packed order of 16-bit
// weights): a lane stores two adjacent outputs at once.  Stores go through a descriptor that
// ends with the tile's last row.
template <int EPI>
__device__ __forceinline__ void epilogue(const Acc& acc, __amdgpu_buffer_rsrc_t ro, unsigned st_voff, unsigned ld_bytes,
                                         int N, int col0, int mi_on) {
    constexpr bool HALF_IN = EPI == MOE_EPI_STORE;
    constexpr int ES = HALF_IN ? 4 : 2;
    unsigned st_base = st_voff;
    asm volatile("" : "+v"(st_base));      // (keeps the row offsets from being formed, and held, up front)
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi) {
        if (mi >= mi_on) continue;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int a = j >> 2, r = j & 3;
            const unsigned voff = st_base + (unsigned)(mi * 64 + a * 16 + r) * ld_bytes;
            if (EPI == MOE_EPI_SWIGLU) {
                // packed weight rows alternate in blocks of 32: gate, up, gate, up, ...
#pragma unroll
                for (int ni = 0; ni < C::NI; ni += 2) {
                    const int pc = col0 + ni * 32;                      // packed column of the gate block
                    if (pc < N)
                        store_pair<HALF_IN>(ro, silu_f(acc[mi][ni][a][0][r]) * acc[mi][ni + 1][a][0][r],
                                            silu_f(acc[mi][ni][a][1][r]) * acc[mi][ni + 1][a][1][r], voff, (unsigned)(pc / 2) * 2u);
                }
            } else {
#pragma unroll
                for (int ni = 0; ni < C::NI; ++ni) {
                    const int col = col0 + ni * 32;
                    if (col < N) {
                        if (EPI == MOE_EPI_RELU)
                            store_pair<HALF_IN>(ro, fmaxf(acc[mi][ni][a][0][r], 0.f), fmaxf(acc[mi][ni][a][1][r], 0.f), voff, (unsigned)col * ES);
                        else
                            store_pair<HALF_IN>(ro, acc[mi][ni][a][0][r], acc[mi][ni][a][1][r], voff, (unsigned)col * ES);
                    }
                }
            }
        }
    }
}

// Scatter epilogue (top-1 routing: Alg. 1's step 6 folded into the second product).  The token and
// the gate value of every row of a tile wait in LDS (rinfo[parity of the item][tokens | gates][row]);
// they are fetched there by two small global -> LDS loads per wavefront during the item's first
// steps: first the tokens of the tile's rows, then, indexed by them, the gate values.
__device__ __forceinline__ void fetch_tokens(const Geo& g, int par, int row_begin, int rc, int wave, int lane) {
    const __amdgpu_buffer_rsrc_t rt = make_rsrc(g.row_token + row_begin, (unsigned)(rc > 0 ? rc : 0) * 4u);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rt, (lds_void_t*)(g.rinfo + par * 2 * C::BM + wave * 64), 4,
                                             (unsigned)(wave * 64 + lane) * 4u, 0, 0, 0);
    if (!g.row_gate) ((float*)g.rinfo)[par * 2 * C::BM + C::BM + wave * 64 + lane] = 1.f;
}
__device__ __forceinline__ void fetch_gates(const Geo& g, int par, int wave, int lane) {
    if (g.row_gate) {
        const unsigned tok = (unsigned)g.rinfo[par * 2 * C::BM + wave * 64 + lane];
        const __amdgpu_buffer_rsrc_t rg = make_rsrc(g.row_gate, (unsigned)g.out_rows * 4u);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rg, (lds_void_t*)(g.rinfo + par * 2 * C::BM + C::BM + wave * 64), 4, tok * 4u, 0, 0, 0);
    }
}
__device__ __forceinline__ void epilogue_scatter(const Acc& acc, const Geo& g, __amdgpu_buffer_rsrc_t ry, int par, int rc,
                                                 int lane_row, unsigned col_off, unsigned ld_bytes, int col0, int mi_on) {
    // The tokens and gates of two row blocks are read before the first of their stores goes out:
    // the compiler cannot tell these LDS reads from the targets of the global -> LDS loads and
    // waits for every outstanding memory operation before each group of reads -- stores included.
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        unsigned voff[2][8];
        float gate[2][8];
#pragma unroll
        for (int m = 0; m < 2; ++m)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int rr = lane_row + (half * 2 + m) * 64 + (j >> 2) * 16 + (j & 3);
                const unsigned tok = (unsigned)g.rinfo[par * 2 * C::BM + rr];
                gate[m][j] = ((const float*)g.rinfo)[par * 2 * C::BM + C::BM + rr];
                // (a row past the tile's end gets an offset no output has: the range check drops it)
                voff[m][j] = (rr < rc ? tok * ld_bytes : 0x80000000u) + col_off;
            }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            const int mi = half * 2 + m;
            if (mi >= mi_on) continue;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int a = j >> 2, r = j & 3;
#pragma unroll
                for (int ni = 0; ni < C::NI; ++ni) {
                    const int col = col0 + ni * 32;
                    if (col < g.N)
                        store_pair<true>(ry, acc[mi][ni][a][0][r] * gate[m][j], acc[mi][ni][a][1][r] * gate[m][j], voff[m][j],
                                         (unsigned)col * 4u);
                }
            }
        }
    }
}

template <int EPI, bool GATHER>
__global__ __launch_bounds__(256) void gemm_wide_kernel(const uint16_t* __restrict__ a_mat, int K, int N,
                                                        const void* const* __restrict__ w_ptrs,
                                                        const moe_tile* __restrict__ tiles,
                                                        const int32_t* __restrict__ hdr, void* __restrict__ out,
                                                        int ld_out, const int32_t* __restrict__ row_token,
                                                        const float* __restrict__ row_gate, int out_rows, int a_div) {
    static_assert(!GATHER || EPI == MOE_EPI_RELU || EPI == MOE_EPI_SWIGLU, "gather: first product");
    constexpr bool SCAT = EPI == MOE_EPI_SCATTER;
    constexpr bool HALF_IN = EPI == MOE_EPI_STORE || SCAT;  // the second product: half operands, fp32 results
    constexpr int ES = HALF_IN ? 4 : 2;
    extern __shared__ __attribute__((aligned(1024))) unsigned char ring[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = sgpr(tid >> 6);
    // wavefront (wm, wn): the 32-row blocks wm, wm + 2, wm + 4, wm + 6 of the tile (interleaved, so that
    // a ragged tile leaves the two row groups the same work) and the columns wn * 128 ...
    const int wm = wave >> 1, wn = wave & 1;
    const int l16 = lane & 15, lq = lane >> 4;               // 16x16x32 fragments: row / column l16, 8-term group lq

    // the bin's work list and this work-group's share of it: a fixed stride (items are long and alike)
    Geo g;
    g.a_mat = a_mat;
    g.w_ptrs = w_ptrs;
    g.tiles = tiles;
    g.row_token = row_token;
    g.row_gate = row_gate;
    g.out_rows = out_rows;
    g.a_div = a_div;
    g.rinfo = (int*)(ring + C::SMEM - C::ROWINFO_BYTES);
    g.K = K;
    g.N = N;
    g.KT = K / C::BK;                                        // (even: K is a multiple of 64)
    g.n_col_blocks = (N + C::BN - 1) / C::BN;
    const int G = hdr[1];
    const int bin = blockIdx.x % G;
    g.stride = ((int)gridDim.x - bin + G - 1) / G;
    const int first = blockIdx.x / G;
    g.bin_start = hdr[4 + bin];
    g.n_tiles = hdr[4 + bin + 1] - g.bin_start;
    g.n_items = g.n_tiles * g.n_col_blocks;
    if (first >= g.n_items) return;

    // blk[p] = first tile and tile count of the block (one expert's tiles on this bin, at most 256)
    // that tile p belongs to
    uint32_t* blk = (uint32_t*)(ring + C::RING_BYTES);
    g.blk = blk;
    g.by_block = g.n_tiles <= C::MAX_BLK_TILES;
    if (g.by_block) {
        int* ex = (int*)ring;                              // the ring is still empty: expert of every tile
        for (int p = tid; p < g.n_tiles; p += C::NTH) ex[p] = tiles[g.bin_start + p].expert;
        __syncthreads();
        for (int p = tid; p < g.n_tiles; p += C::NTH) {
            const int e = ex[p];
            int f = p, l = p;
            while (f > 0 && (f & 255) != 0 && ex[f - 1] == e) --f;
            while (l + 1 < g.n_tiles && ((l + 1) & 255) != 0 && ex[l + 1] == e) ++l;
            blk[p] = (uint32_t)f | ((uint32_t)(l - f + 1) << 16);
        }
    }
    __syncthreads();

    Lane ln;
    ln.wave = wave;
    ln.lane = lane;
    const int ld_row = tid / C::PPR;
    ln.ld_row = ld_row;
    ln.ld_piece = (unsigned)(((tid % C::PPR) ^ C::swz(ld_row)) << 4);
    ln.ld_voff0 = (unsigned)ld_row * (unsigned)K * 2u + ln.ld_piece;
    ln.ld_pass = (unsigned)sgpr(C::ROWS_PER_PASS * K * 2);
    // the B rows of lane l16 sit a wave-uniform distance behind its A rows
    ln.a_rd0 = (wm * 32 + l16) * C::ROW_BYTES + ((lq ^ C::swz(l16)) << 4);
    ln.b_delta = sgpr(C::A_BYTES + (wn * 128 - wm * 32) * C::ROW_BYTES);

    FragSet fr[2];                                          // two sets: the one multiplied, the one being read
    Acc acc;
    StoreCredit sc = {0, 0};

    // ---- prologue: all RING stages on their way; stage 0 read into set 0; stage 1 landed
    Loader L;
    L.item = first;
    L.kt = 0;
    L.buf = 0;
    L.seq = 0;
    if constexpr (GATHER) {                                 // source rows of the first item: fetched and waited for
        fetch_rows(g, 0, first, wave, lane);
        MOE_WAIT_VMCNT(0);
        __syncthreads();
    }
    load_item<GATHER>(g, L, first, wave, lane, ld_row, ln.ld_piece);
    for (int s = 0; s < C::RING; ++s) {
#pragma unroll
        for (int q = 0; q < C::LPS; ++q) issue_load<GATHER>(L, ring, wave, ln.ld_voff0, ln.ld_pass, q);
        issue_done<GATHER>(g, L, wave, lane, ld_row, ln.ld_piece);
    }
    MOE_WAIT_VMCNT((C::RING - 1) * C::LPS);
    wg_barrier();
#pragma unroll
    for (int j = 0; j < 16; ++j) read_frag<0>(fr, ring, j, (unsigned)ln.a_rd0, (unsigned)(ln.a_rd0 + ln.b_delta));
    zero_acc(acc);
    MOE_WAIT_LGKMCNT(0);
    MOE_WAIT_VMCNT(C::WAIT_BASE);
    wg_barrier();
    // (from here on step s issues the loads of stage s + RING into buffer s % RING: L.buf is back at 0)
    int rd_buf = 1;

    const unsigned ld_bytes = (unsigned)ld_out * ES;
    const unsigned st_voff = (unsigned)(wm * 32 + 4 * lq) * ld_bytes + (unsigned)(2 * l16) * ES;
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(out, (unsigned)out_rows * ld_bytes);     // (scatter: the whole output)
    int c_seq = 0;
    for (int item = first; item < g.n_items; item += g.stride, ++c_seq) {
        int cb, ti;
        locate(g, item, ti, cb);
        const moe_tile tile = tiles[g.bin_start + ti];
        const int rc = sgpr(tile.row_count < C::BM ? tile.row_count : C::BM);
        const int col0 = cb * C::BN + wn * 128;
        // 32-row blocks of this wavefront that hold real rows (wave-uniform)
        int mi_on = ((rc + 31) / 32 - wm + 1) / 2;
        mi_on = mi_on < 0 ? 0 : (mi_on > C::MI ? C::MI : mi_on);
        // (scatter: the token load is covered by the waits of the first two steps -- every step
        // issues a stage of operand loads behind it -- and the barriers after them; the gate load
        // likewise by the steps that follow it, long before the item ends: K / 32 >= 8 steps)
        if constexpr (SCAT) fetch_tokens(g, c_seq & 1, tile.row_begin, rc, wave, lane);
        if (mi_on == C::MI) {
            for (int kt = 0; kt < g.KT; kt += 2) {
                if constexpr (SCAT) { if (kt == 4) fetch_gates(g, c_seq & 1, wave, lane); }
                step<0, true, HALF_IN, GATHER>(g, L, ln, ring, acc, fr, rd_buf, sc, mi_on);
                step<1, true, HALF_IN, GATHER>(g, L, ln, ring, acc, fr, rd_buf, sc, mi_on);
            }
        } else {
            for (int kt = 0; kt < g.KT; kt += 2) {
                if constexpr (SCAT) { if (kt == 4) fetch_gates(g, c_seq & 1, wave, lane); }
                step<0, false, HALF_IN, GATHER>(g, L, ln, ring, acc, fr, rd_buf, sc, mi_on);
                step<1, false, HALF_IN, GATHER>(g, L, ln, ring, acc, fr, rd_buf, sc, mi_on);
            }
        }
        if constexpr (SCAT) {
            epilogue_scatter(acc, g, ry, c_seq & 1, rc, wm * 32 + 4 * lq, (unsigned)(2 * l16) * 4u, ld_bytes, col0, mi_on);
        } else {
            const __amdgpu_buffer_rsrc_t ro =
                make_rsrc((const unsigned char*)out + (size_t)tile.row_begin * ld_bytes, (unsigned)(rc > 0 ? rc : 0) * ld_bytes);
            epilogue<EPI>(acc, ro, st_voff, ld_bytes, N, col0, mi_on);
        }
        zero_acc(acc);
        // store instructions just issued (a lower bound is what the waits need)
        int cols = (N - col0 + 31) / 32;
        cols = cols < 0 ? 0 : (cols > C::NI ? C::NI : cols);
        sc.n = mi_on * 8 * (EPI == MOE_EPI_SWIGLU ? (cols + 1) / 2 : cols);
        sc.left = 2;
    }
    MOE_WAIT_VMCNT(0);                                      // (the trailing empty loads still target this LDS)
}

template <int EPI, bool GATHER = false>
int launch_wide(const void* a, int K, int N, const void* const* w, const moe_tile* tiles, const int32_t* hdr, void* out,
                int ld_out, hipStream_t st, const int32_t* row_token = nullptr, const float* row_gate = nullptr,
                int out_rows = 0, int a_div = 1) {
    const int dev_ok = moe_check_gemm_device();
    if (dev_ok != MOE_OK) return dev_ok;
    auto kern = gemm_wide_kernel<EPI, GATHER>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)C::SMEM);
    if (e != hipSuccess) return moe_fail(MOE_ERR_HIP, "moe_grouped_ffn: shared memory attribute: %s", hipGetErrorString(e));
    hipLaunchKernelGGL(kern, dim3(MOE_GEMM_GRID), dim3(C::NTH), C::SMEM, st, (const uint16_t*)a, K, N, w, tiles, hdr, out,
                       ld_out, row_token, row_gate, out_rows, a_div);
    MOE_CHECK_LAUNCH("moe_grouped_ffn (bf16 GEMM, four wavefronts)");
    return MOE_OK;
}

}  // namespace

bool moe_gemm_wide_supports(int epi, int K) {
    return epi >= MOE_EPI_RELU && epi <= MOE_EPI_SCATTER && K % 64 == 0 && K >= 256;
}

int moe_launch_gemm_wide(int epi, const void* a, int K, int N, const void* const* w, const moe_tile* tiles,
                         const int32_t* hdr, void* out, int ld_out, hipStream_t st, const int32_t* row_token,
                         const float* row_gate, int out_rows) {
    if (epi == MOE_EPI_RELU) return launch_wide<MOE_EPI_RELU>(a, K, N, w, tiles, hdr, out, ld_out, st);
    if (epi == MOE_EPI_SWIGLU) return launch_wide<MOE_EPI_SWIGLU>(a, K, N, w, tiles, hdr, out, ld_out, st);
    if (epi == MOE_EPI_STORE) return launch_wide<MOE_EPI_STORE>(a, K, N, w, tiles, hdr, out, ld_out, st);
    if (epi == MOE_EPI_SCATTER)
        return launch_wide<MOE_EPI_SCATTER>(a, K, N, w, tiles, hdr, out, ld_out, st, row_token, row_gate, out_rows);
    return moe_fail(MOE_ERR_UNSUPPORTED, "moe_grouped_ffn: epilogue %d in the four-wavefront kernel", epi);
}

int moe_launch_gemm_wide_gather(int epi, const void* x, int x_rows, int K, int N, const void* const* w,
                                const moe_tile* tiles, const int32_t* hdr, void* out, int ld_out, hipStream_t st,
                                const int32_t* row_src, int src_div) {
    if (epi == MOE_EPI_SWIGLU)
        return launch_wide<MOE_EPI_SWIGLU, true>(x, K, N, w, tiles, hdr, out, ld_out, st, row_src, nullptr, x_rows, src_div);
    return launch_wide<MOE_EPI_RELU, true>(x, K, N, w, tiles, hdr, out, ld_out, st, row_src, nullptr, x_rows, src_div);
}
