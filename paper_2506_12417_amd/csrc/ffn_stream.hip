// Grouped 16-bit GEMM for the weight-bound regime: experts that hold few rows each, so that a
// product's time is the fetch of the expert's weights (section 4.4 of the paper: below the
// threshold q an expert costs its weight fetch).
//
//   out[r, n] = epilogue( sum_k a[r, k] * w_e[n, k] )      r in a tile (at most 128 rows) of expert e
//
// Same work list, same item order, same hand-out and the same arithmetic as the kernels of
// ffn_bf16.hip (v_mfma_f32_16x16x32 over the same 32-term slices in the same order: the results
// are the same bits).  What differs is how the operands travel:
//
//   * Weights go global -> REGISTERS, straight into the matrix instruction's B-fragment layout.
//     A work-group's item is (tile, block of NW*32 packed weight rows); wavefront w owns 32 of
//     those rows and all rows of the tile, so no other wavefront ever needs its weights and
//     they need not pass through LDS.  Every wavefront keeps PF K-steps of weights (4 KB each)
//     on their way, and waits only for its own loads.  A loop of nothing but these loads and
//     the matrix instructions streams c2's weights at 5.1-5.9 TB/s where the LDS ring of
//     ffn_bf16.hip reaches 4.3-4.5.
//   * The rows of the tile (shared by all wavefronts) go global -> LDS into a ring of PF+1
//     stages of one K-step each; one work-group barrier per K-step.
//
// State: correct (bit-identical to ffn_bf16.hip on every test) but on c2 as a whole 15-25 % slower
// than the LDS ring (G1 209 vs 182 us, G2 243 vs 189 us): with one barrier per K-step the
// arithmetic and the stores of an item's results no longer hide under the loads, and the second
// product re-reads its tile of hidden activations once per 128 output columns.  It therefore runs
// on request only (moe_ffn_kernel_mode 2).
//
// The weight loads are written as assembly: for loads whose results it tracks, the compiler
// places its own, stricter waits (it counts the global -> LDS loads differently), which costs a
// fifth of the rate.  The kernel waits with s_waitcnt itself; the build inspects the device
// assembly and fails unless every register such a load writes is read by matrix instructions
// only (build.py: check_stream_registers).
#include <type_traits>
#include <utility>
#include "common.h"
#include "ffn_kernels.h"
#include "gemm_util.h"

namespace {

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>): a loop whose index is a
// compile-time constant in every iteration (register slots are chosen by it)
template <int... I, class F>
__device__ __forceinline__ void for_each_const(std::integer_sequence<int, I...>, F&& f) {
    (f(std::integral_constant<int, I>{}), ...);
}

// one 16-byte piece per lane of a weight fragment: 16 packed rows x 64 bytes per instruction
#define MOE_BLOAD(dst, voff, rsrc, soff, IMM)                                                       \
    asm volatile("buffer_load_dwordx4 %0, %1, %2, %3 offen offset:" #IMM                            \
                 : "=v"(dst) : "v"(voff), "s"(rsrc), "s"(soff) : "memory")

template <int NW_, int PF_>
struct SCfg {
    static constexpr int BM = 128, BK = 64, NW = NW_, PF = PF_, R = PF_ + 1;
    static constexpr int BN = NW * 32, NTH = NW * 64;
    static constexpr int ROW_BYTES = BK * 2, A_BYTES = BM * ROW_BYTES;
    static constexpr int NA = A_BYTES / (NTH * 16);       // global -> LDS loads per lane and K-step
    static constexpr int LPS = NA + 4;                    // loads per lane and K-step
    static constexpr int ROWS_PER_PASS = NTH / 8;
    static constexpr int MB = BM / 16;                    // 16-row blocks of a tile
    static constexpr int MAX_BLK_TILES = 2044;
    static constexpr int ROWINFO_BYTES = 2 * 2 * BM * 4;
    static constexpr size_t RING_BYTES = (size_t)R * A_BYTES;
    static constexpr size_t SMEM = RING_BYTES + (size_t)MAX_BLK_TILES * 4 + 16 + ROWINFO_BYTES;
    static_assert(NA >= 1 && ROWS_PER_PASS % 16 == 0 && (PF - 1) * LPS + 32 < 64, "tile vs threads, vmcnt range");
};

template <int EPI, int NW, int PF, bool GATHER>
__device__ __forceinline__ void gemm_stream_body(const uint16_t* __restrict__ a_mat, int K, int N,
                                                 const void* const* __restrict__ w_ptrs,
                                                 const moe_tile* __restrict__ tiles, int32_t* __restrict__ hdr,
                                                 void* __restrict__ out, int ld_out,
                                                 const int32_t* __restrict__ row_token,
                                                 const float* __restrict__ row_gate, int out_rows, int a_div) {
    using C = SCfg<NW, PF>;
    constexpr bool SCAT = EPI == MOE_EPI_SCATTER;
    constexpr bool HALF_IN = EPI == MOE_EPI_STORE || SCAT;
    static_assert(EPI != MOE_EPI_SWIGLU, "a wavefront owns 32 packed rows: no gate / up pair");
    static_assert(!GATHER || !SCAT, "gather: first product");
    constexpr int BM = C::BM, BN = C::BN, R = C::R, LPS = C::LPS, NA = C::NA, MB = C::MB;
    extern __shared__ __attribute__((aligned(1024))) unsigned char ring[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = sgpr(tid >> 6);
    const int l16 = lane & 15, lq = lane >> 4;
    const int n_col_blocks = (N + BN - 1) / BN;
    const int KT = K / 64;

    // ---- the bin's work list and this work-group's share of it (as in ffn_bf16.hip)
    const int G = hdr[1];
    const int bin = blockIdx.x % G;
    const int stride = ((int)gridDim.x - bin + G - 1) / G;
    const int first = blockIdx.x / G;
    const int bin_start = hdr[4 + bin];
    const int n_tiles = hdr[4 + bin + 1] - bin_start;
    const int n_items = n_tiles * n_col_blocks;
    int32_t* next_ctr = hdr + MOE_PLAN_HDR_CTR + bin;
    int32_t* done_ctr = hdr + MOE_PLAN_HDR_CTR + MOE_MAX_BINS;
    // Items are handed out on demand when an item is long enough for the answer (and, with the
    // gather, the item's source rows) to arrive in time; shorter contractions keep a fixed stride.
    const bool dyn = KT >= 2 * PF;
    int* ids = (int*)(ring + C::SMEM - C::ROWINFO_BYTES - 16);
    auto leave = [&]() __attribute__((always_inline)) {
        if (dyn && tid == 0) {
            const int before = __hip_atomic_fetch_add(done_ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (before == (int)gridDim.x - 1) {
                for (int b = 0; b < G; ++b) __hip_atomic_store(hdr + MOE_PLAN_HDR_CTR + b, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(done_ctr, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    };
    if (first >= n_items) {
        leave();
        return;
    }

    // ---- item order: block after block of the bin's table, column-block-major inside a block
    uint32_t* blk = (uint32_t*)(ring + C::RING_BYTES);
    const bool by_block = n_tiles <= C::MAX_BLK_TILES;
    if (by_block) {
        int* ex = (int*)ring;
        for (int p = tid; p < n_tiles; p += C::NTH) ex[p] = tiles[bin_start + p].expert;
        __syncthreads();
        for (int p = tid; p < n_tiles; p += C::NTH) {
            const int e = ex[p];
            int f = p, l = p;
            while (f > 0 && (f & 255) != 0 && ex[f - 1] == e) --f;
            while (l + 1 < n_tiles && ((l + 1) & 255) != 0 && ex[l + 1] == e) ++l;
            blk[p] = (uint32_t)f | ((uint32_t)(l - f + 1) << 16);
        }
    }
    if (dyn && tid == 0) ids[1] = stride + __hip_atomic_fetch_add(next_ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    auto item_of = [&](int seq, int prev) __attribute__((always_inline)) { return dyn ? sgpr(ids[seq & 3]) : prev + stride; };
    auto locate = [&](int it, int& tile_idx, int& cb) __attribute__((always_inline)) {
        if (by_block) {
            const uint32_t u = (uint32_t)sgpr((int)blk[it / n_col_blocks]);
            const int f = (int)(u & 0xffffu), sz = (int)(u >> 16);
            const int local = it - f * n_col_blocks;
            cb = local / sz;
            tile_idx = f + (local - cb * sz);
        } else {
            cb = it / n_tiles;
            tile_idx = it - cb * n_tiles;
        }
    };
    int* rinfo = (int*)(ring + C::SMEM - C::ROWINFO_BYTES);

    // ---- loader.  Rows of the tile: piece id = q * NTH + tid of a stage: row id / 8, position
    // id % 8 (swizzled as in ffn_bf16.hip: piece p of row r sits at p ^ (r / 2 & 7)).  Weights:
    // lane (l16, lq) fetches terms 8 lq .. 8 lq + 7 of a 32-term slice of packed row 16 b + l16 of
    // the wavefront's 32 rows.
    const int ld_row = tid / 8;
    const unsigned a_piece = (unsigned)(((tid % 8) ^ ((ld_row / 2) & 7)) << 4);
    const unsigned a_voff0 = (unsigned)ld_row * (unsigned)K * 2u + a_piece;
    const unsigned a_pass = (unsigned)sgpr(C::ROWS_PER_PASS * K * 2);
    const unsigned b_voff0 = (unsigned)l16 * (unsigned)K * 2u + (unsigned)lq * 16u;
    const unsigned b_voff1 = b_voff0 + 16u * (unsigned)K * 2u;
    __amdgpu_buffer_rsrc_t l_ra, l_rb;
    int l_item = first, l_seq = 0, l_kt = 0, l_stage = 0, ls = 0;
    int f_seq = -1, f_ready = 0;
    unsigned voff_a[GATHER ? NA : 1];
    u32x4 bq[PF][4];                                         // [slot][2 * (16-row block) + slice]

    auto fetch_rows = [&](int par, int id) __attribute__((always_inline)) {                 // (wavefront 0) source rows of item id -> rinfo[par]
        int cb, ti;
        locate(id, ti, cb);
        const moe_tile t = tiles[bin_start + ti];
        const int rc = t.row_count < BM ? t.row_count : BM;
        const __amdgpu_buffer_rsrc_t rt = make_rsrc(row_token + t.row_begin, (unsigned)(rc > 0 ? rc : 0) * 4u);
#pragma unroll
        for (int i = 0; i < BM / 64; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rt, (lds_void_t*)(rinfo + par * 2 * BM + i * 64), 4,
                                                     (unsigned)(i * 64 + lane) * 4u, 0, 0, 0);
    };
    auto load_item = [&](int it) __attribute__((always_inline)) {
        int cb, ti;
        locate(it, ti, cb);
        const moe_tile t = tiles[bin_start + ti];
        const int rc = t.row_count < BM ? t.row_count : BM;
        const int n0 = cb * BN + wave * 32;
        const int nr = N - n0 >= 32 ? 32 : 0;
        const uint16_t* wmat = (const uint16_t*)w_ptrs[t.expert];
        if constexpr (GATHER) {
            if (!dyn) {
                // short contractions: the item's source rows are fetched on the spot (every
                // wavefront passes here together; only wavefront 0 has to wait for its loads)
                if (wave == 0) {
                    fetch_rows(l_seq & 1, it);
                    MOE_WAIT_VMCNT(0);
                }
                __syncthreads();
            }
            l_ra = make_rsrc(a_mat, (unsigned)out_rows * (unsigned)K * 2u);
#pragma unroll
            for (int q = 0; q < NA; ++q) {
                const int row = q * C::ROWS_PER_PASS + ld_row;
                unsigned src = (unsigned)rinfo[(l_seq & 1) * 2 * BM + row];
                if (a_div != 1) src /= (unsigned)a_div;
                voff_a[q] = row < rc ? src * (unsigned)K * 2u + a_piece : 0xFFFFFFF0u;
            }
        } else {
            l_ra = make_rsrc(a_mat + (size_t)t.row_begin * K, (unsigned)(rc > 0 ? rc : 0) * (unsigned)K * 2u);
        }
        l_rb = make_rsrc(wmat + (size_t)(nr ? n0 : 0) * K, (unsigned)nr * (unsigned)K * 2u);
    };
    // the loads of the next K-step of the stream: rows into LDS stage l_stage, weights into slot p
    auto issue = [&](auto slot) __attribute__((always_inline)) {
        constexpr int p = decltype(slot)::value;
        unsigned char* st = ring + l_stage * C::A_BYTES + wave * 1024;
        const unsigned k_off = (unsigned)sgpr(l_kt * 128);
#pragma unroll
        for (int q = 0; q < NA; ++q)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(l_ra, (lds_void_t*)(st + q * (C::NTH * 16)), 16,
                                                     GATHER ? voff_a[GATHER ? q : 0] : a_voff0 + (unsigned)q * a_pass, k_off, 0, 0);
        MOE_BLOAD(bq[p][0], b_voff0, l_rb, k_off, 0);
        MOE_BLOAD(bq[p][1], b_voff0, l_rb, k_off, 64);
        MOE_BLOAD(bq[p][2], b_voff1, l_rb, k_off, 0);
        MOE_BLOAD(bq[p][3], b_voff1, l_rb, k_off, 64);
        __builtin_amdgcn_sched_barrier(0);
        ++ls;
        l_stage = l_stage + 1 == R ? 0 : l_stage + 1;
        if (++l_kt == KT) {
            l_kt = 0;
            if (l_item < n_items) l_item = item_of(++l_seq, l_item);
            if (l_item < n_items) {
                load_item(l_item);
                if (dyn && wave == 0) {
                    // the id of the item after this one; the answer is older than the next K-step's
                    // loads, so the wait of consumer step `ls` has covered it
                    take_ticket(next_ctr);
                    f_seq = l_seq + 1;
                    f_ready = ls;
                }
            } else {
                // past the last item the loads go on with empty descriptors (nothing is fetched):
                // one loop body, one steady count of outstanding loads
                l_ra = make_rsrc(a_mat, 0u);
                l_rb = l_ra;
            }
        }
    };

    // ---- fragments of the tile's rows: row 16 m + l16, terms 8 lq .. of slice s, at
    // (stage) + row * 128 + ((4 s + lq) ^ swizzle) * 16; slice 1 is slice 0 with bit 6 flipped
    const int a_rd0 = l16 * C::ROW_BYTES + ((lq ^ ((l16 >> 1) & 7)) << 4);
    f32x4 acc[MB][2];
    auto zero_acc = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int m = 0; m < MB; ++m)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[m][b][r] = 0.f;
    };
    auto compute = [&](auto slot, auto full, int stage, int mb_on) __attribute__((always_inline)) {
        constexpr int p = decltype(slot)::value;
        // (the empty asm keeps the compiler from forming every fragment address once, outside the
        // loop, and holding them in registers: the 16-row blocks are immediate offsets of these two)
        unsigned at[2];
        at[0] = (unsigned)(stage * C::A_BYTES + a_rd0);
        asm volatile("" : "+v"(at[0]));
        at[1] = at[0] ^ 64u;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            bf16x8 af[MB];
#pragma unroll
            for (int m = 0; m < MB; ++m)
                if (decltype(full)::value || m < mb_on) af[m] = *(const bf16x8*)(ring + at[s] + m * 16 * C::ROW_BYTES);
#pragma unroll
            for (int m = 0; m < MB; ++m)
                if (decltype(full)::value || m < mb_on) {
#pragma unroll
                    for (int b = 0; b < 2; ++b) {
                        if constexpr (HALF_IN)
                            acc[m][b] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, af[m]),
                                                                                __builtin_bit_cast(f16x8, bq[p][2 * b + s]), acc[m][b], 0, 0, 0);
                        else
                            acc[m][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[m], __builtin_bit_cast(bf16x8, bq[p][2 * b + s]),
                                                                                 acc[m][b], 0, 0, 0);
                    }
                }
        }
    };

    // ---- epilogue.  acc[m][b][r]: row 16 m + 4 lq + r of the tile, packed weight row 16 b + l16 of
    // the wavefront's 32, which is output column 2 l16 + b of its 32 (the packed order of 16-bit
    // weights): a lane stores two adjacent outputs at once.  The row part of a store's address sits
    // in the per-lane offset, the only part the range check sees.
    constexpr int ES = HALF_IN ? 4 : 2;
    const unsigned ld_bytes = (unsigned)ld_out * ES;
    const unsigned st_voff = (unsigned)(4 * lq) * ld_bytes + (unsigned)(2 * l16) * ES;
    auto store_pair = [&](__amdgpu_buffer_rsrc_t ro, float lo, float hi, unsigned voff, unsigned soff) __attribute__((always_inline)) {
        if (HALF_IN) {
            u32x2 v = {__float_as_uint(lo), __float_as_uint(hi)};
            __builtin_amdgcn_raw_buffer_store_b64(v, ro, voff, soff, 0);
        } else {
            // hidden activations saturate at the largest half value instead of becoming infinite
            const f32x2 f = {__builtin_amdgcn_fmed3f(lo, -65504.f, 65504.f), __builtin_amdgcn_fmed3f(hi, -65504.f, 65504.f)};
            const f16x2 b = __builtin_convertvector(f, f16x2);
            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, b), ro, voff, soff, 0);
        }
    };
    auto epilogue = [&](__amdgpu_buffer_rsrc_t ro, int mb_on, int col) __attribute__((always_inline)) {
        if (col >= N) return;
        // (the empty asm keeps the compiler from computing all row offsets once, up front, and
        // holding -- or spilling -- them across the whole kernel)
        unsigned st_base = st_voff;
        asm volatile("" : "+v"(st_base));
#pragma unroll
        for (int m = 0; m < MB; ++m) {
            if (m >= mb_on) continue;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const unsigned voff = st_base + (unsigned)(m * 16 + r) * ld_bytes;
                if (EPI == MOE_EPI_RELU)
                    store_pair(ro, fmaxf(acc[m][0][r], 0.f), fmaxf(acc[m][1][r], 0.f), voff, (unsigned)col * ES);
                else
                    store_pair(ro, acc[m][0][r], acc[m][1][r], voff, (unsigned)col * ES);
            }
        }
    };
    // scatter epilogue (Alg. 1 step 6 folded in for top-1 routing): token and gate value of every
    // row of the tile wait in LDS, rinfo[parity of the item][0: tokens, 1: gates][row]
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(out, (unsigned)out_rows * ld_bytes);
    auto fetch_tokens = [&](int par, int row_begin, int rc) __attribute__((always_inline)) {
        if (wave < BM / 64) {
            const __amdgpu_buffer_rsrc_t rt = make_rsrc(row_token + row_begin, (unsigned)(rc > 0 ? rc : 0) * 4u);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rt, (lds_void_t*)(rinfo + par * 2 * BM + wave * 64), 4,
                                                     (unsigned)(wave * 64 + lane) * 4u, 0, 0, 0);
            if (!row_gate) ((float*)rinfo)[par * 2 * BM + BM + wave * 64 + lane] = 1.f;
        }
    };
    auto fetch_gates = [&](int par) __attribute__((always_inline)) {
        if (row_gate && wave < BM / 64) {
            const unsigned tok = (unsigned)rinfo[par * 2 * BM + wave * 64 + lane];
            const __amdgpu_buffer_rsrc_t rg = make_rsrc(row_gate, (unsigned)out_rows * 4u);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rg, (lds_void_t*)(rinfo + par * 2 * BM + BM + wave * 64), 4, tok * 4u, 0, 0, 0);
        }
    };
    auto epilogue_scatter = [&](int par, int rc, int mb_on, int col) __attribute__((always_inline)) {
        if (col >= N) return;
        const unsigned col_off = (unsigned)(2 * l16) * 4u;
        // (one base address, the rows as immediate offsets: the empty asm keeps the compiler from
        // forming an address register per row)
        unsigned roff = (unsigned)(par * 2 * BM + 4 * lq) * 4u;
        asm volatile("" : "+v"(roff));
        const unsigned char* rbytes = ring + (C::SMEM - C::ROWINFO_BYTES);
#pragma unroll
        for (int m = 0; m < MB; ++m) {
            if (m >= mb_on) continue;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int rr = m * 16 + 4 * lq + r;
                const unsigned tok = *(const unsigned*)(rbytes + roff + (m * 16 + r) * 4);
                const float gate = *(const float*)(rbytes + roff + (BM + m * 16 + r) * 4);
                const unsigned voff = (rr < rc ? tok * ld_bytes : 0x80000000u) + col_off;
                store_pair(ry, acc[m][0][r] * gate, acc[m][1][r] * gate, voff, (unsigned)col * 4u);
            }
            // (one 16-row block at a time: read ahead for all blocks, the tokens and gates would
            // need more registers than the kernel has left)
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // (wavefront 0, after its wait of a K-step) the answer of the last ticket -> ids[], and with
    // the gather the source rows of that item -> rinfo[]
    auto publish = [&](int g) __attribute__((always_inline)) {
        if (dyn && wave == 0 && f_seq >= 0 && g >= f_ready) {
            const int id = stride + read_ticket();
            if (lane == 0) ids[f_seq & 3] = id;
            if constexpr (GATHER) { if (id < n_items) fetch_rows(f_seq & 1, sgpr(id)); }
            f_seq = -1;
            MOE_WAIT_LGKMCNT(0);
        }
    };
    auto step_barrier = [&]() __attribute__((always_inline)) {
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("" ::: "memory");
    };

    // ---- prologue: the first PF K-steps on their way
    if constexpr (GATHER) {
        if (dyn) {                                         // source rows of the first two items: fetched and waited for
            if (wave == 0) {
                fetch_rows(0, first);
                const int second = sgpr(ids[1]);
                if (second < n_items) fetch_rows(1, second);
                MOE_WAIT_VMCNT(0);
            }
            __syncthreads();
        }
    }
    load_item(first);
    for_each_const(std::make_integer_sequence<int, PF>{}, [&](auto slot) { issue(slot); });
    zero_acc();

    // ---- the stream of K-steps
    int item = first, c_seq = 0, kt = 0, g = 0, c_stage = 0;
    int rc = 0, col = 0, mb_on = 0, row_begin = 0;
    int st_steps = 0, st_blocks = 0;                          // stores of the last item still counted by the waits
    __amdgpu_buffer_rsrc_t ro = make_rsrc(out, 0u);
    auto begin_item = [&]() __attribute__((always_inline)) {
        int cb, ti;
        locate(item, ti, cb);
        const moe_tile tile = tiles[bin_start + ti];
        rc = sgpr(tile.row_count < BM ? tile.row_count : BM);
        row_begin = sgpr(tile.row_begin);
        col = cb * BN + wave * 32;
        mb_on = (rc + 15) / 16;
        mb_on = mb_on < 0 ? 0 : (mb_on > MB ? MB : mb_on);
        ro = make_rsrc((const unsigned char*)out + (size_t)row_begin * ld_bytes, (unsigned)(rc > 0 ? rc : 0) * ld_bytes);
    };
    begin_item();
    auto k_step = [&](auto slot) __attribute__((always_inline)) {
        constexpr int p = decltype(slot)::value;
        // this wavefront's loads of the K-step have landed: its rows' pieces in LDS, its weights in slot p.
        // Loads and stores complete in the order they were issued, so what may stay outstanding is
        // everything issued after this K-step's loads: the loads of the PF-1 later K-steps, and --
        // during the PF K-steps after an item's end -- the stores of that item's results (4 per
        // 16-row block and lane).  Without that allowance every item would end with a wait for all
        // the loads in flight.
        if (st_steps > 0) {
            --st_steps;
            switch (st_blocks) {
                case 8: MOE_WAIT_VMCNT((PF - 1) * LPS + 32); break;
                case 7: MOE_WAIT_VMCNT((PF - 1) * LPS + 28); break;
                case 6: MOE_WAIT_VMCNT((PF - 1) * LPS + 24); break;
                case 5: MOE_WAIT_VMCNT((PF - 1) * LPS + 20); break;
                case 4: MOE_WAIT_VMCNT((PF - 1) * LPS + 16); break;
                case 3: MOE_WAIT_VMCNT((PF - 1) * LPS + 12); break;
                case 2: MOE_WAIT_VMCNT((PF - 1) * LPS + 8); break;
                case 1: MOE_WAIT_VMCNT((PF - 1) * LPS + 4); break;
                default: MOE_WAIT_VMCNT((PF - 1) * LPS); break;
            }
        } else {
            MOE_WAIT_VMCNT((PF - 1) * LPS);
        }
        asm volatile("" : "+v"(bq[p][0]), "+v"(bq[p][1]), "+v"(bq[p][2]), "+v"(bq[p][3]));
        publish(g);
        // everyone's pieces of the stage are in LDS, and everyone has read the stage the next loads overwrite
        step_barrier();
        if constexpr (SCAT) {
            if (kt == 0) fetch_tokens(c_seq & 1, row_begin, rc);
            if (kt == PF - 1) fetch_gates(c_seq & 1);
        }
        if (mb_on == MB) compute(slot, std::true_type{}, c_stage, mb_on);
        else compute(slot, std::false_type{}, c_stage, mb_on);
        __builtin_amdgcn_sched_barrier(0);
        issue(slot);
        ++g;
        c_stage = c_stage + 1 == R ? 0 : c_stage + 1;
        if (++kt == KT) {
            kt = 0;
            if constexpr (SCAT) epilogue_scatter(c_seq & 1, rc, mb_on, col);
            else epilogue(ro, mb_on, col);
            // (items shorter than PF K-steps would pile up several items' stores: no allowance then)
            st_blocks = col < N ? mb_on : 0;
            st_steps = KT > PF ? PF : 0;
            zero_acc();
            item = item_of(c_seq + 1, item);
            ++c_seq;
            if (item < n_items) begin_item();
        }
    };
    while (item < n_items) {
        for_each_const(std::make_integer_sequence<int, PF>{}, [&](auto slot) {
            if (item < n_items) k_step(slot);
        });
    }
    // (the trailing empty loads still target this LDS and the weight registers: they must have
    // landed before anything else may use those registers)
    MOE_WAIT_VMCNT(0);
    __builtin_amdgcn_sched_barrier(0);
    leave();
}

// (launch bounds: 8 / NW work-groups per CU, i.e. two wavefronts per SIMD either way: 256 registers each)
template <int EPI, int NW, int PF, bool GATHER>
__global__ __launch_bounds__(NW * 64, 2) void gemm_stream_kernel(const uint16_t* __restrict__ a_mat, int K, int N,
                                                               const void* const* __restrict__ w_ptrs,
                                                               const moe_tile* __restrict__ tiles,
                                                               int32_t* __restrict__ hdr, void* __restrict__ out,
                                                               int ld_out, const int32_t* __restrict__ row_token,
                                                               const float* __restrict__ row_gate, int out_rows,
                                                               int a_div) {
    gemm_stream_body<EPI, NW, PF, GATHER>(a_mat, K, N, w_ptrs, tiles, hdr, out, ld_out, row_token, row_gate, out_rows, a_div);
}

template <int EPI, int NW, int PF, bool GATHER>
int launch(const void* a, int K, int N, const void* const* w, const moe_tile* tiles, int32_t* hdr, void* out,
           int ld_out, const int32_t* row_token, const float* row_gate, int out_rows, int a_div, hipStream_t st) {
    using C = SCfg<NW, PF>;
    static_assert(C::SMEM * (8 / NW) <= 160 * 1024, "LDS: 8 / NW work-groups per CU");
    const int dev_ok = moe_check_gemm_device();
    if (dev_ok != MOE_OK) return dev_ok;
    auto kern = gemm_stream_kernel<EPI, NW, PF, GATHER>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)C::SMEM);
    if (e != hipSuccess) return moe_fail(MOE_ERR_HIP, "moe_grouped_ffn: shared memory attribute: %s", hipGetErrorString(e));
    hipLaunchKernelGGL(kern, dim3(MOE_GEMM_GRID * (8 / NW)), dim3(C::NTH), C::SMEM, st, (const uint16_t*)a, K, N, w, tiles, hdr,
                       out, ld_out, row_token, row_gate, out_rows, a_div);
    MOE_CHECK_LAUNCH("moe_grouped_ffn (bf16 GEMM, weights streamed to registers)");
    return MOE_OK;
}

template <int EPI, bool GATHER>
int launch_width(int narrow, const void* a, int K, int N, const void* const* w, const moe_tile* tiles, int32_t* hdr,
                 void* out, int ld_out, const int32_t* row_token, const float* row_gate, int out_rows, int a_div,
                 hipStream_t st) {
    if (narrow) return launch<EPI, 4, 3, GATHER>(a, K, N, w, tiles, hdr, out, ld_out, row_token, row_gate, out_rows, a_div, st);
    return launch<EPI, 8, 4, GATHER>(a, K, N, w, tiles, hdr, out, ld_out, row_token, row_gate, out_rows, a_div, st);
}

}  // namespace

bool moe_gemm_stream_supports(int epi, int K) {
    if (epi == MOE_EPI_SWIGLU || K % 64 != 0) return false;
    // the scatter epilogue's token and gate tables need 2 * PF K-steps per item to arrive
    return epi != MOE_EPI_SCATTER || K / 64 >= 8;
}

int moe_launch_gemm_stream(int epi, int narrow, const void* a, int K, int N, const void* const* w, const moe_tile* tiles,
                           int32_t* hdr, void* out, int ld_out, hipStream_t st, const int32_t* row_token,
                           const float* row_gate, int out_rows) {
    if (epi == MOE_EPI_RELU) return launch_width<MOE_EPI_RELU, false>(narrow, a, K, N, w, tiles, hdr, out, ld_out, nullptr, nullptr, 0, 1, st);
    if (epi == MOE_EPI_SCATTER)
        return launch_width<MOE_EPI_SCATTER, false>(narrow, a, K, N, w, tiles, hdr, out, ld_out, row_token, row_gate, out_rows, 1, st);
    return launch_width<MOE_EPI_STORE, false>(narrow, a, K, N, w, tiles, hdr, out, ld_out, nullptr, nullptr, 0, 1, st);
}

int moe_launch_gemm_stream_gather(int narrow, const void* x, int x_rows, int K, int N, const void* const* w,
                                  const moe_tile* tiles, int32_t* hdr, void* out, int ld_out, hipStream_t st,
                                  const int32_t* row_src, int src_div) {
    return launch_width<MOE_EPI_RELU, true>(narrow, x, K, N, w, tiles, hdr, out, ld_out, row_src, nullptr, x_rows, src_div, st);
}
