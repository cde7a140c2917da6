// Grouped 16-bit GEMM on the matrix cores: one of the two products of an expert FFN
// (section 4.4: x W1 W2) over rows grouped by expert, driven by the tile table.
//
//   out[r, n] = epilogue( sum_k a[r, k] * w_e[n, k] )      r in a tile of expert e
//
// The first product multiplies bf16 by bf16 and stores the hidden activations H as IEEE half:
// H is the only value the path rounds between its input and its fp32 output, and half keeps 11
// significant bits of it where bf16 keeps 8 (the error of y falls eightfold; it is otherwise
// the largest one, several per cent of the output's RMS for the tokens with the largest gate
// values).  The second product multiplies half by half: moe_pack_w_out has converted W_out,
// which is exact for every bf16 weight of magnitude 2^-14 .. 65504.  Both matrix instructions
// run at the same rate and accumulate in fp32.
//
// The matrix instruction is v_mfma_f32_16x16x32 (bf16 or f16).  Under real data the chip's
// arithmetic rate is set by its power limit, and this shape sustains about 8 % more than
// 32x32x16 in a loop of nothing else; the kernel as a whole gains about 3 % from it.  A lane
// then holds column l16 of a 16-column sub-block; moe_pack_weights orders the weight rows so
// that the two sub-blocks of a 32-column block give the lane two adjacent outputs (packed row
// 16 h + j of every 32 = output 2 j + h), which it stores as one pair without any exchange
// between lanes, and the operand loads stay plain runs of consecutive rows.
//
// Persistent launch, one work-group of 8 wavefronts (2 per SIMD) per CU.  Work-group b serves
// bin b % n_bins: work-groups are dealt round-robin to the 8 XCDs, so a bin's tiles -- and with
// them an expert's weights -- stay inside one XCD's L2.  Inside a bin the work items
// (tile, column block) are taken block after block in the order of the plan's table: the first
// round with a fixed stride, the later ones on demand (a counter per bin), except by the
// 256-row configuration, which keeps the stride.
//
// A work-group's items form ONE stream of K-steps: the operand loads run RING-1 steps ahead of
// the arithmetic and cross item boundaries, so the next item's first tiles are already on their
// way while the current item is finished and stored.
//
// Operands go global -> LDS directly (buffer_load_dwordx4 ... lds: each lane fetches 16 bytes, a
// wavefront fills 1 KB of LDS in lane order).  The loads go through buffer descriptors that
// cover exactly the rows of the tile (and of the column block): rows past the end read as zero
// and stores past the end are dropped by the hardware's range check, so ragged tiles need no
// clamping, and the per-load address arithmetic is scalar.  A K-step is 64 wide: one full
// 128-byte line per row.
//
// LDS layout of an operand tile: row r holds BK bf16 (PPR pieces of 16 bytes), piece p stored
// at position p ^ swz(r); the swizzle is chosen so that the MFMA operand reads of 16 consecutive
// rows touch all 64 banks once, and it is applied on the global side (which piece a lane
// fetches).
//
// Schedule.  The two wavefronts of a SIMD alternate: while one multiplies a chunk of a K-step
// (its operand fragments are in registers), the other reads the fragments of its next chunk from
// LDS, issues its share of the next stage's loads and -- at an item boundary -- stores the
// finished item.  The wavefronts 0-3 ("group 0") run one phase ahead of the wavefronts 4-7; a
// work-group barrier closes every phase, so the matrix cores always have exactly one wavefront
// per SIMD feeding them and never wait for an LDS read.  Both groups execute the same number of
// barriers: group 1 one more at the start, group 0 one more at the end.
#include <type_traits>
#include "common.h"
#include "ffn_kernels.h"
#include "gemm_util.h"

namespace {

template <int BM_, int BN_, int BK_, int RING_, int WM_, int WN_, int CS_>
struct Cfg {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, RING = RING_, WM = WM_, WN = WN_, CS = CS_;
    static constexpr int NW = WM * WN, NTH = NW * 64;
    static constexpr int PPR = BK / 8;                    // 16-byte pieces per row
    static constexpr int ROW_BYTES = BK * 2;
    static constexpr int WRAP = 256 / ROW_BYTES;          // rows per 256 bytes (one sweep of the banks)
    static constexpr int A_BYTES = BM * ROW_BYTES, B_BYTES = BN * ROW_BYTES;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int NA = A_BYTES / (NTH * 16), NB = B_BYTES / (NTH * 16);   // loads per thread and stage
    static constexpr int LPS = NA + NB;
    static constexpr int ROWS_PER_PASS = NTH / PPR;       // operand rows one pass of the work-group's loads covers
    static constexpr int WTM = BM / WM, WTN = BN / WN;    // wavefront tile
    static constexpr int MI = WTM / 32, NI = WTN / 32;
    static constexpr int KS = BK / 16;                    // 16-wide slices per K-step
    static constexpr int PH = KS / CS;                    // chunks (of CS slices) per K-step
    static constexpr size_t RING_BYTES = (size_t)RING * STAGE_BYTES;
    static constexpr int MAX_BLK_TILES = 3068;            // tiles of a bin the block table can hold
    static constexpr int ROWINFO_BYTES = 2 * 2 * BM * 4;  // (token, gate) of a tile's rows, for two items (scatter epilogue)
    static constexpr size_t SMEM = RING_BYTES + (size_t)MAX_BLK_TILES * 4 + 16 + ROWINFO_BYTES;   // + ids[4] of the work hand-out
    static_assert(NA >= 1 && NB >= 1 && A_BYTES % (NTH * 16) == 0 && B_BYTES % (NTH * 16) == 0, "tile vs threads");
    static_assert(ROWS_PER_PASS % (WRAP * PPR) == 0 && 32 % (WRAP * PPR) == 0, "swizzle period");
    static_assert(KS % CS == 0 && NW == 8 && WM == 2, "two groups of four wavefronts, row blocks interleaved");
    static_assert(LPS * (RING - 2 > 0 ? RING - 2 : 0) < 64 && RING <= 4, "vmcnt range");
    __device__ static __forceinline__ int swz(int r) { return (r / WRAP) & (PPR - 1); }
};

// (The body is a __device__ function: it uses buffer-descriptor types that exist only on the
// device side, and the host pass must still be able to instantiate the kernel's stub.)
// (Every lambda of the body is force-inlined: one that the compiler leaves as a call takes its
// captures through memory, and with them go the LDS address space of the ring and the
// wave-uniformity of the item bookkeeping -- flat loads and vector loads with full waits.)
template <int EPI, int BM, int BN, int BK, int RING, int WM, int WN, int CS, bool GATHER>
__device__ __forceinline__ void gemm_bf16_body(const uint16_t* __restrict__ a_mat, int K, int N,
                                               const void* const* __restrict__ w_ptrs,
                                               const moe_tile* __restrict__ tiles, int32_t* __restrict__ hdr,
                                               void* __restrict__ out, int ld_out,
                                               const int32_t* __restrict__ row_token,
                                               const float* __restrict__ row_gate, int out_rows, int a_div) {
    using C = Cfg<BM, BN, BK, RING, WM, WN, CS>;
    // GATHER (first product only): row r of the table's row space is row row_token[r] / a_div of
    // a_mat, which has out_rows rows -- Alg. 1's step 4 (the rows of x brought into expert order)
    // done by the operand loads themselves, whose per-lane addresses are free to choose.
    static_assert(!GATHER || (EPI != MOE_EPI_SCATTER && RING >= 3), "gather: first product, on-demand hand-out");
    constexpr int MI = C::MI, NI = C::NI, PH = C::PH;
    // The first product takes bf16 operands and writes the hidden activations as IEEE half; the
    // second one (plain store of fp32 results) takes those and a half copy of the weights.
    // SCATTER is STORE with Alg. 1's step 6 folded in for top-1 routing: row r goes to output row
    // row_token[r], times row_gate[that token].
    constexpr bool SCAT = EPI == MOE_EPI_SCATTER;
    constexpr bool HALF_IN = EPI == MOE_EPI_STORE || SCAT;
    extern __shared__ __attribute__((aligned(1024))) unsigned char ring[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = sgpr(tid >> 6);
    // Wavefront w sits on SIMD w % 4; group w / 4 takes the 32-row blocks wm, wm + 2, wm + 4, ... of the
    // tile, so that a ragged tile leaves both wavefronts of a SIMD the same amount of work.
    const int wm = wave / C::WN, wn = wave % C::WN;
    const int grp = wm;
    const int l16 = lane & 15, lq = lane >> 4;               // 16x16x32 fragments: row / column l16, 8-term group lq
    const int n_col_blocks = (N + BN - 1) / BN;
    const int KT = K / BK;

    // the bin's work list and this work-group's share of it
    const int G = hdr[1];
    const int bin = blockIdx.x % G;
    const int stride = ((int)gridDim.x - bin + G - 1) / G;
    const int first = blockIdx.x / G;
    const int bin_start = hdr[4 + bin];
    const int n_tiles = hdr[4 + bin + 1] - bin_start;
    const int n_items = n_tiles * n_col_blocks;

    // ---- who takes which item.  The first round is fixed: work-group j of the bin starts with
    // item j.  After that an item goes to whichever work-group of the bin asks next (a counter per
    // bin in the plan header): items differ a lot in duration -- a tile of a cold expert waits for
    // its weights from HBM, a tile of a hot expert finds them in L2 -- and with a fixed stride the
    // work-groups of a bin finish far apart.  The counter is read one item ahead by wavefront 0
    // and handed to the others through LDS (ids[seq % 4]); the answer has a whole item's time to
    // arrive.  Very short contractions (fewer K-steps per item than the answer needs) keep the
    // fixed stride.  The last work-group to finish zeroes the counters for the next launch.
    int32_t* next_ctr = hdr + MOE_PLAN_HDR_CTR + bin;
    int32_t* done_ctr = hdr + MOE_PLAN_HDR_CTR + MOE_MAX_BINS;
    // (the 256-row configuration keeps the fixed stride: its items are long and alike, handing
    // them out on demand measured no gain there, and it has no register to spare)
    const bool dyn = RING >= 3 && KT >= 4;
    int* ids = (int*)(ring + C::SMEM - C::ROWINFO_BYTES - 16);
    auto leave = [&]() __attribute__((always_inline)) {                                    // (every work-group of a dynamic launch passes here once)
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

    // ---- item order.  A bin's table lists its blocks (one expert's rows on this bin) one after
    // the other.  Items are taken block after block, column-block-major inside a block: the
    // work-groups of the XCD then run the column blocks of a one-tile expert side by side (its
    // rows are fetched once and shared through L2), and for an expert with many tiles the same
    // column block of several row tiles (its weights are fetched once).  blk[p] = first tile and
    // tile count of the block that tile p belongs to (blocks longer than 256 tiles are cut).
    uint32_t* blk = (uint32_t*)(ring + C::RING_BYTES);
    const bool by_block = n_tiles <= C::MAX_BLK_TILES;
    if (by_block) {
        int* ex = (int*)ring;                              // the ring is still empty: expert of every tile
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
    // the second item of this work-group (nothing is in flight yet: the answer is simply waited for)
    if (dyn && tid == 0) ids[1] = stride + __hip_atomic_fetch_add(next_ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    // id of the seq-th item of this work-group (seq >= 1)
    auto item_of = [&](int seq, int prev) __attribute__((always_inline)) { return dyn ? sgpr(ids[seq & 3]) : prev + stride; };
    // Wavefront 0 asks for the id of item `seq`; the answer is passed on by publish() once the
    // wait of a later K-step has covered it (loads and this request complete in issue order).
    int f_seq = -1, f_ready = 0;
    // item -> (tile of the bin, column block)
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

    int* rinfo = (int*)(ring + C::SMEM - C::ROWINFO_BYTES);   // per-row tables of two items (scatter epilogue, gather)

    // ---- loader.  Piece id = i * NTH + tid of an operand tile: row id / PPR, position id % PPR;
    // the swizzle does not depend on i, so one per-lane offset serves every load of a stage.
    const int ld_row = tid / C::PPR;
    // The row part of an address must sit in the per-lane offset: only that one is range-checked.
    // (pass i of a stage lies a wave-uniform distance further down: one register, one add per load)
    const unsigned ld_voff0 = (unsigned)ld_row * (unsigned)K * 2u + (unsigned)(((tid % C::PPR) ^ C::swz(ld_row)) << 4);
    const unsigned ld_pass = (unsigned)sgpr(C::ROWS_PER_PASS * K * 2);
    __amdgpu_buffer_rsrc_t l_ra, l_rb;
    int l_item = first, l_seq = 0, l_kt = 0, l_buf = 0, issued = 0;
    int g = 0, c_buf = 0;                                   // K-step counter of the stream, its stage
    // GATHER: the source rows of an item's rows wait in LDS (rinfo[parity of the item's sequence
    // number][row]): wavefront 0 fetches them there with a global -> LDS load as soon as it knows
    // the item's id, one item ahead (see publish()).  When the loader turns to the item, every
    // lane reads the rows of its NA passes and keeps their byte offsets.
    unsigned voff_a[GATHER ? C::NA : 1];
    auto fetch_rows = [&](int par, int id) __attribute__((always_inline)) {               // (wavefront 0)
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
    auto rows_to_offsets = [&](int par, int rc) __attribute__((always_inline)) {
        const unsigned piece = (unsigned)(((tid % C::PPR) ^ C::swz(ld_row)) << 4);
#pragma unroll
        for (int q = 0; q < C::NA; ++q) {
            const int row = q * C::ROWS_PER_PASS + ld_row;
            unsigned src = (unsigned)rinfo[par * 2 * BM + row];
            if (a_div != 1) src /= (unsigned)a_div;
            // (a row past the tile's end gets an offset beyond the matrix: the range check reads zeros)
            voff_a[q] = row < rc ? src * (unsigned)K * 2u + piece : 0xFFFFFFF0u;
        }
    };
    auto load_item = [&](int it) __attribute__((always_inline)) {
        int cb, ti;
        locate(it, ti, cb);
        const moe_tile t = tiles[bin_start + ti];
        const int rc = t.row_count < BM ? t.row_count : BM;
        const int n0 = cb * BN;
        const int nr = N - n0 < BN ? N - n0 : BN;
        const uint16_t* wmat = (const uint16_t*)w_ptrs[t.expert];
        if constexpr (GATHER) {
            l_ra = make_rsrc(a_mat, (unsigned)out_rows * (unsigned)K * 2u);
            rows_to_offsets(l_seq & 1, rc);
        } else {
            l_ra = make_rsrc(a_mat + (size_t)t.row_begin * K, (unsigned)(rc > 0 ? rc : 0) * (unsigned)K * 2u);
        }
        l_rb = make_rsrc(wmat + (size_t)n0 * K, (unsigned)nr * (unsigned)K * 2u);
    };
    // load q of a stage (the A passes first, then the B passes), and the bookkeeping once all are out
    auto issue_load = [&](int q) __attribute__((always_inline)) {
        unsigned char* st = ring + l_buf * C::STAGE_BYTES + wave * 1024;
        const unsigned k_off = (unsigned)l_kt * (BK * 2);
        if (q < C::NA)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(l_ra, (lds_void_t*)(st + q * (C::NW * 1024)), 16,
                                                     GATHER ? voff_a[GATHER ? q : 0] : ld_voff0 + (unsigned)q * ld_pass, k_off, 0, 0);
        else
            __builtin_amdgcn_raw_ptr_buffer_load_lds(l_rb, (lds_void_t*)(st + C::A_BYTES + (q - C::NA) * (C::NW * 1024)), 16,
                                                     ld_voff0 + (unsigned)(q - C::NA) * ld_pass, k_off, 0, 0);
    };
    auto issue_done = [&]() __attribute__((always_inline)) {
        ++issued;
        l_buf = l_buf + 1 == RING ? 0 : l_buf + 1;
        if (++l_kt == KT) {
            l_kt = 0;
            if (l_item < n_items) l_item = item_of(++l_seq, l_item);
            if (l_item < n_items) {
                load_item(l_item);
                if (dyn && wave == 0) {
                    take_ticket(next_ctr);
                    f_seq = l_seq + 1;
                    f_ready = g + RING - 2;
                }
            } else {
                // Past the last item the loads go on with empty descriptors: nothing is fetched, the
                // free ring buffer receives zeros, and the schedule and the count of outstanding
                // loads stay those of the steady state (no second copy of the loop without loads).
                l_ra = make_rsrc(a_mat, 0u);
                l_rb = l_ra;
            }
        }
    };
    auto issue = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < C::LPS; ++q) issue_load(q);
        issue_done();
    };

    // ---- operand fragment reads.  The matrix instruction is 16x16x32 (it draws about 8 % less
    // power per FLOP than 32x32x16 on this chip, and power is what bounds the arithmetic): lane
    // (l16, lq) supplies row l16 of a 16-row block, terms 8 lq .. 8 lq + 7 of a 32-term slice.  A
    // 32x32 block of the output is four 16x16 sub-blocks [a][b]; row block mi of this wavefront is
    // block mi * WM + wm of the tile.
    // Slice q of a row is piece (4 q + lq) ^ swz = (4 q) ^ (lq ^ swz), and every row and stage starts
    // on a multiple of the row size: the address of slice q is the address of slice 0 with bits
    // flipped, so one per-lane register (and one XOR per read) serves all slices.  The swizzle
    // repeats every 16 rows, and the B rows of lane l16 sit a wave-uniform distance behind its A rows.
    static_assert(C::STAGE_BYTES % C::ROW_BYTES == 0 && (C::ROW_BYTES & (C::ROW_BYTES - 1)) == 0, "slice addressing");
    static_assert(CS % 2 == 0 && 16 % (C::WRAP * C::PPR) == 0, "32-term slices, swizzle period");
    constexpr int S32 = CS / 2;                             // 32-term slices per chunk
    int a_rd0 = (wm * 32 + l16) * C::ROW_BYTES + ((lq ^ C::swz(l16)) << 4);
    const int b_delta = sgpr(C::A_BYTES + (wn * C::WTN - wm * 32) * C::ROW_BYTES);
    bf16x8 af[S32][MI][2], bf[S32][NI][2];
    f32x4 acc[MI][NI][2][2];
    auto zero_acc = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int ab = 0; ab < 4; ++ab)
#pragma unroll
                    for (int r = 0; r < 4; ++r) acc[mi][ni][ab >> 1][ab & 1][r] = 0.f;
    };
    // Memory phase of chunk h: the fragments of the slices h*S32 ... of the stage in buffer buf go to
    // registers; the first chunk also issues the next stage's global -> LDS loads.  A load occupies
    // the issuing wavefront until the texture path accepts it (some tens of cycles each when four
    // wavefronts issue at once), the LDS reads do not: the loads are spread between the reads so
    // that the two kinds of waiting overlap instead of adding up.
    auto mem_phase = [&](int buf, int h) __attribute__((always_inline)) {
        constexpr int PER = 2 * (NI + MI), NR = S32 * PER, NL = C::LPS, STEP = NR / NL;
        static_assert(STEP >= 1, "more loads than reads in a chunk");
        // (the empty asm keeps the compiler from forming all slice addresses once, outside the loop,
        // and holding them in registers the 256-row configuration does not have)
        asm volatile("" : "+v"(a_rd0));
        const unsigned a_at = (unsigned)(buf * C::STAGE_BYTES) + (unsigned)a_rd0;
        const unsigned b_at = a_at + (unsigned)b_delta;
#pragma unroll
        for (int j = 0; j < NR; ++j) {
            if (h == 0 && j % STEP == 0 && j / STEP < NL) {
                issue_load(j / STEP);
                __builtin_amdgcn_sched_barrier(0);
            }
            const int s = j / PER, idx = j % PER;
            const unsigned flip = (unsigned)((h * S32 + s) << 6);
            if (idx < 2 * NI)
                bf[s][idx >> 1][idx & 1] =
                    *(const bf16x8*)(ring + (b_at ^ flip) + ((idx >> 1) * 32 + (idx & 1) * 16) * C::ROW_BYTES);
            else
                af[s][(idx - 2 * NI) >> 1][idx & 1] =
                    *(const bf16x8*)(ring + (a_at ^ flip) + (((idx - 2 * NI) >> 1) * (C::WM * 32) + (idx & 1) * 16) * C::ROW_BYTES);
        }
        if (h == 0) issue_done();
    };
    auto mfma_chunk = [&](auto full, int mi_on) __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < S32; ++s)
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                if (decltype(full)::value || mi < mi_on) {
#pragma unroll
                    for (int a = 0; a < 2; ++a)
#pragma unroll
                        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                            for (int b = 0; b < 2; ++b)
                                if constexpr (HALF_IN)
                                    acc[mi][ni][a][b] = __builtin_amdgcn_mfma_f32_16x16x32_f16(
                                        __builtin_bit_cast(f16x8, af[s][mi][a]), __builtin_bit_cast(f16x8, bf[s][ni][b]),
                                        acc[mi][ni][a][b], 0, 0, 0);
                                else
                                    acc[mi][ni][a][b] =
                                        __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[s][mi][a], bf[s][ni][b], acc[mi][ni][a][b], 0, 0, 0);
                }
            }
    };
    // Stage g+1 has landed once only the stages issued after it are outstanding.  (Loads
    // complete in issue order; stores that are still in flight only make the wait longer.)
    auto wait_stage_after = [&](int g) __attribute__((always_inline)) {
        const int younger = issued - g - 2;
        if (RING >= 4 && younger >= 2) MOE_WAIT_VMCNT(2 * C::LPS);
        else if (RING >= 3 && younger >= 1) MOE_WAIT_VMCNT(C::LPS);
        else MOE_WAIT_VMCNT(0);
    };
    // (wavefront 0, after its wait of a K-step)
    auto publish = [&]() __attribute__((always_inline)) {
        if (dyn && wave == 0 && f_seq >= 0 && g >= f_ready) {
            const int id = stride + read_ticket();
            if (lane == 0) ids[f_seq & 3] = id;
            // (gather: the next K-step's wait of this wavefront covers these loads, the barrier
            // after it shows them to the others; the loader turns to the item K-steps later)
            if constexpr (GATHER) { if (id < n_items) fetch_rows(f_seq & 1, sgpr(id)); }
            f_seq = -1;
            MOE_WAIT_LGKMCNT(0);
        }
    };
    // (nothing may move across a phase boundary: neither memory operations nor matrix-core work)
    auto phase_barrier = [&]() __attribute__((always_inline)) {
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("" ::: "memory");
    };

    // ---- epilogue of one item.  acc[mi][ni][a][b][r]: row 16 a + 4 lq + r of the 32x32 block and
    // packed weight row 16 b + l16 of its 32, which is output column 2 l16 + b (the packed order of
    // 16-bit weights): every lane stores two adjacent outputs at once (one packed half pair, or two
    // floats), and one store instruction writes 32 columns of four rows.  Stores go through a
    // descriptor that ends with the tile's last row (the row part of a store's address is
    // range-checked only in the per-lane offset).
    constexpr int ES = HALF_IN ? 4 : 2;
    const unsigned ld_bytes = (unsigned)ld_out * ES;
    const unsigned st_voff = (unsigned)(wm * 32 + 4 * lq) * ld_bytes + (unsigned)(2 * l16) * ES;
    auto store_pair = [&](__amdgpu_buffer_rsrc_t ro, float lo, float hi, unsigned voff, unsigned soff) __attribute__((always_inline)) {
        if (HALF_IN) {
            u32x2 v = {__float_as_uint(lo), __float_as_uint(hi)};
            __builtin_amdgcn_raw_buffer_store_b64(v, ro, voff, soff, 0);
        } else {
            // hidden activations saturate at the largest half value instead of becoming infinite
            const f32x2 f = {__builtin_amdgcn_fmed3f(lo, -65504.f, 65504.f), __builtin_amdgcn_fmed3f(hi, -65504.f, 65504.f)};
            const f16x2 b = __builtin_convertvector(f, f16x2);            // nearest-even
            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, b), ro, voff, soff, 0);
        }
    };
    auto epilogue = [&](__amdgpu_buffer_rsrc_t ro, int mi_on, int n0) __attribute__((always_inline)) {
        // (the empty asm keeps the compiler from computing all row offsets once, up front, and
        // holding -- or spilling -- them across the whole kernel)
        unsigned st_base = st_voff;
        asm volatile("" : "+v"(st_base));
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            if (mi >= mi_on) continue;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int a = j >> 2, r = j & 3;
                const unsigned voff = st_base + (unsigned)(mi * (C::WM * 32) + a * 16 + r) * ld_bytes;
                if (EPI == MOE_EPI_SWIGLU) {
                    // packed weight rows alternate in blocks of 32: gate, up, gate, up, ...
#pragma unroll
                    for (int ni = 0; ni < NI; ni += 2) {
                        const int pc = n0 + wn * C::WTN + ni * 32;          // packed column of the gate block
                        if (pc < N)
                            store_pair(ro, silu_f(acc[mi][ni][a][0][r]) * acc[mi][ni + 1][a][0][r],
                                       silu_f(acc[mi][ni][a][1][r]) * acc[mi][ni + 1][a][1][r], voff, (unsigned)(pc / 2) * 2u);
                    }
                } else {
#pragma unroll
                    for (int ni = 0; ni < NI; ++ni) {
                        const int col = n0 + wn * C::WTN + ni * 32;
                        if (col < N) {
                            if (EPI == MOE_EPI_RELU)
                                store_pair(ro, fmaxf(acc[mi][ni][a][0][r], 0.f), fmaxf(acc[mi][ni][a][1][r], 0.f), voff, (unsigned)col * ES);
                            else
                                store_pair(ro, acc[mi][ni][a][0][r], acc[mi][ni][a][1][r], voff, (unsigned)col * ES);
                        }
                    }
                }
            }
        }
    };

    // ---- scatter epilogue.  The token and the gate value of every row of a tile wait in LDS
    // (rinfo[parity of the item][0: tokens, 1: gates][row]); they were fetched there by two small
    // global -> LDS loads during the item's first K-steps: first the tokens of the tile's rows,
    // then, indexed by them, the gate values.
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
    auto epilogue_scatter = [&](int par, int rc, int mi_on, int n0) __attribute__((always_inline)) {
        const int lane_row = wm * 32 + 4 * lq;
        const unsigned col_off = (unsigned)(2 * l16) * 4u;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            if (mi >= mi_on) continue;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int a = j >> 2, r = j & 3;
                const int rr = lane_row + mi * (C::WM * 32) + a * 16 + r;
                const unsigned tok = (unsigned)rinfo[par * 2 * BM + rr];
                const float gate = ((const float*)rinfo)[par * 2 * BM + BM + rr];
                // (a row past the tile's end gets an offset no output has: the range check drops it)
                const unsigned voff = (rr < rc ? tok * ld_bytes : 0x80000000u) + col_off;
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) {
                    const int col = n0 + wn * C::WTN + ni * 32;
                    if (col < N) store_pair(ry, acc[mi][ni][a][0][r] * gate, acc[mi][ni][a][1][r] * gate, voff, (unsigned)col * 4u);
                }
            }
        }
    };
    // the finished item: p_* describe it
    int p_mi_on = 0, p_n0 = 0, p_rc = 0, p_par = 0;
    __amdgpu_buffer_rsrc_t p_ro = make_rsrc(out, 0u);       // the previous item, stored in the next one's first phase
    auto finish_prev = [&]() __attribute__((always_inline)) {
        if constexpr (SCAT) epilogue_scatter(p_par, p_rc, p_mi_on, p_n0);
        else epilogue(p_ro, p_mi_on, p_n0);
    };

    // ---- prologue: RING-1 stages on their way, the first one landed
    if constexpr (GATHER) {                                 // source rows of the first two items: fetched and waited for
        if (wave == 0) {
            fetch_rows(0, first);
            const int second = sgpr(ids[1]);
            if (second < n_items) fetch_rows(1, second);
        }
        MOE_WAIT_VMCNT(0);
        __syncthreads();
    }
    load_item(first);
#pragma unroll
    for (int s = 0; s < RING - 1; ++s) issue();
    {
        const int younger = issued - 1;
        if (RING >= 4 && younger >= 2) MOE_WAIT_VMCNT(2 * C::LPS);
        else if (RING >= 3 && younger >= 1) MOE_WAIT_VMCNT(C::LPS);
        else MOE_WAIT_VMCNT(0);
        phase_barrier();
    }
    zero_acc();
    if (grp == 1) phase_barrier();                          // group 1 starts one phase late

    int item = first, c_seq = 0;
    while (item < n_items) {
        int cb, ti;
        locate(item, ti, cb);
        const moe_tile tile = tiles[bin_start + ti];
        const int rc = sgpr(tile.row_count < BM ? tile.row_count : BM);
        const int n0 = cb * BN;
        // 32-row blocks of this wavefront that hold real rows (wave-uniform)
        int mi_on = ((rc + 31) / 32 - wm + C::WM - 1) / C::WM;
        mi_on = mi_on < 0 ? 0 : (mi_on > MI ? MI : mi_on);
        const __amdgpu_buffer_rsrc_t ro =
            make_rsrc((const unsigned char*)out + (size_t)tile.row_begin * ld_bytes, (unsigned)(rc > 0 ? rc : 0) * ld_bytes);

        // One K-step of this wavefront: per chunk a memory phase and a multiply phase.
        auto k_step = [&](auto full, bool first_of_item, bool last_of_all) __attribute__((always_inline)) {
#pragma unroll
            for (int h = 0; h < PH; ++h) {
                // ---- memory phase: stage g's buffer is complete; the buffer of stage g-1 has been
                // read by everyone (it is refilled with stage g+RING-1)
                // Stores count in vmcnt like the loads.  With a ring of three or more stages the
                // wait for the next stage is taken BEFORE the previous item is stored (that stage
                // was issued a whole K-step ago), so the stores have until the next K-step's wait
                // to complete; with two stages the stores go first and the wait stays late.
                constexpr bool EARLY = RING >= 3;
                const bool store_now = h == 0 && first_of_item;
                if (store_now && !EARLY) {
                    finish_prev();
                    zero_acc();
                }
                mem_phase(c_buf, h);
                if (store_now && EARLY) {
                    wait_stage_after(g);
                    publish();
                    finish_prev();
                    zero_acc();
                }
                const bool waited = EARLY && first_of_item;
                if (grp == 1 && h == PH - 1 && !waited) wait_stage_after(g);
                MOE_WAIT_LGKMCNT(0);
                phase_barrier();
                // ---- multiply phase (at raised priority: the matrix instructions go first when the
                // other wavefront of the SIMD, in its memory phase, wants to issue in the same cycle)
                __builtin_amdgcn_s_setprio(1);
                mfma_chunk(full, mi_on);
                __builtin_amdgcn_s_setprio(0);
                if (grp == 0 && h == PH - 1 && !waited) {
                    wait_stage_after(g);
                    publish();
                }
                if (!(grp == 1 && last_of_all && h == PH - 1)) phase_barrier();
            }
            ++g;
            c_buf = c_buf + 1 == RING ? 0 : c_buf + 1;
        };

        // The id of the next item is known by this item's last K-step: the loader needed it
        // RING-1 K-steps ago.  (With one K-step per item there is no handing out: fixed stride.)
        int next = item + stride;
        auto run_item = [&](auto full) __attribute__((always_inline)) {
            if constexpr (SCAT) fetch_tokens(c_seq & 1, tile.row_begin, rc);
            k_step(full, true, KT == 1 && next >= n_items);
            for (int kt = 1; kt < KT; ++kt) {
                // (three K-steps of operand loads have been issued since: the waits of the last two
                // K-steps have covered the token load)
                if constexpr (SCAT) { if (kt == 3) fetch_gates(c_seq & 1); }
                bool last = false;
                if (kt == KT - 1) {
                    next = item_of(c_seq + 1, item);
                    last = next >= n_items;
                }
                k_step(full, false, last);
            }
        };
        if (mi_on == MI) run_item(std::true_type{});
        else run_item(std::false_type{});
        p_ro = ro;
        p_mi_on = mi_on;
        p_n0 = n0;
        p_rc = rc;
        p_par = c_seq & 1;
        item = next;
        ++c_seq;
    }
    if constexpr (SCAT) {                                   // (the last item's gates may have been fetched by other wavefronts)
        MOE_WAIT_VMCNT(0);
        __syncthreads();
    }
    finish_prev();
    leave();
    MOE_WAIT_VMCNT(0);                                      // (the trailing empty loads still target this LDS)
}

template <int EPI, int BM, int BN, int BK, int RING, int WM, int WN, int CS, bool GATHER>
__global__ __launch_bounds__(WM * WN * 64) void gemm_bf16_kernel(const uint16_t* __restrict__ a_mat, int K, int N,
                                                                  const void* const* __restrict__ w_ptrs,
                                                                  const moe_tile* __restrict__ tiles,
                                                                  int32_t* __restrict__ hdr, void* __restrict__ out,
                                                                  int ld_out, const int32_t* __restrict__ row_token,
                                                                  const float* __restrict__ row_gate, int out_rows,
                                                                  int a_div) {
    gemm_bf16_body<EPI, BM, BN, BK, RING, WM, WN, CS, GATHER>(a_mat, K, N, w_ptrs, tiles, hdr, out, ld_out, row_token,
                                                              row_gate, out_rows, a_div);
}

struct ScatterArgs {             // MOE_EPI_SCATTER: output row and gate value of every row, rows of the output
    const int32_t* row_token = nullptr;      // gather: source row (times a_div) of every row, rows of the source
    const float* row_gate = nullptr;
    int out_rows = 0;
    int a_div = 1;
};

template <int EPI, class C, bool GATHER = false>
int launch(const void* a, int K, int N, const void* const* w, const moe_tile* tiles, int32_t* hdr, void* out,
           int ld_out, const ScatterArgs& sc, hipStream_t st) {
    static_assert(C::SMEM <= 160 * 1024, "LDS ring too large");
    const int dev_ok = moe_check_gemm_device();
    if (dev_ok != MOE_OK) return dev_ok;
    auto kern = gemm_bf16_kernel<EPI, C::BM, C::BN, C::BK, C::RING, C::WM, C::WN, C::CS, GATHER>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)C::SMEM);
    if (e != hipSuccess) return moe_fail(MOE_ERR_HIP, "moe_grouped_ffn: shared memory attribute: %s", hipGetErrorString(e));
    hipLaunchKernelGGL(kern, dim3(MOE_GEMM_GRID), dim3(C::NTH), C::SMEM, st, (const uint16_t*)a, K, N, w, tiles, hdr, out,
                       ld_out, sc.row_token, sc.row_gate, sc.out_rows, sc.a_div);
    MOE_CHECK_LAUNCH("moe_grouped_ffn (bf16 GEMM)");
    return MOE_OK;
}

//          BM   BN  BK RING WM WN CS
typedef Cfg<256, 256, 64, 2, 2, 4, 2> Tall;     // wavefront tile 128 x 64, two phases pairs per K-step
typedef Cfg<128, 256, 64, 3, 2, 4, 4> Short;    // wavefront tile  64 x 64, one phase pair per K-step
typedef Cfg<128, 128, 64, 4, 2, 4, 4> Narrow;   // wavefront tile  64 x 32: twice the items, for few column blocks

template <int EPI>
int launch_tile(int tile_m, int narrow, const void* a, int K, int N, const void* const* w, const moe_tile* tiles,
                int32_t* hdr, void* out, int ld_out, const ScatterArgs& sc, hipStream_t st) {
    if (tile_m == 256) return launch<EPI, Tall>(a, K, N, w, tiles, hdr, out, ld_out, sc, st);
    if constexpr (EPI != MOE_EPI_SWIGLU) {          // (the SwiGLU epilogue needs a gate and an up block per wavefront)
        if (narrow) return launch<EPI, Narrow>(a, K, N, w, tiles, hdr, out, ld_out, sc, st);
    }
    return launch<EPI, Short>(a, K, N, w, tiles, hdr, out, ld_out, sc, st);
}

}  // namespace

// The persistent launch and its XCD mapping assume the whole MI355X: 256 compute units, dealt
// to 8 XCDs in turn.  Asked of the runtime once per device.
int moe_check_gemm_device() {
    static int cus[64] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return moe_fail(MOE_ERR_HIP, "moe_grouped_ffn: hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= 64) return moe_fail(MOE_ERR_UNSUPPORTED, "moe_grouped_ffn: device %d", dev);
    if (!cus[dev]) {
        int n = 0;
        e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return moe_fail(MOE_ERR_HIP, "moe_grouped_ffn: hipDeviceGetAttribute: %s", hipGetErrorString(e));
        cus[dev] = n;
    }
    if (cus[dev] != MOE_GEMM_GRID)
        return moe_fail(MOE_ERR_UNSUPPORTED, "moe_grouped_ffn: the bf16 kernels are built for a GPU of %d compute units, "
                        "device %d has %d", MOE_GEMM_GRID, dev, cus[dev]);
    return MOE_OK;
}

int moe_launch_gemm_bf16(int epi, int tile_m, int narrow, const void* a, int K, int N, const void* const* w,
                         const moe_tile* tiles, int32_t* hdr, void* out, int ld_out, hipStream_t st,
                         const int32_t* row_token, const float* row_gate, int out_rows) {
    ScatterArgs sc;
    if (epi == MOE_EPI_RELU) return launch_tile<MOE_EPI_RELU>(tile_m, narrow, a, K, N, w, tiles, hdr, out, ld_out, sc, st);
    if (epi == MOE_EPI_SWIGLU) return launch_tile<MOE_EPI_SWIGLU>(tile_m, narrow, a, K, N, w, tiles, hdr, out, ld_out, sc, st);
    if (epi == MOE_EPI_SCATTER) {
        sc.row_token = row_token;
        sc.row_gate = row_gate;
        sc.out_rows = out_rows;
        return launch_tile<MOE_EPI_SCATTER>(tile_m, narrow, a, K, N, w, tiles, hdr, out, ld_out, sc, st);
    }
    return launch_tile<MOE_EPI_STORE>(tile_m, narrow, a, K, N, w, tiles, hdr, out, ld_out, sc, st);
}

int moe_launch_gemm_bf16_gather(int epi, const void* x, int x_rows, int K, int N, const void* const* w,
                                const moe_tile* tiles, int32_t* hdr, void* out, int ld_out, hipStream_t st,
                                const int32_t* row_src, int src_div) {
    ScatterArgs sc;
    sc.row_token = row_src;
    sc.out_rows = x_rows;
    sc.a_div = src_div;
    if (epi == MOE_EPI_SWIGLU) return launch<MOE_EPI_SWIGLU, Short, true>(x, K, N, w, tiles, hdr, out, ld_out, sc, st);
    return launch<MOE_EPI_RELU, Short, true>(x, K, N, w, tiles, hdr, out, ld_out, sc, st);
}
