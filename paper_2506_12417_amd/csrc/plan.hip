// moe_plan_tiles: the load-aware schedule of section 4.2 (Alg. 2) with the GPU's XCDs as bins.
//
// One work-group, everything in LDS, nothing on the host: S[e][g] (rows of expert e run by bin
// g) is built by an initial placement, rebalanced by Alg. 2's loop executed by one wavefront
// (argmax / argmin are wave reductions), then cut into tiles of at most tile_m rows, bin after
// bin, heaviest block first.  The paper's scheduler runs as host-driven tensor ops and costs
// 20-30 % of its layer time (section 5.3.1); here it is a few microseconds on the device.
#include "common.h"
#include "permute_rank.h"
#include <climits>
#include <type_traits>

namespace {

constexpr int NTH = 256;   // >= MOE_MAX_EXPERTS: one thread per expert

// weight of a block of n rows: its tiles (MOE_PLAN_BALANCED) or its rows
__device__ __forceinline__ int weight_of(int n, int tile_m, bool in_tiles) {
    return in_tiles ? (n + tile_m - 1) / tile_m : n;
}

// Loads are kept below 2^26 so that (load << 5 | bin) fits 32 bits (bins < 32): one reduction gives both the
// extreme load and, among equal loads, the lowest bin.
constexpr int BIN_BITS = 5;
__device__ __forceinline__ void argmin_bin(int tg, int lane, int G, int& g, int& v) {
    unsigned key = lane < G ? (((unsigned)tg << BIN_BITS) | (unsigned)lane) : 0xffffffffu;
    key = moe_wave_min_u32(key);
    g = (int)(key & ((1u << BIN_BITS) - 1u));
    v = (int)(key >> BIN_BITS);
}
__device__ __forceinline__ void argmax_bin(int tg, int lane, int G, int& g, int& v) {
    unsigned key = lane < G ? (((unsigned)tg << BIN_BITS) | (unsigned)(MOE_MAX_BINS - 1 - lane)) : 0u;
    key = moe_wave_max_u32(key);
    g = MOE_MAX_BINS - 1 - (int)(key & ((1u << BIN_BITS) - 1u));
    v = (int)(key >> BIN_BITS);
}

// which experts take part in a plan: bit e of word e / 32
struct ExpertMask {
    uint32_t w[MOE_MAX_EXPERTS / 32];
};

// arguments of the launch that also ranks (moe_permute_plan)
struct RankArgs {
    const int32_t* idx;          // expert of every assignment
    int nbits, nb;               // bits of an expert id, blocks of moe_rank::PB assignments
    int32_t *counts, *offsets, *perm, *inv_perm;
};

// MERGED: one launch does the stable rank of moe_permute (work-groups 0 .. nb-1, moe_rank::rank_body
// in the mode that counts by itself) AND the plan (work-group nb, which also counts the experts
// of all assignments itself instead of reading counts and offsets): the two need nothing from
// each other, so the plan's serial loops pass under the ranking instead of after it.
template <bool MERGED>
__global__ __launch_bounds__(NTH) void plan_kernel(const int32_t* __restrict__ counts,
                                                   const int32_t* __restrict__ offsets, int E, int A, int tile_m,
                                                   int G, int q, int policy, ExpertMask mask,
                                                   moe_tile* __restrict__ tiles, int capacity,
                                                   int32_t* __restrict__ hdr, int32_t* __restrict__ sched, RankArgs ra) {
    static_assert(NTH == moe_rank::NTH, "one block size for both roles");
    if (MERGED) {
        if ((int)blockIdx.x < ra.nb) {
            moe_rank::rank_body<2>(ra.idx, A, E, ra.nbits, ra.nb, nullptr, ra.counts, ra.offsets, ra.perm, ra.inv_perm);
            return;
        }
    }
    __shared__ int cnt[MOE_MAX_EXPERTS], order[MOE_MAX_EXPERTS], row0[MOE_MAX_EXPERTS];
    __shared__ __attribute__((aligned(16))) int cost[MOE_MAX_EXPERTS + 4];
    // (not volatile: volatile accesses are compiled to flat instructions that are waited for one by
    // one; where lanes of the serial wavefront exchange values through S a wavefront fence orders them)
    __shared__ int S[MOE_MAX_EXPERTS * MOE_MAX_BINS];
    // non-empty (expert, bin) blocks, one segment per bin: rows and expert id
    __shared__ int blk_n[MOE_MAX_EXPERTS * MOE_MAX_BINS];
    __shared__ unsigned char blk_e[MOE_MAX_EXPERTS * MOE_MAX_BINS];
    __shared__ int blk_t[MOE_MAX_EXPERTS * MOE_MAX_BINS];               // tiles of the block
    __shared__ short blk_key[MOE_MAX_EXPERTS * MOE_MAX_BINS];           // rank of the block among its kind in its bin
    __shared__ int load[MOE_MAX_BINS], bin_blocks[MOE_MAX_BINS + 1], bin_cursor[MOE_MAX_BINS], bin_tiles[MOE_MAX_BINS + 1], bin_long[MOE_MAX_BINS];
    __shared__ int s_tavg, s_moves;
    const int tid = threadIdx.x, lane = tid & 63;
    const bool by_cost = (policy == MOE_PLAN_BALANCED);

    for (int i = tid; i < E * G; i += NTH) S[i] = 0;
    if (tid < G) { load[tid] = 0; bin_blocks[tid] = 0; bin_cursor[tid] = 0; bin_tiles[tid] = 0; }
    if (MERGED) {
        // this work-group's own count of every expert (cnt) and its first row (row0: exclusive prefix)
        cnt[tid] = 0;
        __syncthreads();
        moe_rank::count_experts(ra.idx, A, E, 0, nullptr, cnt);
        __syncthreads();
        const int total = tid < E ? cnt[tid] : 0;
        // inclusive scan over the experts (Hillis-Steele; order[] and cost[] are not in use yet)
        int* buf[2] = {order, cost};
        buf[0][tid] = total;
        __syncthreads();
        int cur = 0;
        for (int step = 1; step < MOE_MAX_EXPERTS; step <<= 1) {
            const int v = buf[cur][tid] + (tid >= step ? buf[cur][tid - step] : 0);
            buf[cur ^ 1][tid] = v;
            cur ^= 1;
            __syncthreads();
        }
        const int first = buf[cur][tid] - total;
        __syncthreads();
        if (tid < E) {
            const int c = ((mask.w[tid >> 5] >> (tid & 31)) & 1u) ? total : 0;
            cnt[tid] = c;
            row0[tid] = first;
            cost[tid] = weight_of(c, tile_m, by_cost);
        }
    } else if (tid < E) {
        int c = ((mask.w[tid >> 5] >> (tid & 31)) & 1u) ? counts[tid] : 0;    // experts left out count as empty
        cnt[tid] = c;
        row0[tid] = offsets[tid];                  // (fetched now: a global load at the end would be waited for in full)
        cost[tid] = weight_of(c, tile_m, by_cost);
    }
    if (tid < 4) cost[E + tid] = -1;
    if (tid == 0) s_moves = 0;
    __syncthreads();

    // ---- initial placement (the paper's initialAssign)
    if (policy == MOE_PLAN_BALANCED) {
        if (tid < E) {   // experts by falling weight, equal weights by rising id
            const int c = cost[tid];
            int r = 0;
            const int4* c4 = (const int4*)cost;                 // (entries past E are never ahead: -1)
#pragma unroll 4
            for (int e2 = 0; e2 < E; e2 += 4) {
                const int4 v = c4[e2 >> 2];
                r += (v.x > c || (v.x == c && e2 < tid)) ? 1 : 0;
                r += (v.y > c || (v.y == c && e2 + 1 < tid)) ? 1 : 0;
                r += (v.z > c || (v.z == c && e2 + 2 < tid)) ? 1 : 0;
                r += (v.w > c || (v.w == c && e2 + 3 < tid)) ? 1 : 0;
            }
            order[r] = tid;
        }
        __syncthreads();
        if (tid < 64) {
            // Each expert whole, on the least loaded bin so far.  The loop is serial and a lone
            // wavefront issues an instruction only every few cycles, so what counts is the number of
            // instructions per expert.  The bins are a list of keys (load << BIN_BITS | bin) sorted
            // by rising key in scalar registers: the head is the least loaded bin (the lowest one
            // among equals); it takes the expert and sinks back to its place by compare-and-swap with
            // its successors.  Unused entries are all ones and stay at the end.  Lane r % 64 notes
            // the bin of the r-th expert; the lanes write S afterwards, all at once.
            constexpr int NJ = MOE_MAX_EXPERTS / 64;
            int ord[NJ], cst[NJ], cn[NJ], bin_of[NJ];
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                const int r = lane + 64 * j;
                ord[j] = r < E ? order[r] : 0;
                cst[j] = r < E ? cost[ord[j]] : 0;
                cn[j] = r < E ? cnt[ord[j]] : 0;
                bin_of[j] = -1;
            }
            int tg = 0;
            auto place = [&](auto max_bins) {
                constexpr int MB = decltype(max_bins)::value;
                unsigned key[MB];
#pragma unroll
                for (int i = 0; i < MB; ++i) key[i] = i < G ? (unsigned)i : 0xffffffffu;
#pragma unroll
                for (int j = 0; j < NJ; ++j) {
                    const int n = E - 64 * j < 64 ? E - 64 * j : 64;
                    for (int r = 0; r < n; ++r) {
                        const unsigned c = (unsigned)__builtin_amdgcn_readlane(cst[j], r);
                        if (c == 0) break;
                        bin_of[j] = lane == r ? (int)(key[0] & ((1u << BIN_BITS) - 1u)) : bin_of[j];
                        key[0] += c << BIN_BITS;
#pragma unroll
                        for (int i = 0; i + 1 < MB; ++i) {
                            const unsigned lo = key[i] < key[i + 1] ? key[i] : key[i + 1];
                            const unsigned hi = key[i] < key[i + 1] ? key[i + 1] : key[i];
                            key[i] = lo;
                            key[i + 1] = hi;
                        }
                    }
                }
#pragma unroll
                for (int i = 0; i < MB; ++i)
                    if (i < G && lane == (int)(key[i] & ((1u << BIN_BITS) - 1u))) tg = (int)(key[i] >> BIN_BITS);
            };
            if (G <= 8) place(std::integral_constant<int, 8>{});
            else place(std::integral_constant<int, MOE_MAX_BINS>{});
#pragma unroll
            for (int j = 0; j < NJ; ++j)
                if (bin_of[j] >= 0) S[ord[j] * G + bin_of[j]] = cn[j];
            if (lane < G) load[lane] = tg;
        }
    } else if (policy == MOE_PLAN_EVEN_SPLIT) {
        if (tid < E) {
            const int c = cnt[tid];
            for (int g = 0; g < G; ++g) {
                const int n = c / G + (g < c % G ? 1 : 0);
                S[tid * G + g] = n;
                atomicAdd(&load[g], n);
            }
        }
    } else {             // contiguous blocks of experts per bin, or experts dealt to the bins in turn
        if (tid < E) {
            const int g = policy == MOE_PLAN_ROUND_ROBIN ? tid % G : (int)(((long long)tid * G) / E);
            S[tid * G + g] = cnt[tid];
            atomicAdd(&load[g], cnt[tid]);
        }
    }
    __syncthreads();

    // ---- Alg. 2: move rows of the largest block of the most loaded bin to the least loaded bin
    if (tid < 64) {
        int tg = lane < G ? load[lane] : 0;
        const int t_avg = (int)(moe_wave_sum_u32((unsigned)tg) / (unsigned)G);
        int moves = 0;
        // the largest block of bin g (most rows, lowest expert among equals)
        auto largest_block = [&](int g, int& e_max, int& rows) {
            if (A < (1 << 24)) {
                // rows and expert in one key (rows << 8 | 255 - expert): one pass, one reduction
                unsigned key = 0;
                for (int e = lane; e < E; e += 64) {
                    const unsigned k2 = ((unsigned)S[e * G + g] << 8) | (unsigned)(255 - e);
                    key = k2 > key ? k2 : key;
                }
                key = moe_wave_max_u32(key);
                rows = (int)(key >> 8);
                e_max = 255 - (int)(key & 255u);
                return;
            }
            int best = -1;
            for (int e = lane; e < E; e += 64) {
                const int sv = S[e * G + g];
                best = sv > best ? sv : best;
            }
            rows = (int)moe_wave_max_u32((unsigned)(best + 1)) - 1;
            unsigned first = 0xffffffffu;
            for (int e = lane; e < E; e += 64)
                if (S[e * G + g] == rows) { first = (unsigned)e; break; }
            e_max = (int)moe_wave_min_u32(first);
        };
        const int max_iters = E * G + 16;
        if (policy == MOE_PLAN_BALANCED) {
            // in tiles: until the most and the least loaded bin differ by at most one tile, half
            // the difference (in whole tiles, or the whole block) moves from the one to the other
            for (int it = 0; it < max_iters; ++it) {
                int g_max, t_max, g_min, t_min;
                argmax_bin(tg, lane, G, g_max, t_max);
                argmin_bin(tg, lane, G, g_min, t_min);
                const int diff = t_max - t_min;
                if (diff <= 1) break;
                int e_max, n_from;
                largest_block(g_max, e_max, n_from);
                const int n_to = S[e_max * G + g_min];
                const int tiles_from = weight_of(n_from, tile_m, true);
                const int m = tiles_from < diff / 2 ? tiles_from : diff / 2;
                const int t_s = m == tiles_from ? n_from : m * tile_m;
                const int d_from = tiles_from - weight_of(n_from - t_s, tile_m, true);
                const int d_to = weight_of(n_to + t_s, tile_m, true) - weight_of(n_to, tile_m, true);
                if (lane == 0) {
                    S[e_max * G + g_max] = n_from - t_s;
                    S[e_max * G + g_min] = n_to + t_s;
                }
                __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");   // the next round's lanes read these
                if (lane == g_max) tg -= d_from;
                if (lane == g_min) tg += d_to;
                ++moves;
            }
        } else if (policy == MOE_PLAN_HARMOENY) {
            // Alg. 2 as printed, loads in rows
            for (int it = 0; it < max_iters; ++it) {
                int g_max, t_max;
                argmax_bin(tg, lane, G, g_max, t_max);
                if (t_max <= t_avg) break;                       // no bin above the average
                int e_max, t_move;
                largest_block(g_max, e_max, t_move);
                if (t_move < q) break;
                int g_min, t_min;
                argmin_bin(tg, lane, G, g_min, t_min);
                if (g_min == g_max || t_min + q > t_avg) break;
                const int t_s = t_move < t_avg - t_min ? t_move : t_avg - t_min;
                const int n_from = S[e_max * G + g_max], n_to = S[e_max * G + g_min];
                if (lane == 0) {
                    S[e_max * G + g_max] = n_from - t_s;
                    S[e_max * G + g_min] = n_to + t_s;
                }
                __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");   // the next round's lanes read these
                if (lane == g_max) tg -= t_s;
                if (lane == g_min) tg += t_s;
                ++moves;
            }
        }
        if (lane < G) load[lane] = tg;
        if (lane == 0) { s_moves = moves; s_tavg = t_avg; }
    }
    __syncthreads();

    // ---- the non-empty blocks of every bin, gathered into per-bin segments (any order)
    // Thread t serves bin t % G and the experts t / G, t / G + NTH / G, ...: it counts its blocks
    // and reserves their places with ONE atomic per pass (an atomic per block made 32 lanes of a
    // wavefront queue up on each of the few bin counters).
    if (sched)
        for (int p = tid; p < E * G; p += NTH) sched[p] = S[p];
    const int per_bin = NTH / G;                             // threads per bin
    const int my_g = tid % G, my_j = tid / G;
    const bool serving = my_j < per_bin;
    int my_blocks = 0;
    if (serving)
        for (int e = my_j; e < E; e += per_bin) my_blocks += S[e * G + my_g] > 0;
    if (my_blocks) atomicAdd(&bin_blocks[my_g], my_blocks);
    __syncthreads();
    if (tid == 0) {
        int run = 0;
        for (int g = 0; g < G; ++g) { const int c = bin_blocks[g]; bin_blocks[g] = run; run += c; }
        bin_blocks[G] = run;
    }
    __syncthreads();
    if (my_blocks) {
        int at = bin_blocks[my_g] + atomicAdd(&bin_cursor[my_g], my_blocks), my_tiles = 0;
        for (int e = my_j; e < E; e += per_bin) {
            const int n = S[e * G + my_g];
            if (n > 0) {
                const int nt = (n + tile_m - 1) / tile_m;
                blk_n[at] = n;
                blk_e[at] = (unsigned char)e;
                blk_t[at] = nt;
                blk_key[at] = (short)my_g;                   // (the bin, until the block's rank replaces it)
                my_tiles += nt;
                ++at;
            }
        }
        atomicAdd(&bin_tiles[my_g], my_tiles);
    }
    __syncthreads();

    // ---- tiles; one block per thread.  Inside a bin the blocks of several tiles ("long": their
    // tiles share the expert's weights through the XCD's L2, the arithmetic bounds them) are
    // spread evenly among the blocks of one tile ("short": each streams its expert's weights
    // from HBM), so that the work-groups of an XCD, which take the blocks in this order, mix the
    // two kinds at all times instead of first computing with the memory idle and then waiting
    // for the memory.  Each kind is ordered by falling row count, then expert id; the i-th of
    // n_long long blocks has the key (2i+1)/n_long, the j-th short one (2j+1)/n_short, and the
    // blocks are listed by rising key, a long one first among equals.  Where the long blocks
    // outnumber the short ones the bin is bound by arithmetic anyway, and the plain order by
    // falling row count (then expert id) is kept: it leaves the smallest blocks for the end,
    // where they even out the finishing times of the work-groups.
    const int n_blocks = bin_blocks[G];
    for (int b = tid; b < n_blocks; b += NTH) {
        const int g = blk_key[b];
        const int n = blk_n[b], e = blk_e[b];
        const bool is_long = n > tile_m;
        int rank = 0, n_long = 0;
        // (bitwise, not short-circuit logic: both reads go out together and the loop has no branches)
        for (int o = bin_blocks[g]; o < bin_blocks[g + 1]; ++o) {
            const int n2 = blk_n[o], e2 = blk_e[o];
            const int long2 = n2 > tile_m;
            n_long += long2;
            rank += (long2 == (int)is_long) & ((n2 > n) | ((n2 == n) & (e2 < e)));
        }
        blk_key[b] = (short)(rank | (g << 9) | (is_long ? 0x4000 : 0));
        bin_long[g] = n_long;                      // (every block of the bin writes the same number)
    }
    if (tid == 0) {
        int run = 0;
        for (int g = 0; g < G; ++g) {
            const int t = bin_tiles[g];
            bin_tiles[g] = run;
            hdr[4 + g] = run < capacity ? run : capacity;
            run += t;
        }
        bin_tiles[G] = run;
        hdr[4 + G] = run < capacity ? run : capacity;
        hdr[0] = run < capacity ? run : capacity;
        hdr[1] = G;
        hdr[2] = s_moves;
        hdr[3] = s_tavg;
    }
    __syncthreads();
    for (int b = tid; b < n_blocks; b += NTH) {
        const int g = (blk_key[b] >> 9) & (MOE_MAX_BINS - 1);
        const int n = blk_n[b], e = blk_e[b];
        const bool is_long = n > tile_m;
        const int n_long = bin_long[g];
        const int n_short = bin_blocks[g + 1] - bin_blocks[g] - n_long;
        // one number per block that rises along the listing: long blocks first, or the merged keys
        // (doubled, a short block's one higher, so that a long one precedes a short one of equal key)
        const bool merged = n_long > 0 && n_long <= n_short;
        auto place = [&](int k) {
            const bool lng = (k & 0x4000) != 0;
            const int rank = k & 0x1ff;
            return merged ? 2 * (2 * rank + 1) * (lng ? n_short : n_long) + (lng ? 0 : 1) : (lng ? rank : 0x4000 + rank);
        };
        const int mine = place(blk_key[b]);
        int before = 0;
        for (int o = bin_blocks[g]; o < bin_blocks[g + 1]; ++o) {
            const int k2 = blk_key[o], t2 = blk_t[o];
            before += place(k2) < mine ? t2 : 0;
        }
        int row = row0[e];
        for (int g2 = 0; g2 < g; ++g2) row += S[e * G + g2];
        const int nt = blk_t[b];
        for (int i = 0; i < nt; ++i) {
            const int at = bin_tiles[g] + before + i;
            if (at < capacity) {
                moe_tile t;
                t.expert = e;
                t.row_begin = row + i * tile_m;
                t.row_count = (n - i * tile_m) < tile_m ? (n - i * tile_m) : tile_m;
                t.bin = g;
                tiles[at] = t;
            }
        }
    }
    if (tid < G) hdr[4 + MOE_MAX_BINS + 1 + tid] = load[tid];
    if (tid <= MOE_MAX_BINS) hdr[MOE_PLAN_HDR_CTR + tid] = 0;     // work counters of the FFN kernels
}


// moe_rebalance: Alg. 2 as printed, with its three-dimensional schedule S[g_from][e][g_to], for
// G GPUs.  One work-group; S lives in LDS; the loop runs in one wavefront with the destination
// GPUs (then the source GPUs, then the experts) across its lanes.
__global__ __launch_bounds__(NTH) void rebalance_kernel(const int32_t* __restrict__ s_in, int G_src, int E, int G, int q,
                                                        int32_t* __restrict__ s_out, int32_t* __restrict__ info) {
    extern __shared__ int Sx[];                              // [G_src][E][G]
    __shared__ int from_load[MOE_MAX_BINS * MOE_MAX_BINS];   // [g_from][g_to] = sum_e S
    __shared__ int load[MOE_MAX_BINS];
    const int tid = threadIdx.x, lane = tid & 63;
    const int n = G_src * E * G;
    for (int i = tid; i < n; i += NTH) Sx[i] = s_in[i];
    __syncthreads();
    for (int p = tid; p < G_src * G; p += NTH) {
        const int gf = p / G, g = p % G;
        int sum = 0;
        for (int e = 0; e < E; ++e) sum += Sx[(gf * E + e) * G + g];
        from_load[gf * MOE_MAX_BINS + g] = sum;
    }
    __syncthreads();
    if (tid < G) {
        int sum = 0;
        for (int gf = 0; gf < G_src; ++gf) sum += from_load[gf * MOE_MAX_BINS + tid];
        load[tid] = sum;
    }
    __syncthreads();
    if (tid < 64) {
        int tg = lane < G ? load[lane] : 0;
        const int t_avg = (int)(moe_wave_sum_u32((unsigned)tg) / (unsigned)G);
        int moves = 0, why = 0;                              // why the loop ended: 0 balanced, 1 block < q, 2 no room, 3 cap
        const int max_iters = n + 16;
        int it = 0;
        for (; it < max_iters; ++it) {
            int g_max, t_max;
            argmax_bin(tg, lane, G, g_max, t_max);
            if (t_max <= t_avg) break;
            // the source GPU that sends most to g_max, then its largest expert block there
            int g_from, f_max;
            argmax_bin(lane < G_src ? from_load[lane * MOE_MAX_BINS + g_max] : 0, lane, G_src, g_from, f_max);
            int best = -1;
            for (int e = lane; e < E; e += 64) {
                const int sv = Sx[(g_from * E + e) * G + g_max];
                best = sv > best ? sv : best;
            }
            const int t_move = (int)moe_wave_max_u32((unsigned)(best + 1)) - 1;
            unsigned first = 0xffffffffu;
            for (int e = lane; e < E; e += 64)
                if (Sx[(g_from * E + e) * G + g_max] == t_move) { first = (unsigned)e; break; }
            const int e_max = (int)moe_wave_min_u32(first);
            if (t_move < q) { why = 1; break; }
            int g_min, t_min;
            argmin_bin(tg, lane, G, g_min, t_min);
            if (g_min == g_max || t_min + q > t_avg) { why = 2; break; }
            const int t_s = t_move < t_avg - t_min ? t_move : t_avg - t_min;
            if (lane == 0) {
                Sx[(g_from * E + e_max) * G + g_max] -= t_s;
                Sx[(g_from * E + e_max) * G + g_min] += t_s;
                from_load[g_from * MOE_MAX_BINS + g_max] -= t_s;
                from_load[g_from * MOE_MAX_BINS + g_min] += t_s;
            }
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
            if (lane == g_max) tg -= t_s;
            if (lane == g_min) tg += t_s;
            ++moves;
        }
        if (it == max_iters) why = 3;
        if (info) {
            if (lane == 0) { info[0] = moves; info[1] = t_avg; info[2] = why; }
            if (lane < G) info[4 + lane] = tg;
        }
    }
    __syncthreads();
    for (int i = tid; i < n; i += NTH) s_out[i] = Sx[i];
}

}  // namespace

extern "C" int moe_plan_capacity(int A, int E, int tile_m, int n_bins) {
    if (A < 0 || E < 1 || tile_m < 1 || n_bins < 1) return 0;
    long long c = ((long long)A + tile_m - 1) / tile_m + (long long)E * n_bins;
    return c > INT_MAX ? INT_MAX : (int)c;
}

static int plan_impl(const char* who, const int32_t* counts, const int32_t* offsets, int E, int A, int tile_m, int n_bins,
                     int q_tokens, int policy, const ExpertMask& mask, moe_tile* tiles, int tile_capacity,
                     int32_t* plan_hdr, int32_t* sched, void* stream) {
    MOE_REQUIRE(E >= 1 && A >= 0, MOE_ERR_ARG, "%s: E=%d A=%d", who, E, A);
    MOE_REQUIRE((long long)A + (long long)E * q_tokens < (1ll << 26), MOE_ERR_UNSUPPORTED,
                "%s: A + E*q_tokens = %lld is not below 2^26", who, (long long)A + (long long)E * q_tokens);
    MOE_REQUIRE(E <= MOE_MAX_EXPERTS, MOE_ERR_UNSUPPORTED, "%s: E=%d > %d", who, E, MOE_MAX_EXPERTS);
    MOE_REQUIRE(n_bins >= 1 && n_bins <= MOE_MAX_BINS, MOE_ERR_ARG, "%s: n_bins=%d outside [1,%d]", who, n_bins, MOE_MAX_BINS);
    MOE_REQUIRE(tile_m >= 1 && q_tokens >= 1, MOE_ERR_ARG, "%s: tile_m=%d q_tokens=%d must be >= 1", who, tile_m, q_tokens);
    MOE_REQUIRE(policy >= MOE_PLAN_BALANCED && policy <= MOE_PLAN_ROUND_ROBIN, MOE_ERR_ARG, "%s: policy %d", who, policy);
    MOE_REQUIRE(counts && offsets && tiles && plan_hdr, MOE_ERR_ARG, "%s: null pointer", who);
    MOE_REQUIRE(tile_capacity >= moe_plan_capacity(A, E, tile_m, n_bins), MOE_ERR_CAPACITY,
                "%s: tile_capacity %d < %d", who, tile_capacity, moe_plan_capacity(A, E, tile_m, n_bins));
    hipLaunchKernelGGL(plan_kernel<false>, dim3(1), dim3(NTH), 0, (hipStream_t)stream, counts, offsets, E, A, tile_m, n_bins,
                       q_tokens, policy, mask, tiles, tile_capacity, plan_hdr, sched, RankArgs());
    MOE_CHECK_LAUNCH(who);
    return MOE_OK;
}

extern "C" int moe_permute_plan(const int32_t* expert_idx, int T, int E, int k, int32_t* counts, int32_t* offsets,
                                int32_t* perm, int32_t* inv_perm, int tile_m, int n_bins, int q_tokens, int policy,
                                moe_tile* tiles, int tile_capacity, int32_t* plan_hdr, int32_t* sched, void* stream) {
    const char* who = "moe_permute_plan";
    MOE_REQUIRE(T >= 1 && E >= 1 && k >= 1, MOE_ERR_ARG, "%s: T=%d E=%d k=%d", who, T, E, k);
    MOE_REQUIRE(E <= MOE_MAX_EXPERTS, MOE_ERR_UNSUPPORTED, "%s: E=%d > %d", who, E, MOE_MAX_EXPERTS);
    MOE_REQUIRE((long long)T * k <= MOE_PERMUTE_PLAN_MAX, MOE_ERR_UNSUPPORTED,
                "%s: T*k = %lld assignments, at most %d (use moe_permute and moe_plan_tiles)", who, (long long)T * k, MOE_PERMUTE_PLAN_MAX);
    const int A = T * k;
    MOE_REQUIRE((long long)A + (long long)E * q_tokens < (1ll << 26), MOE_ERR_UNSUPPORTED,
                "%s: A + E*q_tokens = %lld is not below 2^26", who, (long long)A + (long long)E * q_tokens);
    MOE_REQUIRE(n_bins >= 1 && n_bins <= MOE_MAX_BINS, MOE_ERR_ARG, "%s: n_bins=%d outside [1,%d]", who, n_bins, MOE_MAX_BINS);
    MOE_REQUIRE(tile_m >= 1 && q_tokens >= 1, MOE_ERR_ARG, "%s: tile_m=%d q_tokens=%d must be >= 1", who, tile_m, q_tokens);
    MOE_REQUIRE(policy >= MOE_PLAN_BALANCED && policy <= MOE_PLAN_ROUND_ROBIN, MOE_ERR_ARG, "%s: policy %d", who, policy);
    MOE_REQUIRE(expert_idx && counts && offsets && perm && inv_perm && tiles && plan_hdr, MOE_ERR_ARG, "%s: null pointer", who);
    MOE_REQUIRE(tile_capacity >= moe_plan_capacity(A, E, tile_m, n_bins), MOE_ERR_CAPACITY,
                "%s: tile_capacity %d < %d", who, tile_capacity, moe_plan_capacity(A, E, tile_m, n_bins));
    ExpertMask all;
    for (int i = 0; i < MOE_MAX_EXPERTS / 32; ++i) all.w[i] = 0xffffffffu;
    RankArgs ra;
    ra.idx = expert_idx;
    ra.nb = (A + moe_rank::PB - 1) / moe_rank::PB;
    ra.nbits = 0;
    while ((1 << ra.nbits) < E) ++ra.nbits;
    ra.counts = counts;
    ra.offsets = offsets;
    ra.perm = perm;
    ra.inv_perm = inv_perm;
    hipLaunchKernelGGL(plan_kernel<true>, dim3(ra.nb + 1), dim3(NTH), sizeof(int) * moe_rank::CHUNKS * E, (hipStream_t)stream,
                       (const int32_t*)nullptr, (const int32_t*)nullptr, E, A, tile_m, n_bins, q_tokens, policy, all, tiles,
                       tile_capacity, plan_hdr, sched, ra);
    MOE_CHECK_LAUNCH(who);
    return MOE_OK;
}

extern "C" int moe_plan_tiles(const int32_t* counts, const int32_t* offsets, int E, int A, int tile_m, int n_bins,
                              int q_tokens, int policy, moe_tile* tiles, int tile_capacity, int32_t* plan_hdr,
                              int32_t* sched, void* stream) {
    ExpertMask all;
    for (auto& w : all.w) w = 0xffffffffu;
    return plan_impl("moe_plan_tiles", counts, offsets, E, A, tile_m, n_bins, q_tokens, policy, all, tiles, tile_capacity,
                     plan_hdr, sched, stream);
}

extern "C" int moe_plan_tiles_subset(const int32_t* counts, const int32_t* offsets, int E, int A, int tile_m, int n_bins,
                                     int q_tokens, int policy, const int32_t* expert_ids, int n_ids, moe_tile* tiles,
                                     int tile_capacity, int32_t* plan_hdr, int32_t* sched, void* stream) {
    MOE_REQUIRE(n_ids >= 0 && (n_ids == 0 || expert_ids), MOE_ERR_ARG, "moe_plan_tiles_subset: n_ids=%d", n_ids);
    MOE_REQUIRE(E >= 1 && E <= MOE_MAX_EXPERTS, E < 1 ? MOE_ERR_ARG : MOE_ERR_UNSUPPORTED, "moe_plan_tiles_subset: E=%d", E);
    ExpertMask m;
    for (auto& w : m.w) w = 0u;
    for (int i = 0; i < n_ids; ++i) {
        const int e = expert_ids[i];
        MOE_REQUIRE(e >= 0 && e < E, MOE_ERR_ARG, "moe_plan_tiles_subset: expert id %d outside [0,%d)", e, E);
        m.w[e >> 5] |= 1u << (e & 31);
    }
    return plan_impl("moe_plan_tiles_subset", counts, offsets, E, A, tile_m, n_bins, q_tokens, policy, m, tiles,
                     tile_capacity, plan_hdr, sched, stream);
}

extern "C" int moe_rebalance(const int32_t* s_initial, int G_src, int E, int G, int q_tokens, int32_t* s_out, int32_t* info,
                             void* stream) {
    MOE_REQUIRE(G_src >= 1 && G_src <= MOE_MAX_BINS && G >= 1 && G <= MOE_MAX_BINS, MOE_ERR_ARG,
                "moe_rebalance: G_src=%d G=%d outside [1,%d]", G_src, G, MOE_MAX_BINS);
    MOE_REQUIRE(E >= 1 && q_tokens >= 1, MOE_ERR_ARG, "moe_rebalance: E=%d q_tokens=%d must be >= 1", E, q_tokens);
    MOE_REQUIRE(E <= MOE_MAX_EXPERTS, MOE_ERR_UNSUPPORTED, "moe_rebalance: E=%d > %d", E, MOE_MAX_EXPERTS);
    const size_t bytes = (size_t)G_src * E * G * sizeof(int32_t);
    MOE_REQUIRE(bytes <= 128 * 1024, MOE_ERR_UNSUPPORTED, "moe_rebalance: S of %zu bytes does not fit the work-group's memory", bytes);
    MOE_REQUIRE(s_initial && s_out, MOE_ERR_ARG, "moe_rebalance: null pointer");
    if (bytes > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(rebalance_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
        if (e != hipSuccess) return moe_fail(MOE_ERR_HIP, "moe_rebalance: shared memory attribute: %s", hipGetErrorString(e));
    }
    hipLaunchKernelGGL(rebalance_kernel, dim3(1), dim3(NTH), bytes, (hipStream_t)stream, s_initial, G_src, E, G, q_tokens,
                       s_out, info);
    MOE_CHECK_LAUNCH("moe_rebalance");
    return MOE_OK;
}
