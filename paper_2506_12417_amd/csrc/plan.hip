// moe_plan_tiles: the load-aware schedule of section 4.2 (Alg. 2) with the GPU's XCDs as bins.
//
// One work-group, everything in LDS, nothing on the host: S[e][g] (rows of expert e run by bin
// g) is built by an initial placement, rebalanced by Alg. 2's loop executed by one wavefront
// (argmax / argmin are wave reductions), then cut into tiles of at most tile_m rows, bin after
// bin, heaviest block first.  The paper's scheduler runs as host-driven tensor ops and costs
// 20-30 % of its layer time (section 5.3.1); here it is a few microseconds on the device.
#include "common.h"
#include <climits>

namespace {

constexpr int NTH = 256;   // >= MOE_MAX_EXPERTS: one thread per expert

__device__ __forceinline__ int weight_of(int n, int q, bool by_cost) {
    return by_cost ? (n > 0 ? (n > q ? n : q) : 0) : n;
}
// larger value wins, equal values go to the lower index
__device__ __forceinline__ void wave_argbest(int& v, int& i) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        int ov = __shfl_xor(v, off), oi = __shfl_xor(i, off);
        if (ov > v || (ov == v && oi < i)) { v = ov; i = oi; }
    }
}

__global__ __launch_bounds__(NTH) void plan_kernel(const int32_t* __restrict__ counts,
                                                   const int32_t* __restrict__ offsets, int E, int A, int tile_m,
                                                   int G, int q, int policy, moe_tile* __restrict__ tiles,
                                                   int capacity, int32_t* __restrict__ hdr,
                                                   int32_t* __restrict__ sched) {
    __shared__ int cnt[MOE_MAX_EXPERTS], cost[MOE_MAX_EXPERTS], order[MOE_MAX_EXPERTS];
    __shared__ int S_[MOE_MAX_EXPERTS * MOE_MAX_BINS];
    __shared__ unsigned short NT_[MOE_MAX_EXPERTS * MOE_MAX_BINS];
    __shared__ int load[MOE_MAX_BINS];
    __shared__ int s_tavg, s_moves;
    volatile int* S = S_;
    const int tid = threadIdx.x, lane = tid & 63;
    const bool by_cost = (policy == MOE_PLAN_BALANCED);
    (void)A;

    for (int i = tid; i < E * G; i += NTH) S_[i] = 0;
    if (tid < E) {
        int c = counts[tid];
        cnt[tid] = c;
        cost[tid] = weight_of(c, q, by_cost);
    }
    if (tid == 0) s_moves = 0;
    __syncthreads();

    // ---- initial placement (the paper's initialAssign)
    if (policy == MOE_PLAN_BALANCED) {
        if (tid < E) {   // experts by falling weight, equal weights by rising id
            int c = cost[tid], r = 0;
            for (int e2 = 0; e2 < E; ++e2) {
                int c2 = cost[e2];
                r += (c2 > c || (c2 == c && e2 < tid)) ? 1 : 0;
            }
            order[r] = tid;
        }
        __syncthreads();
        if (tid < 64) {  // each expert whole, on the least loaded bin so far
            int tg = 0;
            for (int r = 0; r < E; ++r) {
                int e = order[r], c = cost[e];
                if (c == 0) break;
                int v = lane < G ? -tg : INT_MIN, g = lane;
                wave_argbest(v, g);
                if (lane == 0) S[e * G + g] = cnt[e];
                if (lane == g) tg += c;
            }
        }
    } else if (policy == MOE_PLAN_EVEN_SPLIT) {
        if (tid < E) {
            int c = cnt[tid];
            for (int g = 0; g < G; ++g) S[tid * G + g] = c / G + (g < c % G ? 1 : 0);
        }
    } else {             // contiguous blocks of experts per bin
        if (tid < E) S[tid * G + (int)(((long long)tid * G) / E)] = cnt[tid];
    }
    __syncthreads();
    if (tid < G) {
        int s = 0;
        for (int e = 0; e < E; ++e) s += weight_of(S[e * G + tid], q, by_cost);
        load[tid] = s;
    }
    __syncthreads();
    if (tid == 0) {
        long long tot = 0;
        for (int g = 0; g < G; ++g) tot += load[g];
        s_tavg = (int)(tot / G);
    }
    __syncthreads();

    // ---- Alg. 2: move rows of the largest block of the most loaded bin to the least loaded bin
    if ((policy == MOE_PLAN_BALANCED || policy == MOE_PLAN_HARMOENY) && tid < 64) {
        const int t_avg = s_tavg;
        const int gran = by_cost ? tile_m : 1;
        int tg = lane < G ? load[lane] : 0;
        int moves = 0;
        const int max_iters = E * G + 16;
        for (int it = 0; it < max_iters; ++it) {
            if (__ballot(lane < G && tg > t_avg) == 0ull) break;
            int v = lane < G ? tg : INT_MIN, g_max = lane;
            wave_argbest(v, g_max);
            int t_move = -1, e_max = INT_MAX;
            for (int e = lane; e < E; e += 64) {
                int s = S[e * G + g_max];
                if (s > t_move) { t_move = s; e_max = e; }
            }
            wave_argbest(t_move, e_max);
            if (t_move < q) break;
            int nv = lane < G ? -tg : INT_MIN, g_min = lane;
            wave_argbest(nv, g_min);
            const int t_min = -nv;
            if (g_min == g_max || t_min + q > t_avg) break;
            int t_s = t_move < t_avg - t_min ? t_move : t_avg - t_min;
            if (by_cost && t_s < t_move) {
                // a split leaves at least q rows behind and moves whole tiles
                if (t_move - t_s < q) t_s = t_move - q;
                t_s = t_s / gran * gran;
                if (t_s < q || t_s <= 0) break;
            }
            const int n_from = S[e_max * G + g_max], n_to = S[e_max * G + g_min];
            const int d_from = weight_of(n_from, q, by_cost) - weight_of(n_from - t_s, q, by_cost);
            const int d_to = weight_of(n_to + t_s, q, by_cost) - weight_of(n_to, q, by_cost);
            if (lane == 0) {
                S[e_max * G + g_max] = n_from - t_s;
                S[e_max * G + g_min] = n_to + t_s;
            }
            if (lane == g_max) tg -= d_from;
            if (lane == g_min) tg += d_to;
            ++moves;
        }
        if (lane < G) load[lane] = tg;
        if (lane == 0) s_moves = moves;
    }
    __syncthreads();

    // ---- tiles, bin after bin; inside a bin blocks by falling row count, then expert id
    const int e = tid;
    if (e < E)
        for (int g = 0; g < G; ++g) NT_[e * G + g] = (unsigned short)((S[e * G + g] + tile_m - 1) / tile_m > 65535 ? 65535 : (S[e * G + g] + tile_m - 1) / tile_m);
    __syncthreads();
    if (e < E) {
        int row = offsets[e], bin_start = 0;
        for (int g = 0; g < G; ++g) {
            const int n = S[e * G + g];
            int before = 0, total = 0;
            for (int e2 = 0; e2 < E; ++e2) {
                int n2 = S[e2 * G + g], t2 = NT_[e2 * G + g];
                total += t2;
                before += (n2 > n || (n2 == n && e2 < e)) ? t2 : 0;
            }
            if (e == 0) hdr[4 + g] = bin_start;
            const int nt = (n + tile_m - 1) / tile_m;
            for (int i = 0; i < nt; ++i) {
                int at = bin_start + before + i;
                if (at < capacity) {
                    moe_tile t;
                    t.expert = e;
                    t.row_begin = row + i * tile_m;
                    t.row_count = (n - i * tile_m) < tile_m ? (n - i * tile_m) : tile_m;
                    t.bin = g;
                    tiles[at] = t;
                }
            }
            if (sched) sched[e * G + g] = n;
            row += n;
            bin_start += total;
        }
        if (e == 0) {
            hdr[4 + G] = bin_start < capacity ? bin_start : capacity;
            hdr[0] = bin_start < capacity ? bin_start : capacity;
            hdr[1] = G;
            hdr[2] = s_moves;
            hdr[3] = s_tavg;
        }
    }
    if (tid < G) hdr[4 + MOE_MAX_BINS + 1 + tid] = load[tid];
}

}  // namespace

extern "C" int moe_plan_capacity(int A, int E, int tile_m, int n_bins) {
    if (A < 0 || E < 1 || tile_m < 1 || n_bins < 1) return 0;
    long long c = ((long long)A + tile_m - 1) / tile_m + (long long)E * n_bins;
    return c > INT_MAX ? INT_MAX : (int)c;
}

extern "C" int moe_plan_tiles(const int32_t* counts, const int32_t* offsets, int E, int A, int tile_m, int n_bins,
                              int q_tokens, int policy, moe_tile* tiles, int tile_capacity, int32_t* plan_hdr,
                              int32_t* sched, void* stream) {
    MOE_REQUIRE(E >= 1 && A >= 0, MOE_ERR_ARG, "moe_plan_tiles: E=%d A=%d", E, A);
    MOE_REQUIRE(E <= MOE_MAX_EXPERTS, MOE_ERR_UNSUPPORTED, "moe_plan_tiles: E=%d > %d", E, MOE_MAX_EXPERTS);
    MOE_REQUIRE(n_bins >= 1 && n_bins <= MOE_MAX_BINS, MOE_ERR_ARG, "moe_plan_tiles: n_bins=%d outside [1,%d]", n_bins, MOE_MAX_BINS);
    MOE_REQUIRE(tile_m >= 1 && q_tokens >= 1, MOE_ERR_ARG, "moe_plan_tiles: tile_m=%d q_tokens=%d must be >= 1", tile_m, q_tokens);
    MOE_REQUIRE(policy >= MOE_PLAN_BALANCED && policy <= MOE_PLAN_EVEN_SPLIT, MOE_ERR_ARG, "moe_plan_tiles: policy %d", policy);
    MOE_REQUIRE(counts && offsets && tiles && plan_hdr, MOE_ERR_ARG, "moe_plan_tiles: null pointer");
    MOE_REQUIRE(tile_capacity >= moe_plan_capacity(A, E, tile_m, n_bins), MOE_ERR_CAPACITY,
                "moe_plan_tiles: tile_capacity %d < %d", tile_capacity, moe_plan_capacity(A, E, tile_m, n_bins));
    hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(NTH), 0, (hipStream_t)stream, counts, offsets, E, A, tile_m, n_bins,
                       q_tokens, policy, tiles, tile_capacity, plan_hdr, sched);
    MOE_CHECK_LAUNCH("moe_plan_tiles");
    return MOE_OK;
}
