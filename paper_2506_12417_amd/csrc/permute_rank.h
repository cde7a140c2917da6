// The stable in-block rank of moe_permute (step 3 of the counting sort) as a device function, shared
// by moe_permute's own launch (permute.hip) and by the launch that runs it side by side with the
// plan (plan.hip: moe_permute_plan).
#pragma once
#include "common.h"

namespace moe_rank {

constexpr int PB = 1024;   // assignments per work-group
constexpr int NTH = 256;
constexpr int CHUNKS = PB / 64;

// MODE 0: offsets[] holds the experts' first positions and block_hist[b][e] the number of
//         assignments of expert e in the blocks before b (a scan launch has run).
// MODE 1: block_hist holds the raw per-block histograms and this work-group does the scan itself
//         (it sums the histograms of the blocks before it and of all blocks, and scans the
//         totals; the first one also writes counts and offsets): one launch less.
// MODE 2: no histogram launch either: the work-group counts the experts of all assignments
//         before its block, and of all assignments, itself (for few blocks: every work-group
//         reads all A ids).
// Adds, for every assignment i < A, one to all_[idx[i]] and -- if i < upto -- to before[idx[i]] (LDS
// counters; before may be null).  Every thread fetches its ids four at a time and sixteen
// fetches at once: the ids are few (A <= 32768), what counts is that the work-group pays one
// memory latency, not one per fetch.
__device__ __forceinline__ void count_experts(const int32_t* __restrict__ idx, int A, int E, int upto, int* before, int* all_) {
    constexpr int NV = 16;
    for (int i0 = 0; i0 < A; i0 += NV * NTH * 4) {
        int4 v[NV];
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int i = i0 + (j * NTH + (int)threadIdx.x) * 4;
            if (i + 3 < A) {
                v[j] = *reinterpret_cast<const int4*>(idx + i);
            } else {
                v[j].x = i < A ? idx[i] : -1;
                v[j].y = i + 1 < A ? idx[i + 1] : -1;
                v[j].z = i + 2 < A ? idx[i + 2] : -1;
                v[j].w = -1;
            }
        }
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int i = i0 + (j * NTH + (int)threadIdx.x) * 4;
            const int e4[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if ((unsigned)e4[c] < (unsigned)E) {
                    atomicAdd(&all_[e4[c]], 1);
                    if (before && i + c < upto) atomicAdd(&before[e4[c]], 1);
                }
        }
    }
}

template <int MODE>
__device__ __forceinline__ void rank_body(const int32_t* __restrict__ idx, int A, int E, int nbits, int nb,
                                          const int32_t* __restrict__ block_hist,
                                          int32_t* __restrict__ counts, int32_t* __restrict__ offsets,
                                          int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm) {
    extern __shared__ int chunk_hist[];   // [CHUNKS][E]
    __shared__ int start_of[MOE_MAX_EXPERTS];      // first position of this work-group's assignments of expert e
    __shared__ int scan_buf[2][MOE_MAX_EXPERTS];
    for (int i = threadIdx.x; i < CHUNKS * E; i += NTH) chunk_hist[i] = 0;
    // this thread's assignments: fetched first, all at once, so that their latency passes under the scan
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int base = blockIdx.x * PB;
    int my_e[CHUNKS / 4], my_rank[CHUNKS / 4];
#pragma unroll
    for (int ci = 0; ci < CHUNKS / 4; ++ci) {
        const int a = base + (ci * 4 + wave) * 64 + lane;
        my_e[ci] = a < A ? idx[a] : -1;
    }
    if (MODE >= 1) {
        static_assert(NTH >= MOE_MAX_EXPERTS, "one thread per expert");
        const int e = threadIdx.x;
        int before = 0, total = 0;
        if (MODE == 2) {
            // counters in LDS (scan_buf is free until the scan below): [0] before this block, [1] all
            scan_buf[0][e] = 0;
            scan_buf[1][e] = 0;
            __syncthreads();
            count_experts(idx, A, E, base, scan_buf[0], scan_buf[1]);
            __syncthreads();
            before = scan_buf[0][e];
            total = scan_buf[1][e];
            __syncthreads();
        } else if (e < E)
            for (int b0 = 0; b0 < nb; b0 += 8) {           // eight loads in flight at a time
                int v[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) v[j] = b0 + j < nb ? block_hist[(size_t)(b0 + j) * E + e] : 0;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    before += b0 + j < (int)blockIdx.x ? v[j] : 0;
                    total += v[j];
                }
            }
        // inclusive scan of the totals over the experts (Hillis-Steele, MOE_MAX_EXPERTS entries)
        scan_buf[0][e] = e < E ? total : 0;
        __syncthreads();
        int cur = 0;
        for (int step = 1; step < MOE_MAX_EXPERTS; step <<= 1) {
            const int v = scan_buf[cur][e] + (e >= step ? scan_buf[cur][e - step] : 0);
            scan_buf[cur ^ 1][e] = v;
            cur ^= 1;
            __syncthreads();
        }
        const int incl = scan_buf[cur][e];
        if (e < E) {
            start_of[e] = incl - total + before;
            if (blockIdx.x == 0) {
                counts[e] = total;
                offsets[e] = incl - total;
                if (e == E - 1) offsets[E] = incl;
            }
        }
    } else {
        for (int e = threadIdx.x; e < E; e += NTH) start_of[e] = offsets[e] + block_hist[(size_t)blockIdx.x * E + e];
    }
    __syncthreads();
#pragma unroll
    for (int ci = 0; ci < CHUNKS / 4; ++ci) {
        const int c = ci * 4 + wave;
        int e = my_e[ci];
        if ((unsigned)e >= (unsigned)E) e = -1;
        unsigned long long peers = __ballot(e >= 0);
        for (int b = 0; b < nbits; ++b) {
            unsigned long long m = __ballot((e >> b) & 1);
            peers &= ((e >> b) & 1) ? m : ~m;
        }
        const unsigned long long below = peers & ((1ull << lane) - 1ull);
        my_e[ci] = e;
        my_rank[ci] = __popcll(below);
        if (e >= 0 && below == 0) chunk_hist[c * E + e] = __popcll(peers);   // lowest peer lane
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += NTH) {
        int run = start_of[e];
        for (int c = 0; c < CHUNKS; ++c) {
            int v = chunk_hist[c * E + e];
            chunk_hist[c * E + e] = run;
            run += v;
        }
    }
    __syncthreads();
#pragma unroll
    for (int ci = 0; ci < CHUNKS / 4; ++ci) {
        const int c = ci * 4 + wave;
        const int a = base + c * 64 + lane;
        if (my_e[ci] >= 0) {
            int pos = chunk_hist[c * E + my_e[ci]] + my_rank[ci];
            perm[pos] = a;
            inv_perm[a] = pos;
        }
    }
}

}  // namespace moe_rank
