// moe_permute: stable counting sort of the A = T*k assignments by expert, and the row gather
// (one-GPU form of Alg. 1 step 4; counts[] is the one-GPU slice of S_initial, step 3).
//
// Four launches, no float atomics, no ordering left to chance:
//   1. per-block histogram of expert ids (1024 assignments per work-group, LDS integer adds)
//   2. one work-group: per-expert exclusive prefix over the blocks -> counts, offsets
//   3. per-block stable rank: inside a wavefront the peers of an assignment (same expert) are
//      found with one ballot per bit of the expert id; popcount of the lower lanes is the rank;
//      per-64-chunk counts are prefix-summed in LDS -> perm, inv_perm
//   4. row gather x_perm[r] = x[perm[r] / k], 16 bytes per lane, fully coalesced
#include "common.h"
#include "permute_rank.h"
#include <mutex>

namespace {

using moe_rank::CHUNKS;
using moe_rank::NTH;
using moe_rank::PB;   // assignments per work-group in steps 1 and 3

__global__ __launch_bounds__(NTH) void hist_kernel(const int32_t* __restrict__ idx, int A, int E,
                                                   int32_t* __restrict__ block_hist) {
    __shared__ int h[MOE_MAX_EXPERTS];
    for (int e = threadIdx.x; e < E; e += NTH) h[e] = 0;
    __syncthreads();
    const int base = blockIdx.x * PB;
    int mine[PB / NTH];                                     // (all loads first: one memory latency, not PB / NTH)
#pragma unroll
    for (int j = 0; j < PB / NTH; ++j) {
        const int a = base + j * NTH + threadIdx.x;
        mine[j] = a < A ? idx[a] : -1;
    }
#pragma unroll
    for (int j = 0; j < PB / NTH; ++j)
        if ((unsigned)mine[j] < (unsigned)E) atomicAdd(&h[mine[j]], 1);
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += NTH) block_hist[(size_t)blockIdx.x * E + e] = h[e];
}

// One work-group.  block_hist[b][e] becomes the number of assignments of expert e in blocks < b.
__global__ __launch_bounds__(NTH) void scan_kernel(int32_t* __restrict__ block_hist, int nb, int E,
                                                   int32_t* __restrict__ counts, int32_t* __restrict__ offsets) {
    __shared__ int tot[MOE_MAX_EXPERTS];
    for (int e = threadIdx.x; e < E; e += NTH) {
        int run = 0;
        for (int b0 = 0; b0 < nb; b0 += 8) {               // eight loads in flight at a time
            int v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = b0 + j < nb ? block_hist[(size_t)(b0 + j) * E + e] : 0;
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (b0 + j < nb) {
                    block_hist[(size_t)(b0 + j) * E + e] = run;
                    run += v[j];
                }
        }
        tot[e] = run;
        counts[e] = run;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int run = 0;
        for (int e = 0; e < E; ++e) { offsets[e] = run; run += tot[e]; }
        offsets[E] = run;
    }
}

template <int MODE>
__global__ __launch_bounds__(NTH) void rank_kernel(const int32_t* __restrict__ idx, int A, int E, int nbits, int nb,
                                                   const int32_t* __restrict__ block_hist,
                                                   int32_t* __restrict__ counts, int32_t* __restrict__ offsets,
                                                   int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm) {
    moe_rank::rank_body<MODE>(idx, A, E, nbits, nb, block_hist, counts, offsets, perm, inv_perm);
}

// x_perm row r <- x row perm[r] / k, in 16-byte pieces (vpr pieces per row)
__global__ __launch_bounds__(NTH) void gather_rows_kernel(const uint4* __restrict__ x, const int32_t* __restrict__ perm,
                                                          int A, int k, int vpr, uint4* __restrict__ x_perm) {
    const size_t total = (size_t)A * vpr;
    for (size_t i = (size_t)blockIdx.x * NTH + threadIdx.x; i < total; i += (size_t)gridDim.x * NTH) {
        int r = (int)(i / vpr), v = (int)(i - (size_t)r * vpr);
        int t = perm[r] / k;
        x_perm[i] = x[(size_t)t * vpr + v];
    }
}

}  // namespace

// Scratch of moe_permute_static: the block histograms, in the library's own device memory (each
// GPU the library runs on holds a copy of this array until the process ends).  Host code never
// passes the array's name to a kernel: it asks the runtime for the array's address on the
// current device, once per device, and uses that pointer.
static __device__ __align__(256) unsigned char scratch[MOE_PERMUTE_STATIC_BYTES];

static int32_t* g_scratch_ptr[64] = {};          // per device, set on first use
static std::mutex g_scratch_mutex;

static int scratch_on_current_device(int32_t** out) {
    int dev = -1;
    MOE_CHECK_HIP(hipGetDevice(&dev));
    MOE_REQUIRE(dev >= 0 && dev < 64, MOE_ERR_UNSUPPORTED, "moe_permute_static: device %d", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        MOE_CHECK_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        MOE_REQUIRE(p != nullptr, MOE_ERR_HIP, "moe_permute_static: no address for the scratch array");
        g_scratch_ptr[dev] = (int32_t*)p;
    }
    *out = g_scratch_ptr[dev];
    return MOE_OK;
}

// Argument checks shared by the two entry points (nothing is enqueued on an error).
static int permute_check(const char* who, const void* x, const int32_t* expert_idx, int T, int d, int E, int k,
                         moe_dtype dt, const int32_t* counts, const int32_t* offsets, const int32_t* perm,
                         const int32_t* inv_perm, const void* x_perm) {
    MOE_REQUIRE(moe_dtype_ok(dt), MOE_ERR_UNSUPPORTED, "%s: dtype %d", who, (int)dt);
    MOE_REQUIRE(T >= 0 && E >= 1 && k >= 1 && d >= 1, MOE_ERR_ARG, "%s: T=%d d=%d E=%d k=%d", who, T, d, E, k);
    MOE_REQUIRE(E <= MOE_MAX_EXPERTS, MOE_ERR_UNSUPPORTED, "%s: E=%d > %d", who, E, MOE_MAX_EXPERTS);
    MOE_REQUIRE((long long)T * k < (1ll << 30), MOE_ERR_UNSUPPORTED, "%s: T*k too large", who);
    MOE_REQUIRE((x == nullptr) == (x_perm == nullptr), MOE_ERR_ARG, "%s: x and x_perm must both be given or both be null", who);
    MOE_REQUIRE(((size_t)d * moe_elem_size(dt)) % 16 == 0, MOE_ERR_UNSUPPORTED, "%s: row of %d elements is not a multiple of 16 bytes", who, d);
    MOE_REQUIRE(counts && offsets, MOE_ERR_ARG, "%s: null pointer", who);
    MOE_REQUIRE((long long)T * k == 0 || (expert_idx && perm && inv_perm), MOE_ERR_ARG, "%s: null pointer", who);
    return MOE_OK;
}

// The launches of the sort; block_hist holds one histogram of E counters per block of PB
// assignments (every entry is written by hist_kernel before anything reads it).
static int permute_launch(const void* x, const int32_t* expert_idx, int T, int d, int E, int k, moe_dtype dt,
                          int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv_perm, void* x_perm,
                          int32_t* block_hist, hipStream_t st) {
    const int A = T * k;
    const int nb = A == 0 ? 1 : (A + PB - 1) / PB;
    int nbits = 0;
    while ((1 << nbits) < E) ++nbits;

    hipLaunchKernelGGL(hist_kernel, dim3(nb), dim3(NTH), 0, st, expert_idx, A, E, block_hist);
    MOE_CHECK_LAUNCH("moe_permute/hist");
    // With few blocks every rank work-group repeats the scan itself (one launch less); with many
    // blocks, or nothing to rank, the scan is a launch of its own.
    const bool fused_scan = A > 0 && nb <= 64;
    if (!fused_scan) {
        hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(NTH), 0, st, block_hist, nb, E, counts, offsets);
        MOE_CHECK_LAUNCH("moe_permute/scan");
    }
    if (A == 0) return MOE_OK;
    if (fused_scan)
        hipLaunchKernelGGL(rank_kernel<1>, dim3(nb), dim3(NTH), sizeof(int) * CHUNKS * E, st, expert_idx, A, E, nbits, nb,
                           block_hist, counts, offsets, perm, inv_perm);
    else
        hipLaunchKernelGGL(rank_kernel<0>, dim3(nb), dim3(NTH), sizeof(int) * CHUNKS * E, st, expert_idx, A, E, nbits, nb,
                           block_hist, counts, offsets, perm, inv_perm);
    MOE_CHECK_LAUNCH("moe_permute/rank");
    if (x) {
        const int vpr = (int)((size_t)d * moe_elem_size(dt) / 16);
        size_t total = (size_t)A * vpr;
        size_t blocks = (total + NTH - 1) / NTH;
        if (blocks > 65536) blocks = 65536;
        hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)blocks), dim3(NTH), 0, st, (const uint4*)x, perm, A, k,
                           vpr, (uint4*)x_perm);
        MOE_CHECK_LAUNCH("moe_permute/gather");
    }
    return MOE_OK;
}

extern "C" int moe_permute(const void* x, const int32_t* expert_idx, int T, int d, int E, int k, moe_dtype dt,
                           int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv_perm, void* x_perm,
                           void* ws, size_t ws_bytes, void* stream) {
    const int rc = permute_check("moe_permute", x, expert_idx, T, d, E, k, dt, counts, offsets, perm, inv_perm, x_perm);
    if (rc != MOE_OK) return rc;
    MOE_REQUIRE(ws, MOE_ERR_ARG, "moe_permute: null pointer");
    MOE_REQUIRE(ws_bytes >= moe_workspace_bytes(MOE_OP_PERMUTE, T, d, 0, E, k, dt), MOE_ERR_WORKSPACE,
                "moe_permute: workspace %zu < %zu bytes", ws_bytes, moe_workspace_bytes(MOE_OP_PERMUTE, T, d, 0, E, k, dt));
    return permute_launch(x, expert_idx, T, d, E, k, dt, counts, offsets, perm, inv_perm, x_perm, (int32_t*)ws,
                          (hipStream_t)stream);
}

extern "C" int moe_permute_static(const void* x, const int32_t* expert_idx, int T, int d, int E, int k, moe_dtype dt,
                                  int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv_perm, void* x_perm,
                                  void* stream) {
    const int rc = permute_check("moe_permute_static", x, expert_idx, T, d, E, k, dt, counts, offsets, perm, inv_perm, x_perm);
    if (rc != MOE_OK) return rc;
    const size_t need = moe_workspace_bytes(MOE_OP_PERMUTE, T, d, 0, E, k, dt);
    MOE_REQUIRE(need <= MOE_PERMUTE_STATIC_BYTES, MOE_ERR_CAPACITY,
                "moe_permute_static: T*k = %lld with E = %d needs %zu bytes of scratch, the built-in array holds %u "
                "(use moe_permute with a workspace)", (long long)T * k, E, need, MOE_PERMUTE_STATIC_BYTES);
    int32_t* block_hist = nullptr;
    const int rs = scratch_on_current_device(&block_hist);
    if (rs != MOE_OK) return rs;
    return permute_launch(x, expert_idx, T, d, E, k, dt, counts, offsets, perm, inv_perm, x_perm, block_hist,
                          (hipStream_t)stream);
}
