/*
 * libmoe -- one Mixture-of-Experts layer forward on one AMD MI355X (gfx950), as a C ABI.
 *
 * The layer is the one of HarMoEny (arXiv 2506.12417), Alg. 1, on a single GPU:
 *
 *   moe_route_topk         step 1  token routing (top-k gating, section 2)
 *   moe_permute            step 4  tokens grouped by their expert (one-GPU form of the scatter)
 *   moe_plan_tiles         step 3  load-aware schedule: Alg. 2 run over the GPU's XCDs
 *   moe_grouped_ffn        step 5  expert FFNs (section 2 / section 4.4: x W1 W2)
 *   moe_unpermute_combine  step 6  original order restored, expert outputs weighted and summed
 *   moe_prefetch_experts   step 5  asynchronous expert fetching by overwrite (section 4.3)
 *
 * Conventions
 *   - Every pointer is DEVICE memory unless its comment says host.  The caller owns every
 *     buffer; the library allocates nothing on the device (the prefetch engine owns a stream
 *     and events only).
 *   - Every call only ENQUEUES work on `stream` (a hipStream_t passed as void*; NULL = the
 *     default stream).  No call synchronises with the host or reads device data on the host.
 *   - Every function returns a moe_status.  Arguments are checked before anything is
 *     enqueued; on an error nothing has been launched and no buffer has been touched.
 *     moe_last_error() gives the text of the calling thread's last error.
 *   - Matrices are row-major and contiguous.  T tokens, d = d_model, F = d_ff, E experts,
 *     k experts per token, A = T*k assignments, assignment id a = t*k + j.
 *   - dtype is the type of activations and weights (MOE_F32 or MOE_BF16); accumulation is
 *     always fp32 or wider, gate weights and layer outputs are fp32.
 */
#ifndef MOE_H
#define MOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* exported from libmoe.so (the library is built with hidden visibility by default) */
#define MOE_API __attribute__((visibility("default")))

typedef enum {
    MOE_OK = 0,
    MOE_ERR_ARG = -1,          /* null pointer, size or range */
    MOE_ERR_UNSUPPORTED = -2,  /* dtype, activation, alignment or a size beyond a stated limit */
    MOE_ERR_WORKSPACE = -3,    /* workspace smaller than moe_workspace_bytes() */
    MOE_ERR_CAPACITY = -4,     /* tile table or expert slots too small */
    MOE_ERR_HIP = -5           /* the HIP runtime reported an error */
} moe_status;

typedef enum { MOE_F32 = 0, MOE_BF16 = 1 } moe_dtype;
typedef enum { MOE_RELU = 0, MOE_SWIGLU = 1 } moe_act;

/* Limits (MOE_ERR_UNSUPPORTED beyond them). */
#define MOE_MAX_EXPERTS 256
#define MOE_MAX_TOPK 8
#define MOE_MAX_BINS 16

/* ------------------------------------------------------------------------------------------
 * Step 1, token routing (Alg. 1 line "m_expert <- router(x)"; section 2: the router gives each
 * expert a value in (0,1), the token goes to the k highest, outputs are weighted by them).
 *
 *   logits[t,e] = bias[e] + sum_i x[t,i] * w_gate[i,e]
 *   value       = softmax over all E logits
 *   expert_idx[t,0..k) = the k experts with the largest logits, in descending order; equal
 *                 logits go to the lower expert index
 *   gate_w[t,j] = value of expert_idx[t,j]; renorm != 0 divides the k values by their sum
 *
 * The top-k decision is taken as if the logits were computed in float64: the kernel works in
 * fp32 with a rigorous error bound and recomputes in fp64 every token whose decision gaps are
 * inside that bound.
 *
 *   x       [T,d]  dtype dt        w_gate [d,E] dtype dt       bias [E] fp32, may be NULL
 *   expert_idx [T,k] int32 out     gate_w [T,k] fp32 out
 *   logits_out [T,E] fp32 out, may be NULL (diagnostic)
 * Requires 1 <= k <= min(E, MOE_MAX_TOPK), E <= MOE_MAX_EXPERTS, d % 8 == 0.  T = 0 is a no-op.
 */
MOE_API int moe_route_topk(const void* x, const void* w_gate, const float* bias,
                   int T, int d, int E, int k, int renorm, moe_dtype dt,
                   int32_t* expert_idx, float* gate_w, float* logits_out, void* stream);

/* The same routing step with a router prepared once, outside the hot path (W_g is a parameter
 * of the layer): moe_pack_router rewrites w_gate [d,E] as w_gate_t [E,d] (contraction index
 * contiguous, same dtype) and gives w_norm2[e] = sum_i w_gate[i,e]^2 (fp32, rounded up), which
 * the kernel's error bound uses.  moe_route_topk_packed computes exactly what moe_route_topk
 * computes (same selection rule, same exact-arithmetic guarantee); it reads x once at HBM speed.
 * bf16 only, d % 64 == 0 (MOE_ERR_UNSUPPORTED otherwise: use moe_route_topk).
 *
 *   w_gate_t [E,d] dt out      w_norm2 [E] fp32 out
 */
MOE_API int moe_pack_router(const void* w_gate, int d, int E, moe_dtype dt, void* w_gate_t, float* w_norm2,
                            void* stream);
MOE_API int moe_route_topk_packed(const void* x, const void* w_gate_t, const float* w_norm2, const float* bias,
                                  int T, int d, int E, int k, int renorm, moe_dtype dt,
                                  int32_t* expert_idx, float* gate_w, float* logits_out, void* stream);

/* ------------------------------------------------------------------------------------------
 * Step 4 on one GPU (Alg. 1 "scatter tokens"; counts[] is the one-GPU slice of the initial
 * schedule S_initial of step 3): a stable counting sort of the A assignments by expert.
 *
 *   counts[e]  = number of assignments with expert e        offsets = exclusive scan, [E+1]
 *   pos(a)     = offsets[idx[a]] + #{a' < a : idx[a'] = idx[a]}
 *   perm[pos(a)] = a      inv_perm[a] = pos(a)      x_perm[pos(a),:] = x[a div k,:] (bit copy)
 *
 *   x [T,d] dt (may be NULL together with x_perm: indices only)
 *   expert_idx [T,k] int32, every entry in [0,E) (entries outside are not detected)
 *   ws / ws_bytes: scratch of at least moe_workspace_bytes(MOE_OP_PERMUTE, ...)
 */
MOE_API int moe_permute(const void* x, const int32_t* expert_idx, int T, int d, int E, int k, moe_dtype dt,
                int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv_perm, void* x_perm,
                void* ws, size_t ws_bytes, void* stream);

/* moe_permute for callers that cannot allocate device memory and have no workspace to pass:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * kernels, same results; the block histograms go to an array of MOE_PERMUTE_STATIC_BYTES
 * bytes (1 MiB) that is part of the library's device image, so nothing is allocated, neither
 * here nor by the caller.  MOE_ERR_CAPACITY if moe_workspace_bytes(MOE_OP_PERMUTE, ...) exceeds
 * that size (ceil(T*k / 1024) * E * 4 bytes: T*k up to 2 Mi assignments at E = 128); nothing is
 * enqueued then.  The stream must belong to the current device.  Every call on a GPU uses that
 * GPU's one array: calls that may run at the same time on one GPU (two streams) race; calls
 * on one stream are safe, nothing has to be cleared between them. */
#define MOE_PERMUTE_STATIC_BYTES (1u << 20)
MOE_API int moe_permute_static(const void* x, const int32_t* expert_idx, int T, int d, int E, int k, moe_dtype dt,
                int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv_perm, void* x_perm,
                void* stream);

/* ------------------------------------------------------------------------------------------
 * Step 3 on one GPU: the load-aware token schedule (section 4.2, Alg. 2) with the GPU's
 * n_bins XCDs in the role of the paper's GPUs.  S[e,g] = rows of expert e processed by bin g.
 *
 * policy
 *   MOE_PLAN_BALANCED  Alg. 2 in units of tiles: a block of n rows of one expert on one bin
 *                      weighs ceil(n / tile_m), because the kernels work tile by tile and a tile
 *                      costs about the same whether it holds many rows (arithmetic) or few (the
 *                      fetch of the expert's weights; section 4.4, Eq. 1).  Experts are first
 *                      placed whole, heaviest first, each on the least loaded bin; then, until
 *                      the most and the least loaded bin differ by at most one tile, half their
 *                      difference moves from the one to the other, taken in whole tiles from
 *                      the largest block (or the whole block).  q_tokens is not used.
 *   MOE_PLAN_HARMOENY  Alg. 2 as printed: expert e starts on bin e*n_bins/E (contiguous
 *                      blocks of experts), loads are row counts, any number of rows may move,
 *                      a move needs at least q_tokens rows.
 *   MOE_PLAN_STATIC    the starting placement of MOE_PLAN_HARMOENY, no rebalancing.
 *   MOE_PLAN_EVEN_SPLIT every expert's rows are divided evenly over all bins (section 5.3.2,
 *                      policy 3); the remainder goes one row each to the lowest bins.
 *   MOE_PLAN_ROUND_ROBIN experts dealt to the bins in turn (expert e on bin e mod n_bins), every
 *                      row goes to its expert's bin, no rebalancing (section 5.3.2, policy 1).
 *
 * Output: a table of tiles, bin after bin.  A tile is at most tile_m consecutive rows of one
 * expert; the tiles cover rows [0,A) exactly once.  A block = the rows of one expert on one
 * bin; its tiles are listed together, by rising row_begin.  The order of a bin's blocks is the
 * order in which moe_grouped_ffn takes them (the paper leaves the order inside a GPU open):
 * blocks of more than one tile and blocks of one tile are each ordered by falling row count,
 * then expert id; if the first kind outnumbers the second (or one is missing) it comes first,
 * otherwise the two lists are merged evenly (the i-th of L has the key (2i+1)/L, rising keys,
 * the multi-tile block first among equals), so that work bound by arithmetic (tiles that share
 * an expert's weights) and work bound by memory (one-tile experts, each streaming its own
 * weights) run side by side.
 *
 *   counts [E], offsets [E+1] int32 (device, e.g. from moe_permute)
 *   tiles  [tile_capacity] out;  tile_capacity >= moe_plan_capacity(A, E, tile_m, n_bins)
 *   plan_hdr [MOE_PLAN_HDR_INTS] int32 out:
 *       [0] n_tiles  [1] n_bins  [2] number of Alg. 2 moves made  [3] t_avg
 *       [4 .. 4+n_bins]  bin_start (n_bins+1 entries; bin g owns tiles [bin_start[g], bin_start[g+1]))
 *       [4+MOE_MAX_BINS+1 .. +n_bins)  load of each bin after rebalancing (in the policy's unit)
 *       [MOE_PLAN_HDR_CTR .. +MOE_MAX_BINS]  work counters of moe_grouped_ffn, left at zero
 *   sched  [E*n_bins] int32 out, may be NULL: the schedule S, row-major [E, n_bins]
 * Requires 1 <= E <= MOE_MAX_EXPERTS, 1 <= n_bins <= MOE_MAX_BINS, tile_m >= 1, q_tokens >= 1,
 * A + E*q_tokens < 2^26.
 */
typedef struct { int32_t expert, row_begin, row_count, bin; } moe_tile;

enum { MOE_PLAN_BALANCED = 0, MOE_PLAN_HARMOENY = 1, MOE_PLAN_STATIC = 2, MOE_PLAN_EVEN_SPLIT = 3,
       MOE_PLAN_ROUND_ROBIN = 4 };
#define MOE_PLAN_HDR_CTR (4 + 2 * (MOE_MAX_BINS + 1))
#define MOE_PLAN_HDR_INTS (MOE_PLAN_HDR_CTR + MOE_MAX_BINS + 1)

MOE_API int moe_plan_capacity(int A, int E, int tile_m, int n_bins);

MOE_API int moe_plan_tiles(const int32_t* counts, const int32_t* offsets, int E, int A,
                   int tile_m, int n_bins, int q_tokens, int policy,
                   moe_tile* tiles, int tile_capacity, int32_t* plan_hdr, int32_t* sched,
                   void* stream);

/* moe_permute (the sort only: no row gather) and moe_plan_tiles in ONE launch: the stable rank
 * and the schedule need nothing from each other -- both start from the expert ids -- so the
 * plan's serial loops (a single work-group) run beside the ranking work-groups instead of after
 * them, and the histogram launch goes too (every work-group counts the experts of the
 * assignments it needs by itself).  Outputs are those of the two calls, bit for bit; no
 * workspace is needed.  For T*k <= MOE_PERMUTE_PLAN_MAX (every work-group reads all ids);
 * MOE_ERR_UNSUPPORTED beyond: use the two calls.  T >= 1. */
#define MOE_PERMUTE_PLAN_MAX 32768
MOE_API int moe_permute_plan(const int32_t* expert_idx, int T, int E, int k,
                   int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv_perm,
                   int tile_m, int n_bins, int q_tokens, int policy,
                   moe_tile* tiles, int tile_capacity, int32_t* plan_hdr, int32_t* sched, void* stream);

/* The same schedule over SOME of the experts: expert_ids (HOST array of n_ids ids in [0,E), any
 * order, repeats allowed) names the experts that take part; the others count as empty.  This
 * is how the experts of Alg. 1 step 5 are run in groups as their weights become available
 * (section 4.3): one plan + moe_grouped_ffn per group, over the same counts, offsets and rows. */
MOE_API int moe_plan_tiles_subset(const int32_t* counts, const int32_t* offsets, int E, int A,
                   int tile_m, int n_bins, int q_tokens, int policy,
                   const int32_t* expert_ids /*host*/, int n_ids,
                   moe_tile* tiles, int tile_capacity, int32_t* plan_hdr, int32_t* sched,
                   void* stream);

/* ------------------------------------------------------------------------------------------
 * Alg. 2 (token rebalancing) as printed, for a group of G GPUs, on the device and without a host
 * loop (section 4.2; the paper runs it as tensor operations driven by a host loop on every GPU
 * and reports 20-31 % of the layer's time for it, section 5.3).
 *
 *   S[g_from, e, g_to] = tokens that GPU g_from sends to GPU g_to for expert e  (S_initial from
 *   Alg. 1 step 3: everything goes to the expert's home GPU).
 *   A GPU's load is everything addressed to it; the target is the floor of the mean load.  One
 *   move takes tokens off the most loaded GPU: of the sources that send to it, the one sending
 *   most (summed over experts), and of that source's blocks there the largest; they go to the
 *   least loaded GPU, as many as bring it up to the target, at most the whole block.  No move is
 *   made -- and the schedule is final -- once no GPU is above the target, once that largest block
 *   is smaller than q, or once the least loaded GPU has room for fewer than q tokens (or is the
 *   most loaded one itself).  Equal values: the lowest index, in every choice.
 *
 *   s_initial [G_src, E, G] int32 (device)     s_out [G_src, E, G] int32 (device; may alias s_initial)
 *   info [4 + MOE_MAX_BINS] int32 (device) or NULL: [0] moves made, [1] the target, [2] why the loop
 *        ended (0 no GPU above the average, 1 block below q, 2 no room on the least loaded GPU,
 *        3 iteration cap), [4 ..] the GPUs' loads afterwards
 * Requires G_src, G <= MOE_MAX_BINS, E <= MOE_MAX_EXPERTS, q_tokens >= 1 and S at most 128 KiB.
 * Entries must be non-negative with a total below 2^26.
 */
MOE_API int moe_rebalance(const int32_t* s_initial, int G_src, int E, int G, int q_tokens,
                          int32_t* s_out, int32_t* info, void* stream);

/* ------------------------------------------------------------------------------------------
 * Weight layout of the FFN kernels.  The paper writes an expert as x W1 W2 with W1: d x F and
 * W2: F x d (section 4.4).  The kernels read every weight matrix "output-major": row n holds
 * the d (or F) input coefficients of output feature n, i.e. the transpose, so that the
 * contraction index is contiguous for both operands.  moe_pack_weights makes that layout once,
 * outside the hot path.
 *
 *   w_a [n, K, N] dt : n matrices in the paper's orientation (K inputs, N outputs)
 *   w_b [n, K, N] dt or NULL.  If given (SwiGLU: w_a = W_gate, w_b = W_up) the output has 2N
 *        rows per matrix, in blocks of 32 rows: block 2j holds outputs [32j, 32j+32) of w_a,
 *        block 2j+1 the same outputs of w_b.  Requires N % 32 == 0.
 *   out  [n, N or 2N, K] dt
 * MOE_BF16 also orders the rows inside every block of 32 for the 16x16x32 matrix instruction of
 * the FFN kernels: packed row 16 h + j of a block holds the block's output 2 j + h (h = 0, 1;
 * j = 0 .. 15), so that a lane's two accumulator columns are adjacent outputs.  Requires
 * N % 32 == 0 then.  MOE_F32 keeps the outputs in order.
 */
MOE_API int moe_pack_weights(const void* w_a, const void* w_b, int n, int K, int N, moe_dtype dt,
                     void* out, void* stream);

/* The same layout for the second matrix of an expert (W2 / W_down: F inputs, d outputs, section
 * 4.4), in the number format the second product of moe_grouped_ffn reads:
 *
 *   w   [n, F, d] dt
 *   out [n, d, F]   MOE_F32: fp32 as given.  MOE_BF16: rows ordered as by moe_pack_weights
 *        (d % 32 == 0) and every value converted to IEEE half
 *        (binary16, nearest-even).  That is exact for bf16 values of magnitude 2^-14 .. 65504;
 *        smaller ones are rounded to the half subnormals (absolute error <= 2^-25), larger ones
 *        become infinite.  The kernels keep the hidden activations in half as well (see
 *        moe_grouped_ffn), saturated at +-65504.
 */
MOE_API int moe_pack_w_out(const void* w, int n, int F, int d, moe_dtype dt, void* out, void* stream);

/* ------------------------------------------------------------------------------------------
 * Step 5, expert processing (Alg. 1 "experts(S, x')"; section 2: two dense layers with an
 * activation between; section 4.4: no biases).  For every row r of expert e
 * (offsets[e] <= r < offsets[e+1]):
 *
 *   MOE_RELU    y_perm[r] = max(0, x_perm[r] W1_e) W2_e
 *   MOE_SWIGLU  y_perm[r] = (silu(x_perm[r] Wgate_e) * (x_perm[r] Wup_e)) Wdown_e,  silu(z) = z/(1+exp(-z))
 *
 * The work is taken from the tile table of moe_plan_tiles: each XCD runs the tiles of its bin.
 *
 *   x_perm [A,d] dt
 *   w_in  : device array of E device pointers; w_in[e] = packed [F,d] (ReLU) or [2F,d] (SwiGLU,
 *           gate/up interleaved by moe_pack_weights)
 *   w_out : device array of E device pointers; w_out[e] = packed [d,F] from moe_pack_w_out
 *   tiles, plan_hdr : from moe_plan_tiles with the same E and A; tile_m as given to the plan:
 *           moe_ffn_tile_m(dt), or for bf16 128 or 256 (moe_ffn_pick_tile_m).  The bf16 kernels
 *           hand the tiles of a bin to its work-groups through the counters at
 *           plan_hdr[MOE_PLAN_HDR_CTR ...]: they must be zero on entry (moe_plan_tiles leaves
 *           them so) and are zero again when the call's kernels have finished, so a plan can be
 *           run any number of times; two calls that use the same plan_hdr must not overlap.
 *   h_scratch [A,F] : hidden activations (written, then read); fp32 for MOE_F32, 2 bytes per
 *           value for MOE_BF16
 *   y_perm    [A,d] fp32 out
 * Requires d % 64 == 0 and F % 64 == 0 for MOE_BF16 (d % 4, F % 4 for MOE_F32).  MOE_BF16
 * accumulates both products in fp32 and rounds the hidden activations once, to IEEE half: 11
 * significant bits, so the result is within about 1e-3 of the output's RMS of the exact one
 * (bf16 activations would be eight times coarser); a hidden activation beyond +-65504 (the
 * largest half value) is stored as +-65504: it saturates, y_perm stays finite.  The bf16 kernels
 * are persistent launches laid out for the whole MI355X (256 compute units in 8 XCDs):
 * MOE_ERR_UNSUPPORTED on a device that reports another count.
 */
MOE_API int moe_ffn_tile_m(moe_dtype dt);
/* bf16 has two tile heights, 128 and 256 rows; this picks one from the mean rows per expert
 * (256 once A/E >= 1024: under skewed routing most experts hold far fewer rows than the mean, and
 * their tiles are mostly empty at 256 rows).  Plan and FFN must be given the same value. */
MOE_API int moe_ffn_pick_tile_m(moe_dtype dt, int A, int E);

/* Each bf16 tile height has two families of kernels that compute the same bits.
 * 128 rows: one stages both operands through an LDS ring (eight wavefronts), the other streams
 * the weights straight into registers (meant for experts with few rows, where a product costs
 * the fetch of its weights: section 4.4's regime below q; it covers the ReLU first product and
 * the second product, the scatter form from F >= 512 on).  The LDS ring is the default: it is
 * the faster one on every workload measured so far.
 * 256 rows: the LDS ring with eight wavefronts of 128 x 64 outputs each, and four wavefronts of
 * 128 x 128 (a third less LDS traffic per multiply-add, which is what the arithmetic-bound case
 * pays for; d and F multiples of 64, at least 256).  The four wavefronts are the default; only
 * they offer the row gather of moe_grouped_ffn_fused at this height.
 * moe_ffn_kernel_mode sets the choice for the process -- 0 default, 1 the LDS ring with eight
 * wavefronts at both heights, 2 the streaming kernels wherever they cover the call, -1 leaves
 * it -- and returns the previous setting (a negative moe_status on a bad argument).  For
 * measurements and tests. */
MOE_API int moe_ffn_kernel_mode(int mode);

MOE_API int moe_grouped_ffn(const void* x_perm, int A, int d, int F, int E, moe_act act, moe_dtype dt,
                    const void* const* w_in, const void* const* w_out,
                    const moe_tile* tiles, int32_t* plan_hdr, int tile_m,
                    void* h_scratch, float* y_perm, void* stream);

/* One of the two grouped GEMMs of moe_grouped_ffn on its own (same kernels, same arguments):
 * phase 1 computes the hidden activations H = act(x_perm W_in) into h_scratch (w_out and y_perm
 * may be NULL), phase 2 computes y_perm = H W_out from h_scratch (x_perm and w_in may be NULL).
 * moe_grouped_ffn is phase 1 followed by phase 2 on the same stream.  Lets a caller time, or
 * interleave other work between, the two products of section 4.4's x W1 W2. */
MOE_API int moe_grouped_ffn_phase(int phase, const void* x_perm, int A, int d, int F, int E, moe_act act,
                                  moe_dtype dt, const void* const* w_in, const void* const* w_out,
                                  const moe_tile* tiles, int32_t* plan_hdr, int tile_m,
                                  void* h_scratch, float* y_perm, void* stream);

/* Steps 5 and 6 in one call for top-1 routing (k = 1, so A = T and row r of x_perm is token
 * perm[r]): the second product writes its rows straight to their tokens' places, weighted,
 *
 *   y[perm[r]] = gate_w[perm[r]] * FFN_e(x_perm[r])          r in expert e's group
 *
 * which is what moe_grouped_ffn followed by moe_unpermute_combine computes (bit for bit: one
 * fp32 multiplication either way) without writing and re-reading y_perm.
 *
 *   perm   [T] int32 : from moe_permute (a permutation of 0..T-1)
 *   gate_w [T] fp32 or NULL (all ones)
 *   y      [T,d] fp32 out; every row is written exactly once
 * other arguments as moe_grouped_ffn.  MOE_BF16 only, F >= 512 (MOE_ERR_UNSUPPORTED otherwise:
 * use the two separate calls).
 */
MOE_API int moe_grouped_ffn_top1(const void* x_perm, int T, int d, int F, int E, moe_act act, moe_dtype dt,
                                 const void* const* w_in, const void* const* w_out,
                                 const moe_tile* tiles, int32_t* plan_hdr, int tile_m,
                                 void* h_scratch, const int32_t* perm, const float* gate_w, float* y,
                                 void* stream);
/* One of its two products on its own, like moe_grouped_ffn_phase (phase 1 is the same first
 * product; perm, gate_w and y may then be NULL). */
MOE_API int moe_grouped_ffn_top1_phase(int phase, const void* x_perm, int T, int d, int F, int E, moe_act act,
                                       moe_dtype dt, const void* const* w_in, const void* const* w_out,
                                       const moe_tile* tiles, int32_t* plan_hdr, int tile_m,
                                       void* h_scratch, const int32_t* perm, const float* gate_w, float* y,
                                       void* stream);

/* Steps 4 (the row gather), 5 and, for top-1 routing, 6 in one call: the first product fetches
 * its rows from x itself,
 *
 *   row r of expert e's group = x[perm[r] / k]                (what moe_permute writes to x_perm[r])
 *
 * so moe_permute can be called without x / x_perm (it then only sorts), and x_perm is neither
 * written nor read.  The results are those of the separate calls, bit for bit.
 *
 *   x      [T,d] dt
 *   perm   [T*k] int32 : from moe_permute
 *   k == 1 : y_out = y [T,d] fp32, y[perm[r]] = gate_w[perm[r]] * FFN_e(x[perm[r]]) as in
 *            moe_grouped_ffn_top1 (gate_w [T] fp32 or NULL; F >= 512)
 *   k  > 1 : y_out = y_perm [T*k,d] fp32 as in moe_grouped_ffn (gate_w is not used); the caller
 *            combines with moe_unpermute_combine
 * other arguments as moe_grouped_ffn.  MOE_BF16 only, d >= 256, x smaller than 4 GiB; with
 * tile_m = 256 only while moe_ffn_kernel_mode is not 1 (MOE_ERR_UNSUPPORTED otherwise: use the
 * separate calls).
 */
MOE_API int moe_grouped_ffn_fused(const void* x, int T, int d, int F, int E, int k, moe_act act, moe_dtype dt,
                                  const void* const* w_in, const void* const* w_out,
                                  const moe_tile* tiles, int32_t* plan_hdr, int tile_m,
                                  void* h_scratch, const int32_t* perm, const float* gate_w, float* y_out,
                                  void* stream);
/* One of its two products on its own, like moe_grouped_ffn_phase (phase 2 does not read x). */
MOE_API int moe_grouped_ffn_fused_phase(int phase, const void* x, int T, int d, int F, int E, int k, moe_act act,
                                        moe_dtype dt, const void* const* w_in, const void* const* w_out,
                                        const moe_tile* tiles, int32_t* plan_hdr, int tile_m,
                                        void* h_scratch, const int32_t* perm, const float* gate_w,
                                        float* y_out, void* stream);

/* ------------------------------------------------------------------------------------------
 * Step 6 (Alg. 1 "reconstruct"; section 2: the experts' outputs are weighted by the router's
 * values and combined):
 *
 *   y[t] = sum_{j<k} gate_w[t,j] * y_perm[inv_perm[t*k+j]]  (+ shared[t]),  j ascending, fp32
 *
 *   y_perm [A,d] fp32   inv_perm [A] int32   gate_w [T,k] fp32 (NULL = all ones)
 *   shared [T,d] fp32 or NULL (output of an always-on shared expert)      y [T,d] fp32 out
 */
MOE_API int moe_unpermute_combine(const float* y_perm, const int32_t* inv_perm, const float* gate_w,
                          const float* shared, int T, int d, int k, float* y, void* stream);

/* ------------------------------------------------------------------------------------------
 * Asynchronous expert fetching (section 4.3): experts whose weights live in pinned host
 * memory are copied into device slots on a stream of the engine's own while the caller's
 * stream computes; a slot whose expert has finished is overwritten by the next expert
 * (nothing is written back).  The engine owns one stream and two events per slot.
 *
 *   moe_prefetch_create   n_slots >= 1 slots of slot_bytes each, laid out back to back from
 *                         slot_base (device memory of the caller)
 *   moe_prefetch_experts  enqueue the copies of n experts, in the given order.  Expert i is
 *                         copied from host_w[i] (HOST pinned pointer, bytes_each bytes, already
 *                         in the packed layout) into slot (first free, else the slot released
 *                         longest ago); slot_ptrs_out[i] (HOST array) receives the slot's
 *                         device address.  A copy into a slot in use waits for that slot's
 *                         release.  MOE_ERR_CAPACITY if a slot is needed and none was released.
 *   moe_prefetch_wait     make `stream` wait until expert_id's copy has landed (before its FFN).
 *                         Copies complete in the order they were enqueued, so one wait for the
 *                         expert fetched last covers every expert fetched before it.
 *   moe_prefetch_release  declare that work enqueued so far on `stream` is the last use of
 *                         expert_id's slot (after its FFN); the slot may then be overwritten
 *   moe_prefetch_reset    between two passes over the experts: every resident expert must have
 *                         been released; afterwards no expert counts as resident and the next
 *                         fetches take the slots in order 0, 1, 2, ... (an overwrite still waits
 *                         for the slot's last use)
 *   moe_prefetch_destroy  waits for the engine's stream, frees stream and events
 */
typedef struct moe_prefetch moe_prefetch;

MOE_API int moe_prefetch_create(moe_prefetch** h, int n_slots, size_t slot_bytes, void* slot_base);
MOE_API int moe_prefetch_experts(moe_prefetch* h, const int32_t* expert_ids /*host*/, int n,
                         const void* const* host_w /*host array of pinned host pointers*/,
                         size_t bytes_each, const void** slot_ptrs_out /*host*/);
MOE_API int moe_prefetch_wait(moe_prefetch* h, int expert_id, void* stream);
MOE_API int moe_prefetch_release(moe_prefetch* h, int expert_id, void* stream);
MOE_API int moe_prefetch_reset(moe_prefetch* h);
MOE_API int moe_prefetch_destroy(moe_prefetch* h);

/* The addresses that moe_prefetch_experts chose, entered into the device pointer tables that
 * moe_grouped_ffn reads (the library alone decides which slot an expert goes to; the caller
 * passes the answers on before the expert's FFN).  For i < n:
 *
 *   w_in[expert_ids[i]] = ptrs[i]        w_out[expert_ids[i]] = ptrs[i] + out_offset   (w_out may be NULL)
 *
 * written by a small kernel on `stream`, ordered like every other call (a host-to-device copy
 * of the table would queue behind the expert copies on the DMA engine).
 *   w_in, w_out : device arrays of E device pointers      expert_ids, ptrs : HOST arrays of n
 *   out_offset  : bytes from an expert's first matrix to its second inside a slot
 */
MOE_API int moe_set_expert_pointers(const void** w_in, const void** w_out, int E, const int32_t* expert_ids /*host*/,
                                    int n, const void* const* ptrs /*host*/, size_t out_offset, void* stream);

/* Token threshold q of section 4.4, Eq. 4: the row count above which running an expert takes
 * longer than fetching its weights, q = phi * d_type / (2 * beta), rounded up.
 *   phi: arithmetic rate in FLOP/s   d_type: bytes per weight   beta: fetch rate in bytes/s */
MOE_API int moe_token_threshold(double phi, int d_type, double beta);

/* Scratch sizes.  op selects the call. */
enum { MOE_OP_PERMUTE = 1 };
MOE_API size_t moe_workspace_bytes(int op, int T, int d, int F, int E, int k, moe_dtype dt);

/* Diagnostic: a plain device-to-device copy of `bytes` bytes (a multiple of 16; src and dst
 * 16-byte aligned, not overlapping), one kernel on `stream`.  It moves a known amount of data
 * through HBM and serves as the reference when hardware traffic counters are scaled. */
MOE_API int moe_copy_bytes(const void* src /*device*/, void* dst /*device*/, size_t bytes, void* stream);

MOE_API const char* moe_last_error(void);
MOE_API const char* moe_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MOE_H */
