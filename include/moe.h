/* moe.h -- C ABI of the per-GPU Mixture-of-Experts expert layer for AMD MI355X (gfx950).
 *
 * The layer is the one GEM (GPU-variability-aware expert-to-GPU mapping) profiles and balances:
 * a router selects the top-k of E experts for every token (paper Sec. 2.1), the token is sent to
 * the GPU holding those experts, each expert is a feed-forward network, and the results return
 * to the token (Sec. 7).  The latency of this layer as a function of the number of tokens a GPU
 * receives is the per-GPU curve C_g(n) of the paper's score (Sec. 3.3.3, Eq. 1); the per-expert
 * token counts are one row of its expert-utilisation trace (Sec. 3.3.1).  The paper gives no
 * formulas for the layer itself; the ones used here are the standard ones: softmax over the k
 * selected router logits, SwiGLU experts  y = W2^T( silu(W1^T x) * (W3^T x) ).
 *
 * Conventions
 *   - Every tensor pointer is DEVICE memory owned by the caller, unless marked "host".
 *     The library allocates no device memory: its scratch is the workspace given to moe_create.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All calls enqueue
 *     work on it and return; none synchronises with the host.
 *   - bf16 tensors are passed as void*; they are row-major and 16-byte aligned.
 *   - Shapes: T tokens, d model width, f expert width, E experts seen by the router, k experts
 *     per token, experts [e_lo, e_lo+E_local) resident on this GPU.  d and f must be multiples
 *     of 64; 1 <= k <= min(E, 16); E <= 256; 1 <= E_local <= E.
 *   - Errors are return codes.  Arguments are validated on the host before any launch: a call that
 *     returns MOE_ERR_INVALID_ARG, MOE_ERR_UNSUPPORTED_SHAPE or MOE_ERR_WORKSPACE_TOO_SMALL has launched
 *     nothing.  MOE_ERR_DEVICE reports a HIP call that failed part-way; in a call of several stages
 *     (moe_permute, moe_grouped_ffn, moe_layer_forward) the stages enqueued before it still run, and the
 *     outputs are then undefined.  T == 0 is MOE_OK and a no-op.
 *   - Calls on one moe_ctx must not overlap in time (they share its workspace).
 *   - The calls that take a stream only launch kernels on it (no memsets, no allocation, no host
 *     synchronisation), so they may be recorded under stream capture and replayed as a HIP graph; the
 *     exceptions are contexts created with MOE_FLAG_STAGE_EVENTS (they record events), moe_profile_ffn
 *     moe_measure_mfma_rate(_of) and moe_measure_hbm_read_rate (they time and wait).
 */
#ifndef MOE_H_
#define MOE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct moe_ctx moe_ctx; /* opaque, host memory */

typedef enum {
    MOE_OK = 0,
    MOE_ERR_INVALID_ARG = 1,        /* null / misaligned pointer, T out of range, ...          */
    MOE_ERR_UNSUPPORTED_SHAPE = 2,  /* shape outside the limits listed above                   */
    MOE_ERR_WORKSPACE_TOO_SMALL = 3,
    MOE_ERR_DEVICE = 4              /* a HIP call failed (launch error, wrong architecture)    */
} moe_status;

typedef struct {
    int32_t T_max;    /* largest T any call will pass                                          */
    int32_t d, f;     /* model width, expert FFN width                                         */
    int32_t E, k;     /* experts seen by the router, experts per token                         */
    int32_t e_lo;     /* first resident expert                                                 */
    int32_t E_local;  /* number of resident experts (== E: all of them)                        */
    uint32_t flags;   /* MOE_FLAG_*                                                            */
} moe_shape;

#define MOE_FLAG_STAGE_EVENTS 1u /* moe_layer_forward records HIP events around every stage   */

enum { MOE_STAGE_ROUTE = 0, MOE_STAGE_PERMUTE = 1, MOE_STAGE_GEMM1 = 2, MOE_STAGE_GEMM2 = 3,
       MOE_STAGE_COMBINE = 4, MOE_NUM_STAGES = 5 };

const char* moe_status_string(moe_status s);

/* Text of the most recent failing HIP call behind a MOE_ERR_DEVICE on this thread, or of a size limit that
 * a call without a context exceeded ("" if none).
 * The pointer stays valid; the text changes with the next device error. */
const char* moe_last_device_error(void);

/* Bytes of device workspace a context of this shape needs (0 if the shape is unsupported). */
size_t moe_workspace_bytes(const moe_shape* shape /* host */);

/* Creates a context over a caller-owned device workspace of at least moe_workspace_bytes().
 * The workspace must stay valid until moe_destroy.  Must be called with the target device
 * current; clears a few KB of the workspace with a blocking memset.  *ctx is NULL on error. */
moe_status moe_create(moe_ctx** ctx, const moe_shape* shape /* host */, void* workspace,
                      size_t workspace_bytes);
void moe_destroy(moe_ctx* ctx);

/* Number of rows the staged buffers (xp, y, tok_of) must hold for T tokens:
 * T * min(k, E_local), the largest possible number of local (token, expert) assignments. */
int64_t moe_rows_capacity(const moe_shape* shape /* host */, int32_t T);

/* ---- one-off, at model-load time (the analogue of loading each expert's weights onto its
 * assigned GPU, paper Sec. 3.3.4); not part of the layer latency ------------------------------ */

/* Router matrix Wg [d, E] fp32 row-major -> opaque packed form (two bf16 terms per weight, laid
 * out in the order the matrix-core operand fragments are loaded). */
size_t moe_packed_router_bytes(const moe_shape* shape /* host */);
moe_status moe_pack_router(moe_ctx* ctx, const float* Wg, void* router_packed, void* stream);

/* Expert weights W1, W3 [E_local, d, f] and W2 [E_local, f, d], bf16 row-major -> opaque packed
 * form (3 * E_local * d * f bf16 values: every 32-column x 16-reduction-element block stored as the
 * 1 KB matrix-core operand fragment one wavefront loads; W1 and W3 interleaved in blocks of 32
 * output columns so one accumulator tile holds both branches of the SwiGLU). */
size_t moe_packed_weight_bytes(const moe_shape* shape /* host */);
moe_status moe_pack_weights(moe_ctx* ctx, const void* W1, const void* W3, const void* W2,
                            void* packed, void* stream);

/* ---- the hot path ---------------------------------------------------------------------------- */

/* Router (paper Sec. 2.1: per-token choice of the k experts; Sec. 3.3.1: its output is the trace):
 *   logit[t,e] = sum_i x[t,i] * Wg[i,e] (+ bias[e]);  topk_idx[t,0..k) = the k largest, slot 0
 *   the largest, equal logits resolved to the lower expert index;  topk_w[t,j] = softmax over
 *   the k selected logits;  counts[e] = number of (t, j) with topk_idx[t,j] == e, over all E.
 * x [T, d] bf16; bias [E] fp32 or NULL; topk_idx [T, k] int32; topk_w [T, k] fp32;
 * counts [E] int32 (overwritten). */
moe_status moe_route(moe_ctx* ctx, const void* x, const void* router_packed, const float* bias,
                     int32_t T, int32_t* topk_idx, float* topk_w, int32_t* counts, void* stream);

/* Dispatch by expert (paper Sec. 2.1: each token goes to where its experts are hosted):
 *   offsets[e'] = number of assignments to resident experts before e_lo + e' (exclusive prefix
 *   sum, offsets[E_local] = number of local assignments);  the destination row of (t, j) with
 *   e = topk_idx[t,j] resident is row_of[t,j] = offsets[e-e_lo] + #{t' < t : t' selected e}
 *   (expert-contiguous, ascending token order inside an expert); row_of = -1 for non-resident
 *   experts;  tok_of[row] = t;  xp[row, :] = x[t, :].
 * xp [rows_capacity, d] bf16 or NULL (skip the row copy); offsets [E_local+1]; row_of [T, k];
 * tok_of [rows_capacity]. */
moe_status moe_permute(moe_ctx* ctx, const void* x, const int32_t* topk_idx, int32_t T, void* xp,
                       int32_t* offsets, int32_t* row_of, int32_t* tok_of, void* stream);

/* moe_permute for callers that can neither allocate device memory nor bring a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  No context: the shape comes as
 * arguments (d is only used for the row copy), the outputs are those of moe_permute, bit for bit.  The call
 * allocates nothing and frees nothing; its only scratch, the per-256-token-block expert histograms, is a
 * static device array of 1 MiB that every GPU the library runs on holds until the process ends.  Limit:
 * ceil(T / 256) * E_local <= 262144 entries (e.g. T = 2^20 with up to 64 resident experts, T = 262144 with
 * 256), otherwise MOE_ERR_WORKSPACE_TOO_SMALL with the sizes in moe_last_device_error(); T <= 2^20.  The array
 * keeps the previous call's contents (every entry a call reads it has written itself first), and calls that
 * overlap in time on one GPU share it and race: run them on one stream, or otherwise one after the other.
 * The first call on a device looks up the array's device address (no allocation, but do it outside a
 * stream capture). */
moe_status moe_permute_noalloc(const void* x, const int32_t* topk_idx, int32_t T, int32_t d, int32_t E,
                               int32_t k, int32_t e_lo, int32_t E_local, void* xp, int32_t* offsets,
                               int32_t* row_of, int32_t* tok_of, void* stream);

/* Expert FFN over expert-contiguous rows (the expert kernel the paper profiles in isolation, Sec. 3.3.2):
 *   for offsets[e'] <= r < offsets[e'+1]:
 *       y[r, :] = W2[e']^T ( silu(W1[e']^T xp[r]) * (W3[e']^T xp[r]) )
 *   bf16 operands, fp32 accumulation; the intermediate [rows, f] is stored as bf16 in the
 *   workspace.  Experts with no rows cost nothing and their weights are not read.
 * xp, y [n_rows_cap, d] bf16; offsets [E_local+1] (device; values are not read by the host);
 * n_rows_cap: host upper bound on offsets[E_local], at most moe_rows_capacity(shape, T_max).  The launches
 * are sized from it (the per-expert counts stay on the device), so a tight bound is cheaper than a loose
 * one; at low loads (up to 192 rows per expert on average) the second GEMM runs as several reduction
 * ranges whose fp32 partial sums are added in a fixed order.  The bound is checked on the device: if
 * offsets[E_local] exceeds n_rows_cap the call computes nothing (no row of y is written) and sets the flag
 * moe_ffn_refused_flag points to; the host cannot see that without reading the flag, the return code stays
 * MOE_OK. */
moe_status moe_grouped_ffn(moe_ctx* ctx, const void* xp, const int32_t* offsets,
                           int32_t n_rows_cap, const void* packed, void* y, void* stream);

/* Weighted return to token order (paper Sec. 7: tokens return to their origin):
 *   out[t, :] = sum_j topk_w[t,j] * y[row_of[t,j], :]   (slots with row_of < 0 contribute 0),
 *   summed in slot order in fp32, one write per output element, no atomics.
 * y [rows_capacity, d] bf16; out [T, d] bf16. */
moe_status moe_combine(moe_ctx* ctx, const void* y, const int32_t* row_of, const float* topk_w,
                       int32_t T, void* out, void* stream);

/* The whole layer on one stream with no host synchronisation: route, dispatch, experts, combine.
 * Intermediates live in the workspace; the row copy is folded into the first GEMM's operand load.
 * With E_local < E, `out` is this GPU's partial sum (tokens with no resident expert give 0).
 * counts_out [E] int32 or NULL. */
moe_status moe_layer_forward(moe_ctx* ctx, const void* x, const void* router_packed,
                             const float* bias, const void* packed, int32_t T, void* out,
                             int32_t* counts_out, void* stream);

/* ---- introspection --------------------------------------------------------------------------- */

/* Mean milliseconds of each stage over the moe_layer_forward calls made since the previous
 * read-out (at most the 64 most recent) on a context created with MOE_FLAG_STAGE_EVENTS.
 * Blocks until the last of those calls has completed.  ms: host, MOE_NUM_STAGES floats. */
moe_status moe_stage_times(moe_ctx* ctx, float* ms /* host */);

/* Largest token-tile height of the expert GEMMs for this shape.  An expert's rows are cut into
 * ceil(n / height) tiles of nearly equal height (multiples of 32 rows); the work per tile grows in
 * steps of 32 rows, which sets the staircase of the latency-vs-load curve (the
 * paper's tile boundaries, Sec. 3.3.2). */
int32_t moe_tile_rows(const moe_ctx* ctx);

/* Variability-profiling microbenchmark (paper Sec. 3.3.2, "Step-2"): launches the isolated expert
 * kernels (moe_grouped_ffn: GEMM1 + SwiGLU + GEMM2) on synthetic rows at each target token count
 * and records the average latency -- one sample of this GPU's token-vs-latency curve C_g(n) per
 * count.  For point i, token_counts[i] rows of xp are spread evenly over the E_local resident
 * experts (the first token_counts[i] % E_local experts get one more), the kernels are launched
 * warmup + iters times on `stream`, and ms[i] = mean milliseconds per launch over the timed ones
 * (HIP events on `stream`).  xp and y: device, at least max(token_counts) rows of d bf16 values each;
 * token_counts and ms: host, n_points entries; every count <= moe_rows_capacity(shape, T_max).
 * Unlike the hot-path calls this one BLOCKS until the measurements are done, and it overwrites the
 * context's offsets scratch. */
moe_status moe_profile_ffn(moe_ctx* ctx, const void* xp, const void* packed, void* y,
                           const int32_t* token_counts /* host */, int32_t n_points, int32_t warmup,
                           int32_t iters, float* ms /* host */, void* stream);

/* ---- host-side steps (everything below up to moe_gem_place takes HOST pointers and runs on the CPU, as in
 * the paper; the inputs are what the GPU path produces) ------------------------------------------------- */

/* Sampling plan of the variability profiler (paper Sec. 3.3.2, Step-2: latency jumps at tile boundaries,
 * so sample there; sample sparsely at high counts).  Token counts to measure, ascending, no duplicates:
 * 1; every multiple m*boundary up to min(dense_max, n_max) together with m*boundary + after (the first
 * count at which the jump is complete) where that is <= n_max; then every sparse_step tokens from the last
 * dense boundary on, below n_max; and n_max.  Requires boundary, sparse_step, n_max >= 1,
 * 1 <= after <= boundary, dense_max >= 0.  *n_out = number of counts; with cap == 0 nothing is written (size
 * query); cap < *n_out gives MOE_ERR_WORKSPACE_TOO_SMALL. */
moe_status moe_curve_sample_counts(int32_t boundary, int32_t dense_max, int32_t n_max, int32_t sparse_step,
                                   int32_t after, int32_t* counts_out /* [cap] */, int32_t cap, int32_t* n_out);

/* The curve C_g(n) rebuilt from n_samples measured points (counts strictly ascending, ms their latencies;
 * Sec. 3.3.2: linear interpolation between samples): ms_out[i] = latency at tokens[i] tokens = the straight
 * line between the neighbouring samples, the first sample's value below it, the last one's above it, 0 for
 * tokens <= 0.  The mapping search (moe_gem_*) reads its curves the same way. */
moe_status moe_curve_eval(const int32_t* counts, const double* ms, int32_t n_samples, const int32_t* tokens,
                          int32_t n_tokens, double* ms_out /* [n_tokens] */);

/* Sum of C_g(n) over n_lo <= n <= n_hi: the kernel time a sweep of every token count would cost, for the
 * comparison with the sampled profile (Sec. 4.6 of the paper reports that ratio). */
moe_status moe_curve_sum(const int32_t* counts, const double* ms, int32_t n_samples, int32_t n_lo, int32_t n_hi,
                         double* sum_out);

/* Statistics of the expert-utilisation trace (paper Sec. 3.3.1, Step-1; Sec. 3.2): trace[t*E + e] = tokens
 * routed to expert e at step t.  u_out[e] = mean over the S steps.  r_out[a*E + b] = Pearson correlation
 * coefficient of the loads of experts a and b across the steps (NaN if either load is constant). */
moe_status moe_trace_mean_utilisation(const int32_t* trace, int32_t S, int32_t E, double* u_out /* [E] */);
moe_status moe_trace_correlation(const int32_t* trace, int32_t S, int32_t E, double* r_out /* [E*E] */);

/* Mapping search (paper Sec. 3.3.3 "Step-3", Eq. 1; appendix algorithms for the initial mapping, the
 * refinement and the restarts).  trace as above (the counts_out rows of S consecutive calls); one
 * token-vs-latency curve per GPU (moe_profile_ffn samples): GPU g's samples are curve_counts / curve_ms
 * [curve_offsets[g], curve_offsets[g+1]), token counts strictly ascending, read as in moe_curve_eval.
 * E must be a multiple of G: every GPU hosts E / G experts.  mapping[e] = GPU of expert e. */

/* S(M) = sum over steps of max over GPUs of C_g(tokens routed to GPU g at that step)  (Eq. 1). */
moe_status moe_gem_score(const int32_t* trace, int32_t S, int32_t E, int32_t G, const int32_t* curve_counts,
                         const float* curve_ms, const int32_t* curve_offsets /* [G+1] */,
                         const int32_t* mapping /* [E] */, double* score_out);

/* K restarts of: greedy initial mapping (experts by mean utilisation, heaviest first, each on the
 * GPU with a free slot that gives the lowest score of the partial mapping; restart i > 0 sorts by
 * u_e * (1 + 0.2 * noise[i*E + e]), noise in [-1, 1) drawn by the caller), then repeated best
 * cross-GPU swap until the best swap lowers the score by less than 0.1 %.  Returns the
 * lowest-scoring mapping, its score and (optionally) the number of swaps its refinement took.
 * noise may be NULL when K == 1.  Ties go to the lower expert / GPU index and the first pair. */
moe_status moe_gem_place(const int32_t* trace, int32_t S, int32_t E, int32_t G, const int32_t* curve_counts,
                         const float* curve_ms, const int32_t* curve_offsets /* [G+1] */,
                         const float* noise /* [K][E] */, int32_t K, int32_t* mapping_out /* [E] */,
                         double* score_out, int32_t* swaps_out /* or NULL */);

/* Tuning hook: force the token-tile class of the expert GEMMs (1: row tiles of up to 288 rows, the main
 * class; 5: the class of decode-sized loads -- two wavefronts per workgroup, 128 weight rows and up to 64
 * token rows per work item, four workgroups to a compute unit; 0, 2, 3, 4: alternative kernels with row tiles
 * of up to 128, 64, 32, 256 rows kept for tuning runs; -1: choose from the expected rows per expert, the
 * default: class 0 below 12 rows per expert, class 5 up to 24, class 1 above). */
moe_status moe_set_tile_class(moe_ctx* ctx, int32_t tile_class);

/* Measurement aid for roofline reports: the bf16 matrix-core rate this device SUSTAINS under a load of
 * nothing but v_mfma_f32_16x16x32_bf16 (the instruction the grouped GEMM issues) on changing pseudo-random
 * operands (no memory traffic, every SIMD of every compute unit busy, independent accumulators), in
 * TFLOP/s.  The published peak assumes the maximum clock; under a dense MFMA load the chip runs at the clock
 * its power limit allows.  Runs `launches` >= 1 launches of iters_per_wave * 128 MFMAs per wavefront on
 * `stream`, times them with events and waits for them.
 * tflops: host pointer.  Errors: MOE_ERR_INVALID_ARG, MOE_ERR_DEVICE. */
moe_status moe_measure_mfma_rate(int32_t iters_per_wave, int32_t launches, float* tflops /* host */, void* stream);
/* The same measurement on a chosen instruction shape: 0 = v_mfma_f32_32x32x16_bf16 (half as many instructions
 * for the same flop), 1 = v_mfma_f32_16x16x32_bf16 (identical to moe_measure_mfma_rate).  Under the power limit
 * the sustained rate depends on the shape.  Errors as above. */
moe_status moe_measure_mfma_rate_of(int32_t shape, int32_t iters_per_wave, int32_t launches,
                                    float* tflops /* host */, void* stream);

/* Measurement aid for roofline reports: the rate at which this device streams `bytes` bytes (>= 16; the tail
 * below a multiple of 16 is not read) of the device buffer `buf` (16-byte aligned, only read) through a
 * read-only kernel whose threads keep eight 16-byte loads in flight, with plain loads (nontemporal == 0) or
 * with the non-temporal hint the weight-streaming kernels use, in GB/s.  What a memory-bound kernel can
 * reach lies below the published 8 TB/s; this is the reference the weight-streaming launches are held
 * against.  Runs one warm-up launch and `launches` >= 1 timed ones on `stream` and waits for them.
 * gb_per_s: host pointer.  Errors: MOE_ERR_INVALID_ARG, MOE_ERR_DEVICE. */
moe_status moe_measure_hbm_read_rate(const void* buf /* device */, size_t bytes, int32_t nontemporal,
                                     int32_t launches, float* gb_per_s /* host */, void* stream);

/* Device pointer (into the workspace) to an int32 that the most recent moe_grouped_ffn / moe_layer_forward /
 * moe_profile_ffn call on this context set to 1 if it refused its offsets (offsets[E_local] above the host's
 * row bound; nothing was computed) and to 0 otherwise. */
moe_status moe_ffn_refused_flag(moe_ctx* ctx, const int32_t** flag);

/* Device pointers into the workspace holding the intermediates of the most recent
 * moe_layer_forward: topk_idx [T,k], topk_w [T,k], offsets [E_local+1], row_of [T,k]. */
moe_status moe_layer_intermediates(moe_ctx* ctx, const int32_t** topk_idx, const float** topk_w,
                                   const int32_t** offsets, const int32_t** row_of);

#ifdef __cplusplus
}
#endif
#endif /* MOE_H_ */
