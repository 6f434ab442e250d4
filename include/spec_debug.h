/*
 * Parity hooks, measurement aids and single kernels of the speculative-decoding library (spec.h).
 *
 * Nothing here is needed to run speculative decoding: the spec_debug_* calls let a test read what a step left behind
 * or set up a state without a prefill, the spec_profile_* calls time one kernel class inside a run, and the spec_k_*
 * calls run one kernel of the step (Background section: draft decode, verification pass, accept / resample) on
 * caller buffers.  Same conventions as spec.h: 0 or a negative SPEC_E* code, device / host pointers as stated.
 */
#ifndef SPEC_DEBUG_H
#define SPEC_DEBUG_H

#include <stdint.h>

#include "spec.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Parity hooks.  which = 0: draft logits of the last spec_draft, rows [batch][gamma] (row-major,
 * `vocab` floats each); which = 1: target logits of the last spec_verify, rows [batch][gamma+1].
 * host_out has room for cap floats; *rows receives rows per sequence.  Synchronises. */
int spec_debug_logits(spec_ctx *ctx, int32_t which, float *host_out, int64_t cap, int32_t *rows);

/* Tokens drafted by the last spec_draft for sequence b (valid until spec_accept): host int32, capacity cap;
 * *n receives their number.  Synchronises. */
int spec_debug_drafted(spec_ctx *ctx, int32_t b, int32_t *host_out, int32_t cap, int32_t *n);

/* Continue a generation that was loaded with spec_prefill*: the next step gets ordinal `step`
 * (Philox counters) and sequence b counts its first prompt_lens[b] tokens as the prompt (forced
 * acceptance is indexed by tokens generated after the prompt).  Parity tests use it to restart
 * the library from a token sequence produced elsewhere. */
int spec_debug_set_step(spec_ctx *ctx, int32_t step, const int32_t *prompt_lens);

/* Copy the first `bytes` bytes of an internal buffer of the draft (model 0) or target (model 1) to host
 * memory, as left by the last forward pass: which = 0 residual stream, 1 rotated queries, 2 attention
 * output, 3 SwiGLU output, 4 normed-input copy, 5 sum-of-squares slots, 6/7/8 attention chunk partials
 * (max, sum, vectors), 9..12 the bf16 copies of attention output, normed input, SwiGLU output and queries,
 * 100 + l / 200 + l the K / V page pool of layer l.  The caller must know the sizes;
 * debugging aid only.  Synchronises. */
int spec_debug_read(spec_ctx *ctx, int32_t model, int32_t which, void *host_out, int64_t bytes);

/* Fill both KV caches with seeded values in [-1, 1) for positions 0..len-1 and set every sequence
 * length to len+1 with token 0 as the last token (verify-only sweeps).  Synchronises. */
int spec_debug_fill_kv(spec_ctx *ctx, int32_t len, uint64_t seed);

/* Overwrite positions pos0 .. pos0+n-1 of one sequence in the KV cache of one layer (model 0 = draft, 1 = target)
 * with caller data: k_host, v_host host fp32 [n][n_kv_heads][head_dim], rounded to the cache type.  Lets a parity
 * test give the library and its reference the same synthetic cache without a prefill.  Synchronises. */
int spec_debug_write_kv(spec_ctx *ctx, int32_t model, int32_t layer, int32_t seq, int32_t pos0, int32_t n,
                        const float *k_host, const float *v_host);

/* Replace the logical-to-physical KV page map of both models: host int32 [batch][max_seq/page_tokens],
 * a permutation of 0..batch*pages-1.  Must be called before spec_prefill. */
int spec_debug_set_block_table(spec_ctx *ctx, const int32_t *table);

/* Time kernel classes with HIP event pairs on the context's stream.  model: 0 draft, 1 target.
 * kind: 1 QKV projection, 2 output and down projection together, 3 gate/up projection with SwiGLU, 4 LM head,
 * 5 output projection, 6 down projection, 7 attention with the merge of its chunk partials; 0 times every class of
 * both models (model is then ignored); -1 switches timing off.  Projections are timed by the dispatch itself (kernel
 * start to kernel end), class 7 by events recorded on the stream around its two launches.  Only launches made outside
 * captured graphs (use_graphs = 0) are timed.  spec_profile_read_class() waits for the stream and returns the number
 * of timed launches of one (model, kind) and the sum of their durations in milliseconds since the last
 * spec_profile_read(), which returns the same over everything timed and clears the record. */
int spec_profile_kernel(spec_ctx *ctx, int32_t model, int32_t kind);
int spec_profile_read_class(spec_ctx *ctx, int32_t model, int32_t kind, int32_t *launches, double *total_ms);
int spec_profile_read(spec_ctx *ctx, int32_t *launches, double *total_ms);

/* One target verification pass of `rows` rows per sequence (1 <= rows <= gamma_max + 1: the last committed token and
 * the rows - 1 token slots behind it) on the current state, asynchronous, with no draft phase before it and no accept
 * after it: the verification-only sweeps over rows, cache length and batch (spec_debug_fill_kv sets up the cache).
 * The state machine stays where it was; the KV entries of those positions are overwritten.  Until the next
 * spec_draft, spec_debug_logits(which = 1) returns this pass's rows, [batch][rows]. */
int spec_debug_verify_rows(spec_ctx *ctx, int32_t rows);

/* ---- single kernels on caller buffers (parity tests and roofline measurement) ---------------- */

/* y[r][n] = sum_k x[r][k] * W[n][k].  W: device, row-major [N][K], dtype SPEC_F32 or SPEC_BF16
 * (for path SPEC_PATH_MFMA: the re-tiled copy produced by spec_k_retile, bf16 only, N % 16 == 0,
 * K % 32 == 0).  x: device fp32 [R][K] (the matrix-core path multiplies by its two-term bf16 split, about 16
 * significant bits); y: device fp32 [R][N]; 1 <= R <= 128.  Asynchronous on `stream`. */
int spec_k_gemv(const void *w, int32_t dtype, int32_t N, int32_t K, const float *x, int32_t R,
                float *y, int32_t path, void *stream);

/* The matrix-core kernel alone, asynchronous, no allocation: w_tiled from spec_k_retile, x_bf16 device bf16
 * [R][K], x_lo_bf16 an optional second bf16 term of x (same shape, same allocation as x_bf16; NULL: none; the
 * kernel multiplies by x_bf16 + x_lo_bf16), y device fp32 [R][N].  cfg = 0 picks the launch shape from (N, K, R); cfg = 100 * groups + waves forces
 * one of (1,16) (1,8) (1,4) (2,8) (2,4) (4,4) when groups * waves * ceil16(R)/16 <= 32 (kernel tuning). */
int spec_k_gemv_tiled(const void *w_tiled, int32_t N, int32_t K, const void *x_bf16, const void *x_lo_bf16, int32_t R,
                      float *y, int32_t cfg, void *stream);

/* The dense-contraction kernel alone (prompt ingestion, verification of large batches: many rows on the matrix
 * cores), asynchronous, no allocation: y[r][n] = sum_k x[r][k] * W[n][k] with w_tiled from spec_k_retile (N % 16 == 0,
 * K % 32 == 0), x device fp32 [R][K] (multiplied as its two-term bf16 split, about 16 significant bits), y device
 * fp32 [R][N], any R >= 1.  cfg = 0 picks the block shape and the split of K from (N, K, R); otherwise cfg = 1000 *
 * shares + shape with shape 808 / 408 / 404 / 304 / 204 / 104 (blocks of 256 x 256, 128 x 256, 128 x 128, 96 x 128, 64 x 128, 32 x 128 rows of x by rows of W; 0: automatic) and shares = 2..8
 * workgroups per block, each multiplying its share of K, followed by a summing pass (0: automatic).
 * workspace: device scratch for the shares' partial results, at least shares * R * N * 4 bytes (NULL: never split).
 * SPEC_EINVAL when the forced split does not fit (workspace too small, fewer k-tiles than shares). */
int spec_k_gemm_tiled(const void *w_tiled, int32_t N, int32_t K, const float *x, int32_t R, float *y, int32_t cfg,
                      void *workspace, int64_t workspace_bytes, void *stream);

/* 8-bit weights, W[n][k] = w_scale[n] * q[n][k] with q int8 in [-127, 127] (the quantised matrices of the paper's
 * largest pair stand behind this; here they are synthetic).  spec_k_retile_q8 re-tiles q [N][K] (device, row-major,
 * K % 64 == 0, N % 16 == 0) into 16-row groups of 1 KiB tiles of 16 rows x 64 k (N*K bytes).  The two kernels
 * below are spec_k_gemv_tiled / spec_k_gemm_tiled on such a matrix: the int8 values become bf16 in registers
 * (exactly), and the result is multiplied by w_scale (device, fp32 [N]). */
int spec_k_retile_q8(const void *w_q8, int32_t N, int32_t K, void *out, void *stream);
int spec_k_gemv_tiled_q8(const void *w_tiled, const float *w_scale, int32_t N, int32_t K, const void *x_bf16,
                         const void *x_lo_bf16, int32_t R, float *y, void *stream);
int spec_k_gemm_tiled_q8(const void *w_tiled, const float *w_scale, int32_t N, int32_t K, const float *x, int32_t R,
                         float *y, int32_t cfg, void *workspace, int64_t workspace_bytes, void *stream);

/* Re-tile a row-major bf16 matrix [N][K] into the streaming layout of the matrix-core kernel:
 * 16-row groups, each group a run of 1 KiB tiles (16 rows x 32 k) stored lane-major.  out: device,
 * N*K*2 bytes. */
int spec_k_retile(const void *w, int32_t N, int32_t K, void *out, void *stream);

/* dst[0..bytes) = src[0..bytes): a plain device-to-device copy kernel, 16 bytes per lane (bytes % 16 == 0, both
 * device, 16-byte aligned, not overlapping).  Measurement aid: the known traffic that scales profiler byte counters. */
int spec_k_copy(void *dst, const void *src, int64_t bytes, void *stream);

/* out[i] = Philox4x32-10(counter = ctr[i][0..3], key = seed); ctr, out: device uint32 [n][4]. */
int spec_k_philox(uint64_t seed, const uint32_t *ctr, int32_t n, uint32_t *out, void *stream);

/* Stand-alone accept / resample over caller logits (one sequence): p_logits device fp32 [k+1][vocab],
 * q_logits device fp32 [k][vocab], drafted device int32 [k]; result device int32 [2] = {A, y}.
 * Natural or greedy acceptance with the uniforms of step ordinal `step`, sequence 0. */
int spec_k_accept(const float *p_logits, const float *q_logits, const int32_t *drafted, int32_t k,
                  int32_t vocab, float temperature, uint64_t seed, int32_t step, int32_t *result,
                  void *stream);

/* For callers that cannot allocate device memory - code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc: spec_k_accept with its scratch (tile partials of the k + 1 target rows and k draft rows, row
 * statistics, step state: 256-byte blocks, about 2.1 MiB at the limits) in a fixed device array of the library
 * instead of a hipMalloc'ed block.  Same arguments and the same result as spec_k_accept; limits k <= 64 and
 * vocab <= 262144 (SPEC_EINVAL with a message in spec_last_error(NULL) beyond them).  Calls no hipMalloc / hipFree
 * and no routine that allocates; every step is a kernel launch on `stream` (no memset or copy nodes), and the call
 * does NOT synchronise: `result` is valid once the stream has passed the call's last kernel.  The array (one copy
 * per GPU, held until the process ends) is shared by every call on that GPU and keeps the last call's contents; the
 * call clears what it uses first.  Calls that overlap on one GPU (different streams, or several threads) race on
 * it: serialise them. */
int spec_k_accept_static(const float *p_logits, const float *q_logits, const int32_t *drafted, int32_t k,
                         int32_t vocab, float temperature, uint64_t seed, int32_t step, int32_t *result,
                         void *stream);

#ifdef __cplusplus
}
#endif
#endif
