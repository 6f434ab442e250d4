/*
 * Speculative-decoding step engine for one MI355X (gfx950).
 *
 * One speculative step (Background section): the draft model proposes gamma
 * tokens autoregressively (spec_draft), the target model scores all of them in
 * one pass over its weights against its KV cache (spec_verify), and the
 * accept / resample rule emits the accepted prefix plus one target-distributed
 * token (spec_accept).  The next gamma comes from gammatune_update()
 * (gammatune.h; GammaTune section, Algorithm 1).  GammaTune+ (confidence-guided
 * early stopping) is switched on with spec_set_early_stop().
 *
 * General rules
 *  - Every function returns 0 (SPEC_OK) or a negative SPEC_E* code; nothing
 *    throws or aborts across this boundary.  spec_strerror() names a code;
 *    spec_last_error() gives the text of the last failure of a context.
 *  - "device" pointers are HIP device addresses on the current device, "host"
 *    pointers ordinary host memory.  The library never frees caller memory.
 *  - Weights are BORROWED: the caller keeps them alive and unchanged until
 *    spec_destroy().  The library only reads them (and may keep a re-tiled
 *    device copy of its own).
 *  - All work is enqueued on the stream given at init; only spec_accept(),
 *    spec_prefill(), spec_read_tokens() and the spec_debug_* calls synchronise.
 *  - One context per host thread; calls on one context must not overlap.
 *  - Models are Llama-style decoders: RMSNorm, rotary embedding with
 *    rotate-half pairing (element j pairs with j + head_dim/2, angle
 *    pos * theta^(-2j/head_dim)), grouped-query attention (query head h reads
 *    kv head h / (n_q_heads / n_kv_heads)), SwiGLU MLP, no biases.
 */
#ifndef SPEC_H
#define SPEC_H

#include <stdint.h>

#include "gammatune.h"

#ifdef __cplusplus
extern "C" {
#endif

enum {
    SPEC_OK       = 0,
    SPEC_EINVAL   = -1,  /* null pointer, bad shape, gamma out of range, buffer too small */
    SPEC_ESTATE   = -2,  /* call order violated (prefill -> draft -> verify -> accept -> draft ...) */
    SPEC_ENOMEM   = -3,  /* device or host allocation failed */
    SPEC_EHIP     = -4,  /* a HIP runtime call failed; see spec_last_error() */
    SPEC_ECAP     = -5,  /* the step would exceed max_seq */
    SPEC_ENOTIMPL = -6
};

enum { SPEC_F32 = 0, SPEC_BF16 = 1, SPEC_Q8 = 2 };
enum { SPEC_ACCEPT_NATURAL = 0, SPEC_ACCEPT_FORCED = 1 };
enum { SPEC_PATH_AUTO = 0, SPEC_PATH_WAVEDOT = 1, SPEC_PATH_MFMA = 2 };

typedef struct spec_ctx spec_ctx; /* opaque */

typedef struct {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
    int32_t dtype;      /* SPEC_F32 or SPEC_BF16: storage type of every weight and of the KV cache.  SPEC_Q8: the seven
                           projection matrices of every layer and the LM head are int8 with one fp32 scale per output
                           row (W[n][k] = scale[n] * q[n][k], |q| <= 127); embedding, norm weights and the KV cache
                           are bf16.  Needs d_model, n_q_heads * head_dim and d_ffn multiples of 64, vocab of 16. */
    float   rope_theta; /* rotary base */
    float   rms_eps;
} spec_shape;

/* Device pointers.  Matrices are row-major [n_out][n_in] with n_in contiguous,
 * element type per spec_shape.dtype, each row 16-byte aligned.  The per-layer
 * members are HOST arrays of n_layers device pointers. */
typedef struct {
    const void *tok_embed;                           /* [vocab][d_model] */
    const void *const *wq;                           /* [n_q_heads*head_dim][d_model] */
    const void *const *wk, *const *wv;               /* [n_kv_heads*head_dim][d_model] */
    const void *const *wo;                           /* [d_model][n_q_heads*head_dim] */
    const void *const *w_gate, *const *w_up;         /* [d_ffn][d_model] */
    const void *const *w_down;                       /* [d_model][d_ffn] */
    const void *const *attn_norm, *const *ffn_norm;  /* [d_model] */
    const void *final_norm;                          /* [d_model] */
    const void *lm_head;                             /* [vocab][d_model]; may alias tok_embed (not with SPEC_Q8) */
    /* SPEC_Q8 only (ignored otherwise): fp32 scales, one per output row of the matrix of the same name */
    const void *const *wq_scale, *const *wk_scale, *const *wv_scale, *const *wo_scale;
    const void *const *w_gate_scale, *const *w_up_scale, *const *w_down_scale;
    const void *lm_head_scale;
} spec_weights;

typedef struct {
    int32_t  batch;        /* sequences decoded in lock-step, 1..64; batch * (gamma_max + 1) rows make one verification
                              pass: at most 128, or 1024 when the target is a bf16 model on the matrix-core kernels */
    int32_t  max_seq;      /* capacity in tokens per sequence (prompt + generated + gamma_max + 1) */
    int32_t  page_tokens;  /* tokens per KV page, a power of two >= 8; 0 -> 64 */
    int32_t  gamma_max;    /* largest gamma ever passed to spec_draft, 1..64 */
    float    temperature;  /* 0 -> greedy; same temperature for draft and target */
    uint64_t seed;         /* Philox key */
    int32_t  accept_mode;  /* SPEC_ACCEPT_NATURAL or SPEC_ACCEPT_FORCED */
    int32_t  gemv_path;    /* SPEC_PATH_AUTO, or force one kernel family (bf16 models; fp32 models always use WAVEDOT) */
    int32_t  use_graphs;   /* 1: replay one captured HIP graph per gamma; 0: launch kernel by kernel */
    int32_t  attn_chunk;   /* KV positions per attention workgroup (bf16 models): 0 = automatic, else 64, 128, 256 or 512 */
    void    *hip_stream;   /* hipStream_t to enqueue on (borrowed); NULL = a stream the context creates and owns */
} spec_config;

/* Create a context: validates shapes (both models must share `vocab`), allocates the
 * paged KV caches, activations and logits buffers, re-tiles bf16 and 8-bit weights for the
 * matrix-core kernels, builds the rotary tables.  On failure *out is NULL. */
int spec_init(const spec_shape *target, const spec_weights *target_w,
              const spec_shape *draft, const spec_weights *draft_w,
              const spec_config *cfg, spec_ctx **out);

/* Load the prompts: host_tokens is host int32 [batch][n], n >= 1, every id in
 * [0, vocab).  Both models ingest tokens 0..n-2 into their KV caches (the last
 * prompt token is fed by the first step), up to 1024 rows per launch for a model on the
 * matrix-core kernels (32 rows per sequence otherwise); the draft model ingests on a second
 * stream of the library's own beside the target (environment variable SPEC_PREFILL_ONE_STREAM:
 * both on the context's stream, for kernel traces).  Resets step counter, lengths and
 * generated count; may be called again to start a new generation.  Synchronises. */
int spec_prefill(spec_ctx *ctx, const int32_t *host_tokens, int32_t n);

/* Same for prompts of different lengths: host_tokens is host int32 [batch][n_max], sequence b uses its
 * first lens[b] entries (1 <= lens[b] <= n_max). */
int spec_prefill_ragged(spec_ctx *ctx, const int32_t *host_tokens, int32_t n_max, const int32_t *lens);

/* Draft phase of one step, asynchronous.  Runs gamma draft-model decode steps; step i
 * draws x_i from softmax(draft logits / T) by index-order inverse CDF with the uniform
 * Philox(seed; counter = (step, i, DRAFT, b)) (argmax if T == 0), appends it to the
 * sequence, and keeps the draft logits row for the accept phase.  With early stopping
 * enabled drafting of a sequence ends after the first x_i whose confidence is below tau;
 * that x_i is kept; the call then launches pass by pass and waits for each pass's verdict (a few words
 * in pinned memory) before it launches the next, so it returns when the last pass has been enqueued.  1 <= gamma <= gamma_max.  SPEC_ECAP if len + gamma + 1 > max_seq. */
int spec_draft(spec_ctx *ctx, int32_t gamma);

/* Same with one planned gamma per sequence (host int32 [batch]); the launch uses the
 * largest, a sequence stops drafting at its own gamma. */
int spec_draft_batch(spec_ctx *ctx, const int32_t *gammas);

/* Verify phase, asynchronous: one target forward over the gamma+1 rows
 * [last token, x_1 .. x_gamma] of every sequence, causal inside the rows, against the
 * target KV cache; produces the logits rows p_1 .. p_{gamma+1}.  `gamma` must equal the
 * (largest) gamma of the preceding spec_draft call.  After spec_draft_batch with differing
 * gammas a bf16 / 8-bit target on the matrix-core kernels runs only the gamma_b + 1 rows each
 * sequence planned (spec_debug_logits still returns the padded [batch][gamma + 1] layout). */
int spec_verify(spec_ctx *ctx, int32_t gamma);

/* Accept phase: runs the fused accept / resample kernels, waits for the stream, and
 * returns per sequence (host int32 [batch] each, any may be NULL):
 *   n_accepted  A  = number of leading drafted tokens accepted
 *                    natural: u * q_i(x_i) < p_i(x_i), u = Philox(step, i, ACCEPT, b)
 *                    greedy (T == 0): x_i == argmax p_i
 *                    forced: Philox(g, 0, FORCED, b) < alpha[g], g = index of the generated token
 *   next_token  y  = A < drafted: draw from norm(max(0, p_{A+1} - q_{A+1})) with u(step, A+1, RESID, b)
 *                    A == drafted: draw from p_{drafted+1} with u(step, drafted+1, BONUS, b)
 *                    (argmax of the same row if T == 0)
 *   n_drafted   k  = tokens actually drafted (< gamma only with early stopping or a smaller per-sequence gamma)
 * The sequence grows by x_1..x_A, y; the step counter advances. */
int spec_accept(spec_ctx *ctx, int32_t *n_accepted, int32_t *next_token, int32_t *n_drafted);

/* Forced acceptance landscape: alpha is host float [n], alpha[g] in [0,1] for generated index g
 * (the last value repeats beyond n).  Only used with SPEC_ACCEPT_FORCED.  In forced mode the
 * confidence seen by early stopping is the synthetic clamp(alpha[g] + (0.5 - Philox(g, 0, FORCED, b)) / 2, 0, 1). */
int spec_set_forced_alpha(spec_ctx *ctx, const float *alpha, int32_t n);

/* GammaTune+ threshold: stop drafting when the draft's top probability
 * max softmax(logits / T_eff), T_eff = T > 0 ? T : 1, is below tau.  tau <= 0 disables. */
int spec_set_early_stop(spec_ctx *ctx, float tau);

/* Totals of a spec_generate() call over all sequences and steps. */
typedef struct {
    int64_t steps;      /* speculative steps (draft + verify + accept) */
    int64_t generated;  /* tokens emitted, counted up to n_generate per sequence */
    int64_t accepted;   /* accepted draft tokens */
    int64_t drafted;    /* drafted tokens */
    int64_t gamma_sum;  /* planned gammas, one per (sequence, step) */
} spec_gen_stats;

/* The decode loop in native code: speculative steps until every sequence has n_generate tokens more than when the
 * call began.  controllers: host array of `batch` GammaTune states, updated in place with gammatune_update(A, k)
 * after every step, or NULL for the fixed speculation length fixed_gamma.  Must follow spec_prefill() or
 * spec_accept().  Equivalent to calling spec_draft_batch / spec_verify / spec_accept / gammatune_update from the
 * host in a loop; stats may be NULL.  SPEC_ECAP when a step would exceed max_seq. */
int spec_generate(spec_ctx *ctx, gt_state *controllers, int32_t fixed_gamma, int32_t n_generate, spec_gen_stats *stats);

/* Copy the tokens of sequence b (prompt + generated so far) to host_out (host int32, capacity cap);
 * *n receives the length.  Synchronises. */
int spec_read_tokens(spec_ctx *ctx, int32_t b, int32_t *host_out, int32_t cap, int32_t *n);

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

/* Time one kernel class with HIP event pairs on the context's stream.  model: 0 draft, 1 target.
 * kind: 1 QKV projection, 2 output/down projection with residual, 3 gate/up projection with SwiGLU,
 * 4 LM head; -1 switches timing off.  Only launches made outside captured graphs (use_graphs = 0)
 * are timed.  spec_profile_read() waits for the stream, returns the number of timed launches and the
 * sum of their durations in milliseconds since the last read, and clears the record. */
int spec_profile_kernel(spec_ctx *ctx, int32_t model, int32_t kind);
int spec_profile_read(spec_ctx *ctx, int32_t *launches, double *total_ms);

/* Device bytes the context allocated (KV pages, activations, logits, re-tiled weights). */
int64_t spec_device_bytes(const spec_ctx *ctx);

void spec_destroy(spec_ctx *ctx);
const char *spec_strerror(int code);
const char *spec_last_error(const spec_ctx *ctx);

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

#ifdef __cplusplus
}
#endif
#endif
