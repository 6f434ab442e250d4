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

/* Set-up of the models of a speculative step (Background section: a draft model M_q and a target model M_p).
 * Create a context: validates shapes (both models must share `vocab`), allocates the
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

/* Draft phase of one step (Background section: the draft model proposes gamma tokens autoregressively; GammaTune+
 * paragraph: drafting stops early below the confidence threshold), asynchronous.  Runs gamma draft-model decode steps; step i
 * draws x_i from softmax(draft logits / T) by index-order inverse CDF with the uniform
 * Philox(seed; counter = (step, i, DRAFT, b)) (argmax if T == 0), appends it to the
 * sequence, and keeps the draft logits row for the accept phase.  With early stopping
 * enabled drafting of a sequence ends after the first x_i whose confidence is below tau;
 * that x_i is kept; the call then launches pass by pass and waits for each pass's outcome (a few words
 * in pinned memory) before it launches the next, so it returns when the last pass has been enqueued.  1 <= gamma <= gamma_max.  SPEC_ECAP if len + gamma + 1 > max_seq. */
int spec_draft(spec_ctx *ctx, int32_t gamma);

/* Same with one planned gamma per sequence (host int32 [batch]); the launch uses the
 * largest, a sequence stops drafting at its own gamma. */
int spec_draft_batch(spec_ctx *ctx, const int32_t *gammas);

/* Verify phase (Background section: the target model scores the gamma proposals in one parallel pass), asynchronous: one target forward over the gamma+1 rows
 * [last token, x_1 .. x_gamma] of every sequence, causal inside the rows, against the
 * target KV cache; produces the logits rows p_1 .. p_{gamma+1}.  `gamma` must equal the
 * (largest) gamma of the preceding spec_draft call.  After spec_draft_batch with differing
 * gammas a bf16 / 8-bit target on the matrix-core kernels runs only the gamma_b + 1 rows each
 * sequence planned (spec_debug_logits still returns the padded [batch][gamma + 1] layout). */
int spec_verify(spec_ctx *ctx, int32_t gamma);

/* Accept phase (Background section; rule of the speculative-sampling works cited there): runs the fused accept / resample kernels, waits for the stream, and
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
    int64_t seq_steps;  /* (sequence, step) pairs counted above: a sequence that has reached n_generate is not counted */
} spec_gen_stats;

/* The decode loop of Algorithm 1's setting in native code: speculative steps until every sequence has n_generate tokens more than when the
 * call began.  controllers: host array of `batch` GammaTune states, updated in place with gammatune_update(A, k)
 * after every step, or NULL for the fixed speculation length fixed_gamma.  Must follow spec_prefill() or
 * spec_accept().  Equivalent to calling spec_draft_batch / spec_verify / spec_accept / gammatune_update from the
 * host in a loop; stats may be NULL.  A sequence that already has its n_generate tokens rides along with gamma = 1
 * until the slowest one is done (at most two more tokens per step: max_seq >= prompt + 3 * n_generate + gamma_max + 1
 * is always enough), its controller is no longer updated and it is left out of stats.  SPEC_ECAP when a step would
 * exceed max_seq. */
int spec_generate(spec_ctx *ctx, gt_state *controllers, int32_t fixed_gamma, int32_t n_generate, spec_gen_stats *stats);

/* Copy the tokens of sequence b (prompt + generated so far) to host_out (host int32, capacity cap);
 * *n receives the length.  Synchronises. */
int spec_read_tokens(spec_ctx *ctx, int32_t b, int32_t *host_out, int32_t cap, int32_t *n);

/* Device bytes the context allocated (KV pages, activations, logits, re-tiled weights). */
int64_t spec_device_bytes(const spec_ctx *ctx);

void spec_destroy(spec_ctx *ctx);
const char *spec_strerror(int code);
const char *spec_last_error(const spec_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif
