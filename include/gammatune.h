/*
 * GammaTune speculation-length controller (host side, no GPU dependency).
 *
 * Implements the update of the GammaTune section: the adaptive-expansion rule
 * (offset delta when every drafted token was accepted), the clamped
 * exponentially weighted moving average of the accepted count ("adaptive
 * window estimation"), and gamma <- ceil(gamma_bar) (Algorithm 1).
 *
 * A is the number of ACCEPTED DRAFT tokens of the step just finished
 * (0 <= A <= gamma); the bonus / resampled token is not counted.
 *
 * Algorithm 1 as printed assigns gamma <- A + delta and then unconditionally
 * overwrites gamma <- ceil(gamma_bar), which makes the expansion branch dead
 * and the window unable to grow.  `reading` selects how that is resolved:
 *   GT_EXPAND_A   (0, default) the offset is added to the observation:
 *                 A_eff = (A == gamma) ? A + delta : A, EMA on A_eff
 *   GT_LITERAL    (1) exactly as printed: EMA on raw A
 *   GT_SHORT_TERM (2) EMA on raw A; after a fully accepted step the returned
 *                 gamma is min(gamma_max, gamma + delta), else ceil(gamma_bar)
 *
 * Arithmetic: IEEE double, the EMA is evaluated exactly as
 *   (1.0 - eta) * gamma_bar + eta * (double)A_eff
 * without fused multiply-add, then clamped to [gamma_min, gamma_max], then
 * ceil().  The integer result is therefore reproducible bit for bit.
 *
 * GammaTune+ (confidence-guided early stopping) leaves the update unchanged:
 * pass drafted < gamma for a step that stopped early; "A == gamma" compares
 * with the planned gamma held in the state, so such a step never expands.
 */
#ifndef GAMMATUNE_H
#define GAMMATUNE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { GT_EXPAND_A = 0, GT_LITERAL = 1, GT_SHORT_TERM = 2 };

typedef struct {
    double  eta;        /* EMA weight in [0, 1] */
    int32_t delta;      /* expansion offset, >= 0 */
    int32_t gamma_min;  /* >= 1 */
    int32_t gamma_max;  /* >= gamma_min */
    int32_t reading;    /* GT_EXPAND_A / GT_LITERAL / GT_SHORT_TERM */
} gt_params;

/* Caller-owned plain data; copy it to checkpoint the controller. */
typedef struct {
    double    gamma_bar;
    int32_t   gamma;
    gt_params p;
} gt_state;

/* Initialise `st` (host memory) with gamma = gamma_bar = clamp(gamma0).
 * Returns 0, or -1 (SPEC_EINVAL) on a null pointer or parameters outside the
 * ranges above; `st` is untouched on error. */
int gammatune_init(gt_state *st, const gt_params *p, int32_t gamma0);

/* Consume one step: `accepted` = A, `drafted` = number of tokens actually
 * drafted (pass gamma when no early stop; only checked, accepted <= drafted <=
 * gamma).  Returns the next gamma (>= 1) and stores it in st->gamma, or a
 * negative value on invalid input (state untouched). */
int32_t gammatune_update(gt_state *st, int32_t accepted, int32_t drafted);

#ifdef __cplusplus
}
#endif
#endif
