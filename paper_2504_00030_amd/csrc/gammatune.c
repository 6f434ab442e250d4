/* GammaTune controller: GammaTune section, eq. adaptive expansion, eq. adaptive
 * window estimation, Algorithm 1.  See include/gammatune.h for the readings.
 * Build with -ffp-contract=off so the EMA is not fused. */
#include "gammatune.h"

#include <math.h>
#include <stddef.h>

int gammatune_init(gt_state *st, const gt_params *p, int32_t gamma0)
{
    if (st == NULL || p == NULL) return -1;
    if (!(p->eta >= 0.0 && p->eta <= 1.0)) return -1;
    if (p->delta < 0 || p->gamma_min < 1 || p->gamma_max < p->gamma_min) return -1;
    if (p->reading != GT_EXPAND_A && p->reading != GT_LITERAL && p->reading != GT_SHORT_TERM) return -1;
    int32_t g = gamma0;
    if (g < p->gamma_min) g = p->gamma_min;
    if (g > p->gamma_max) g = p->gamma_max;
    st->p = *p;
    st->gamma = g;
    st->gamma_bar = (double)g;
    return 0;
}

int32_t gammatune_update(gt_state *st, int32_t accepted, int32_t drafted)
{
    if (st == NULL) return -1;
    if (accepted < 0 || accepted > st->gamma) return -1;
    if (drafted < accepted || drafted > st->gamma) return -1;
    const gt_params *p = &st->p;
    const int full = (accepted == st->gamma);
    int32_t a_eff = accepted;
    if (full && p->reading == GT_EXPAND_A) a_eff = accepted + p->delta;
    volatile double keep = (1.0 - p->eta) * st->gamma_bar;   /* two rounded products, one rounded sum */
    volatile double add = p->eta * (double)a_eff;
    double ema = keep + add;
    if (ema < (double)p->gamma_min) ema = (double)p->gamma_min;
    if (ema > (double)p->gamma_max) ema = (double)p->gamma_max;
    st->gamma_bar = ema;
    int32_t next = (int32_t)ceil(ema);
    if (p->reading == GT_SHORT_TERM && full) {
        next = st->gamma + p->delta;
        if (next > p->gamma_max) next = p->gamma_max;
    }
    st->gamma = next;
    return next;
}
