/* Host-only driver for the sanitizer build (address + undefined behaviour) of the controller and of the argument
 * checks of the C ABI.  No GPU is touched: every spec_* call below must fail on its arguments before any device
 * work.  Mode "controller <golden file>": replays the hand-worked trajectories (GammaTune section, Algorithm 1) and a
 * few thousand random scripts with invalid inputs mixed in.  Mode "api": null pointers, bad shapes, bad sizes. */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "gammatune.h"
#ifdef WITH_API
#include "spec.h"
#include "spec_debug.h"
#endif

static int fails = 0;
#define CHECK(cond) do { if (!(cond)) { printf("FAILED line %d: %s\n", __LINE__, #cond); ++fails; } } while (0)

static int controller(const char *golden) {
    FILE *f = fopen(golden, "r");
    if (!f) { printf("cannot open %s\n", golden); return 2; }
    char line[4096];
    int n_lines = 0;
    while (fgets(line, sizeof line, f)) {
        if (line[0] == '#' || line[0] == '\n') continue;
        char *name = strtok(line, "|"), *eta_s = strtok(NULL, "|"), *script = strtok(NULL, "|"), *gam = strtok(NULL, "|"),
             *bars = strtok(NULL, "|");
        if (!name || !eta_s || !script || !gam) continue;
        gt_params p = {atof(eta_s), 1, 1, 8, GT_EXPAND_A};
        gt_state st;
        CHECK(gammatune_init(&st, &p, 4) == 0);
        int want[64], nw = 0, a[64], na = 0;
        double wb[64]; int nb = 0;
        char *save = NULL;
        for (char *t = strtok_r(script, " \n", &save); t && na < 64; t = strtok_r(NULL, " \n", &save)) a[na++] = strcmp(t, "inf") ? atoi(t) : 1 << 20;
        for (char *t = strtok_r(gam, " \n", &save); t && nw < 64; t = strtok_r(NULL, " \n", &save)) want[nw++] = atoi(t);
        if (bars) for (char *t = strtok_r(bars, " \n", &save); t && nb < 64; t = strtok_r(NULL, " \n", &save)) wb[nb++] = atof(t);
        CHECK(na == nw);
        for (int i = 0; i < na; ++i) {
            const int A = a[i] < st.gamma ? a[i] : st.gamma;
            const int g = gammatune_update(&st, A, st.gamma);
            CHECK(g == want[i]);
            if (i < nb) CHECK(st.gamma_bar == wb[i]);
        }
        ++n_lines;
    }
    fclose(f);
    CHECK(n_lines >= 4);
    /* random scripts, all readings, invalid calls in between (they must leave the state alone) */
    unsigned long long rng = 88172645463325252ULL;
    for (int rep = 0; rep < 3000; ++rep) {
        rng ^= rng << 13; rng ^= rng >> 7; rng ^= rng << 17;
        gt_params p = {(double)(rng % 17) / 16.0, (int)((rng >> 8) % 4), 1 + (int)((rng >> 16) % 3), 0, (int)((rng >> 24) % 3)};
        p.gamma_max = p.gamma_min + (int)((rng >> 32) % 20);
        gt_state st;
        CHECK(gammatune_init(&st, &p, (int)((rng >> 40) % 40) - 5) == 0);
        for (int i = 0; i < 40; ++i) {
            rng ^= rng << 13; rng ^= rng >> 7; rng ^= rng << 17;
            const gt_state before = st;
            CHECK(gammatune_update(&st, st.gamma + 1, st.gamma + 1) < 0);
            CHECK(gammatune_update(&st, -1, 0) < 0);
            CHECK(gammatune_update(&st, 1, 0) < 0 || st.gamma < 1);
            CHECK(memcmp(&before, &st, sizeof st) == 0);
            const int k = 1 + (int)(rng % (unsigned)st.gamma), A = (int)((rng >> 20) % (unsigned)(k + 1));
            const int g = gammatune_update(&st, A, k);
            CHECK(g >= p.gamma_min && g <= p.gamma_max && g == st.gamma);
            CHECK(st.gamma_bar >= p.gamma_min && st.gamma_bar <= p.gamma_max);
        }
    }
    gt_params bad = {1.5, 1, 1, 8, 0};
    gt_state st;
    CHECK(gammatune_init(&st, &bad, 4) < 0);
    CHECK(gammatune_init(NULL, &bad, 4) < 0);
    CHECK(gammatune_update(NULL, 0, 0) < 0);
    return fails ? 1 : 0;
}

#ifdef WITH_API
static int api(void) {
    spec_ctx *ctx = (spec_ctx *)0x1;
    CHECK(spec_init(NULL, NULL, NULL, NULL, NULL, &ctx) == SPEC_EINVAL && ctx == NULL);
    CHECK(spec_init(NULL, NULL, NULL, NULL, NULL, NULL) == SPEC_EINVAL);
    CHECK(spec_prefill(NULL, NULL, 1) == SPEC_EINVAL);
    int32_t lens[1] = {1}, toks[1] = {0};
    CHECK(spec_prefill_ragged(NULL, toks, 1, lens) == SPEC_EINVAL);
    CHECK(spec_draft(NULL, 1) == SPEC_EINVAL);
    CHECK(spec_draft_batch(NULL, lens) == SPEC_EINVAL);
    CHECK(spec_verify(NULL, 1) == SPEC_EINVAL);
    CHECK(spec_accept(NULL, NULL, NULL, NULL) == SPEC_EINVAL);
    CHECK(spec_generate(NULL, NULL, 1, 1, NULL) == SPEC_EINVAL);
    float alpha = 0.5f;
    CHECK(spec_set_forced_alpha(NULL, &alpha, 1) == SPEC_EINVAL);
    CHECK(spec_set_early_stop(NULL, 0.4f) == SPEC_EINVAL);
    int32_t n = 0;
    CHECK(spec_read_tokens(NULL, 0, toks, 1, &n) == SPEC_EINVAL);
    CHECK(spec_debug_verify_rows(NULL, 1) == SPEC_EINVAL);
    CHECK(spec_profile_kernel(NULL, 0, 1) == SPEC_EINVAL);
    double ms = 0;
    CHECK(spec_profile_read(NULL, &n, &ms) == SPEC_EINVAL);
    CHECK(spec_profile_read_class(NULL, 0, 1, &n, &ms) == SPEC_EINVAL);
    CHECK(spec_device_bytes(NULL) == 0);
    spec_destroy(NULL);
    CHECK(strcmp(spec_strerror(SPEC_OK), "ok") == 0);
    CHECK(strlen(spec_strerror(-12345)) > 0);
    CHECK(spec_last_error(NULL) != NULL);
    /* single kernels: null pointers and sizes outside their documented ranges */
    float y[4];
    CHECK(spec_k_gemv(NULL, SPEC_BF16, 16, 32, y, 1, y, SPEC_PATH_MFMA, NULL) == SPEC_EINVAL);
    CHECK(spec_k_gemv(y, 7, 16, 32, y, 1, y, SPEC_PATH_WAVEDOT, NULL) == SPEC_EINVAL);
    CHECK(spec_k_gemv(y, SPEC_BF16, 16, 33, y, 1, y, SPEC_PATH_WAVEDOT, NULL) == SPEC_EINVAL);
    CHECK(spec_k_gemv(y, SPEC_BF16, 16, 32, y, 129, y, SPEC_PATH_WAVEDOT, NULL) == SPEC_EINVAL);
    CHECK(spec_k_gemv_tiled(y, 15, 32, y, NULL, 1, y, 0, NULL) == SPEC_EINVAL);
    CHECK(spec_k_gemv_tiled(y, 16, 32, y, NULL, 1, y, 316, NULL) == SPEC_EINVAL);
    CHECK(spec_k_gemm_tiled(y, 16, 32, y, 0, y, 0, NULL, 0, NULL) == SPEC_EINVAL);
    CHECK(spec_k_gemm_tiled(y, 16, 32, y, 4, y, 777, NULL, 0, NULL) == SPEC_EINVAL);
    CHECK(spec_k_retile(y, 16, 31, y, NULL) == SPEC_EINVAL);
    CHECK(spec_k_retile_q8(y, 16, 32, y, NULL) == SPEC_EINVAL);
    CHECK(spec_k_copy(y, y, 15, NULL) == SPEC_EINVAL);
    CHECK(spec_k_philox(0, NULL, 1, NULL, NULL) == SPEC_EINVAL);
    int32_t res[2];
    CHECK(spec_k_accept(y, y, toks, 0, 100, 1.0f, 0, 0, res, NULL) == SPEC_EINVAL);
    CHECK(spec_k_accept(y, y, toks, 65, 100, 1.0f, 0, 0, res, NULL) == SPEC_EINVAL);
    CHECK(spec_k_accept_static(y, y, toks, 65, 100, 1.0f, 0, 0, res, NULL) == SPEC_EINVAL);
    CHECK(spec_k_accept_static(y, y, toks, 2, 262145, 1.0f, 0, 0, res, NULL) == SPEC_EINVAL);
    CHECK(spec_k_accept_static(y, y, toks, 2, 100, -1.0f, 0, 0, res, NULL) == SPEC_EINVAL);
    return fails ? 1 : 0;
}
#endif

int main(int argc, char **argv) {
    if (argc >= 3 && strcmp(argv[1], "controller") == 0) return controller(argv[2]);
#ifdef WITH_API
    if (argc >= 2 && strcmp(argv[1], "api") == 0) return api();
#endif
    printf("usage: driver controller <golden file> | api\n");
    return 2;
}
