/*
 * Driver for an AddressSanitizer / UndefinedBehaviorSanitizer build of the float64 CPU oracle
 * (tests/test_oracle_sanitizer.py compiles oracle/esrnn_oracle.c together with this file and runs it).
 * It calls every entry point of the oracle on small batches that exercise its index arithmetic: ragged
 * lengths down to the minimum, periods longer than a series' usable range, two seasonalities, no
 * seasonality, dilations beyond the number of window positions, three blocks, a category block, the
 * cell-state penalty and named sides at the kink of the loss.  Inputs come from a linear congruential
 * generator; nothing of the method is computed here.  Exit code 0 = the sanitizers saw nothing and every
 * result is finite.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../oracle/esrnn_oracle.h"

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static double uniform01(void)
{
    rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
    return (double)(rng_state >> 11) / 9007199254740992.0;
}

static int all_finite(const double *a, int64_t n)
{
    for (int64_t i = 0; i < n; ++i)
        if (!isfinite(a[i])) return 0;
    return 1;
}

static int run_case(eso_config cfg, int ragged, int use_sides, const char *what)
{
    const int B = cfg.B, T = cfg.T, I = cfg.I, H = cfg.H, h = cfg.hidden;
    int32_t *cat = NULL;
    if (cfg.n_cat > 0) {
        cat = (int32_t *)malloc(sizeof(int32_t) * B);
        for (int b = 0; b < B; ++b) cat[b] = (int32_t)(uniform01() * cfg.n_cat) % cfg.n_cat;
        cfg.categories = cat;
    }
    const int K = eso_es_param_rows(&cfg), L = eso_num_layers(&cfg);
    const int64_t nw = eso_weight_count(&cfg);
    if (K < 0 || L < 0 || nw < 0) { fprintf(stderr, "%s: configuration refused\n", what); return 1; }
    const int P = T - I - H + 1, Iw = I + cfg.n_cat;
    int32_t *len = (int32_t *)malloc(sizeof(int32_t) * B);
    for (int b = 0; b < B; ++b) len[b] = ragged ? I + H + (int32_t)(uniform01() * (T - I - H + 1)) : T;
    len[0] = T;
    if (ragged && B > 1) len[B - 1] = I + H;
    double *y = (double *)malloc(sizeof(double) * T * B);
    for (int64_t i = 0; i < (int64_t)T * B; ++i) y[i] = 50.0 + 100.0 * uniform01();
    double *es = (double *)malloc(sizeof(double) * K * B);
    for (int64_t i = 0; i < (int64_t)K * B; ++i)
        es[i] = cfg.param_space ? (uniform01() - 0.5) : 0.2 + 0.6 * uniform01() + (i >= (int64_t)(1 + cfg.n_seas) * B ? 0.5 : 0.0);
    double *w = (double *)malloc(sizeof(double) * nw);
    for (int64_t i = 0; i < nw; ++i) w[i] = (uniform01() - 0.5) * 0.6;

    eso_tape tp;
    memset(&tp, 0, sizeof(tp));
    tp.alpha = (double *)calloc(B, sizeof(double));
    tp.gamma1 = (double *)calloc(B, sizeof(double));
    tp.gamma2 = (double *)calloc(B, sizeof(double));
    tp.l = (double *)calloc((size_t)B * T, sizeof(double));
    tp.S1 = (double *)calloc((size_t)B * T, sizeof(double));
    tp.S2 = (double *)calloc((size_t)B * T, sizeof(double));
    tp.u = (double *)calloc((size_t)B * T, sizeof(double));
    tp.v = (double *)calloc((size_t)B * T, sizeof(double));
    tp.X = (double *)calloc((size_t)B * P * Iw, sizeof(double));
    tp.Z = (double *)calloc((size_t)B * P * H, sizeof(double));
    tp.gates = (double *)calloc((size_t)L * B * P * 4 * h, sizeof(double));
    tp.c = (double *)calloc((size_t)L * B * P * h, sizeof(double));
    tp.h = (double *)calloc((size_t)L * B * P * h, sizeof(double));
    tp.blk = (double *)calloc((size_t)cfg.n_blocks * B * P * h, sizeof(double));
    tp.a = (double *)calloc((size_t)B * P * h, sizeof(double));
    tp.o = (double *)calloc((size_t)B * P * H, sizeof(double));
    double loss = 0.0;
    double *fc = (double *)calloc((size_t)P * B * H, sizeof(double));
    int bad = 0;
    int rc = eso_forward(&cfg, y, len, es, w, &tp, &loss, fc);
    if (rc || !isfinite(loss) || !all_finite(fc, (int64_t)P * B * H)) { fprintf(stderr, "%s: forward rc %d loss %g\n", what, rc, loss); bad = 1; }

    int8_t *side = NULL;
    if (use_sides) {
        side = (int8_t *)calloc((size_t)B * P * H, 1);
        for (int64_t i = 0; i < (int64_t)B * P * H; i += 7) side[i] = (i & 1) ? 1 : -1;
        cfg.pin_side = side;
    }
    eso_adjoint adj;
    adj.gO = (double *)calloc((size_t)B * P * H, sizeof(double));
    adj.gR = (double *)calloc((size_t)B * P * h, sizeof(double));
    adj.gX = (double *)calloc((size_t)B * P * Iw, sizeof(double));
    adj.gu = (double *)calloc((size_t)B * T, sizeof(double));
    adj.gv = (double *)calloc((size_t)B * T, sizeof(double));
    double *ges = (double *)calloc((size_t)K * B, sizeof(double));
    double *gw = (double *)calloc((size_t)nw, sizeof(double));
    rc = eso_backward(&cfg, y, len, es, w, &tp, &adj, ges, gw);
    if (rc || !all_finite(ges, (int64_t)K * B) || !all_finite(gw, nw)) { fprintf(stderr, "%s: backward rc %d\n", what, rc); bad = 1; }
    rc = eso_backward(&cfg, y, len, es, w, &tp, NULL, ges, gw);
    if (rc) { fprintf(stderr, "%s: backward without adjoints rc %d\n", what, rc); bad = 1; }

    /* out-of-sample forecasts from lengths that leave no room for targets */
    for (int b = 0; b < B; ++b) len[b] = (b & 1) ? T : (I > 1 ? I + (T - I) / 2 : T);
    double *pf = (double *)calloc((size_t)B * H, sizeof(double));
    rc = eso_predict(&cfg, y, len, es, w, pf);
    if (rc || !all_finite(pf, (int64_t)B * H)) { fprintf(stderr, "%s: predict rc %d\n", what, rc); bad = 1; }

    free(pf); free(gw); free(ges); free(adj.gv); free(adj.gu); free(adj.gX); free(adj.gR); free(adj.gO); free(side);
    free(fc); free(tp.o); free(tp.a); free(tp.blk); free(tp.h); free(tp.c); free(tp.gates); free(tp.Z); free(tp.X);
    free(tp.v); free(tp.u); free(tp.S2); free(tp.S1); free(tp.l); free(tp.gamma2); free(tp.gamma1); free(tp.alpha);
    free(w); free(es); free(y); free(len); free(cat);
    printf("%-28s %s (loss %.6f)\n", what, bad ? "FAILED" : "ok", loss);
    return bad;
}

static eso_config base(void)
{
    eso_config c;
    memset(&c, 0, sizeof(c));
    c.B = 5; c.T = 30; c.n_seas = 1; c.m1 = 4; c.I = 3; c.H = 4; c.hidden = 5;
    c.n_blocks = 2; c.layers_in_block[0] = 2; c.layers_in_block[1] = 2;
    c.dilation[0][0] = 1; c.dilation[0][1] = 2; c.dilation[1][0] = 3; c.dilation[1][1] = 5;
    c.tau = 0.48; c.lambda_lv = 50.0;
    return c;
}

int main(void)
{
    int bad = 0;
    eso_config c = base();
    bad |= run_case(c, 0, 0, "single, full length");
    bad |= run_case(c, 1, 1, "single, ragged, sides");
    c.param_space = 1;
    bad |= run_case(c, 1, 0, "single, logit space");
    c = base(); c.n_seas = 0; c.m1 = 0;
    bad |= run_case(c, 1, 0, "level only");
    c = base(); c.n_seas = 2; c.m1 = 3; c.m2 = 7; c.T = 36;
    bad |= run_case(c, 1, 0, "two seasonalities");
    c = base(); c.m1 = 24; c.T = 40;                    /* period above the shortest series' range */
    bad |= run_case(c, 1, 0, "long period");
    c = base(); c.T = 12; c.I = 4; c.H = 8; c.dilation[1][1] = 30;   /* one window position, dilation beyond it */
    bad |= run_case(c, 0, 0, "single position");
    c = base(); c.n_blocks = 3; c.layers_in_block[2] = 1; c.dilation[2][0] = 1; c.n_cat = 6; c.lambda_c = 0.3;
    bad |= run_case(c, 1, 1, "three blocks, categories");
    c = base(); c.B = 1;
    bad |= run_case(c, 0, 0, "one series");
    return bad;
}
