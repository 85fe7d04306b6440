/*
 * Float64 CPU oracle for one ES-RNN training step.  See esrnn_oracle.h for
 * scope, layouts and the list of paper passages; TEST INFRASTRUCTURE ONLY.
 *
 * Everything is done one series at a time (series never interact except
 * through the shared network weights and the two loss normalisers), in the
 * order the paper presents the method: smoothing recursions, windows, network,
 * loss; then the same chain in reverse for the gradients.
 */
#include "esrnn_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define MAX_LAYERS 16

typedef struct {
    int L;
    int dil[MAX_LAYERS];
    int block_of[MAX_LAYERS];
    int first_in_block[MAX_LAYERS];
    int last_in_block[MAX_LAYERS];
    int in_dim[MAX_LAYERS];
    int64_t W_off[MAX_LAYERS], b_off[MAX_LAYERS];
    int64_t Wa_off, ba_off, Wo_off, bo_off, n_weights;
    int P, K;
    int row_gamma1, row_gamma2, row_s1, row_s2;
} plan_t;

static int make_plan(const eso_config *c, plan_t *pl)
{
    if (c->B < 1 || c->T < 1 || c->I < 1 || c->H < 1 || c->hidden < 1) return 1;
    if (c->n_seas < 0 || c->n_seas > 2) return 1;
    if (c->n_seas >= 1 && (c->m1 < 1 || c->m1 > c->T)) return 1;
    if (c->n_seas >= 2 && (c->m2 < 1 || c->m2 > c->T)) return 1;
    if (c->I + c->H > c->T) return 1;
    if (c->n_blocks < 1 || c->n_blocks > 4) return 1;
    if (c->n_cat < 0 || c->n_cat > 16 || (c->n_cat > 0 && !c->categories)) return 1;
    if (!(c->tau > 0.0 && c->tau < 1.0)) return 1;
    int L = 0;
    int64_t off = 0;
    const int h = c->hidden;
    for (int k = 0; k < c->n_blocks; ++k) {
        if (c->layers_in_block[k] < 1 || c->layers_in_block[k] > 4) return 1;
        for (int j = 0; j < c->layers_in_block[k]; ++j) {
            if (c->dilation[k][j] < 1) return 1;
            pl->dil[L] = c->dilation[k][j];
            pl->block_of[L] = k;
            pl->first_in_block[L] = (j == 0);
            pl->last_in_block[L] = (j == c->layers_in_block[k] - 1);
            pl->in_dim[L] = (L == 0) ? c->I + c->n_cat : h;   /* window, then the category one-hot (Section 5.3) */
            pl->W_off[L] = off;
            off += (int64_t)4 * h * (pl->in_dim[L] + h);
            pl->b_off[L] = off;
            off += 4 * h;
            ++L;
        }
    }
    pl->L = L;
    pl->Wa_off = off; off += (int64_t)h * h;
    pl->ba_off = off; off += h;
    pl->Wo_off = off; off += (int64_t)c->H * h;
    pl->bo_off = off; off += c->H;
    pl->n_weights = off;
    pl->P = c->T - c->I - c->H + 1;
    int r = 1;
    pl->row_gamma1 = pl->row_gamma2 = pl->row_s1 = pl->row_s2 = -1;
    if (c->n_seas >= 1) pl->row_gamma1 = r++;
    if (c->n_seas >= 2) pl->row_gamma2 = r++;
    if (c->n_seas >= 1) { pl->row_s1 = r; r += c->m1; }
    if (c->n_seas >= 2) { pl->row_s2 = r; r += c->m2; }
    pl->K = r;
    return 0;
}

int eso_es_param_rows(const eso_config *cfg) { plan_t pl; return make_plan(cfg, &pl) ? -1 : pl.K; }
int64_t eso_weight_count(const eso_config *cfg) { plan_t pl; return make_plan(cfg, &pl) ? -1 : pl.n_weights; }
int eso_num_layers(const eso_config *cfg) { plan_t pl; return make_plan(cfg, &pl) ? -1 : pl.L; }
int eso_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Limits the host threads of the later calls (timing runs only; results do not depend on it beyond the
 * order in which per-thread weight-gradient sums are added). */
void eso_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

static double sigmoid(double x) { return 1.0 / (1.0 + exp(-x)); }

/* Normalisers of the two loss terms: the number of unmasked head outputs and
 * the number of second differences of the log level (Section 3.5: padded
 * outputs are left out of the loss). */
static void loss_counts(const eso_config *c, const int32_t *lengths, double *n_pin, double *n_lv)
{
    double np_ = 0.0, nl = 0.0;
    for (int b = 0; b < c->B; ++b) {
        int len = lengths[b];
        int Pb = len - c->I - c->H + 1;
        if (Pb > 0) np_ += (double)Pb * c->H;
        if (len > 2) nl += (double)(len - 2);
    }
    *n_pin = c->n_pin > 0.0 ? c->n_pin : np_;
    *n_lv = c->n_lv > 0.0 ? c->n_lv : nl;
}

/* ------------------------------------------------------------------------- */
/* Forward, one series                                                        */
/* ------------------------------------------------------------------------- */

/* Section 3.1 Eq. (1), (3) without trend (b == 1, text after Eq. (4)), with
 * the Section 8.2 variants.  S[t] is the seasonal factor that applies to time
 * t: the paper's s_{t-m} in Eq. (1); Eq. (3) produces the factor for t + m.
 * Reading for the state before the first observation (Section 3.3 only asks
 * for some initial estimate): l_{-1} = y_0 / S[0], which makes l_0 = y_0 / S[0] and
 * the first updated factor equal to the initial one. */
static void es_forward_series(const eso_config *c, const plan_t *pl, int b, int len,
                              const double *y, const double *es, eso_tape *tp)
{
    const int B = c->B, T = c->T;
    double *l = tp->l + (int64_t)b * T, *S1 = tp->S1 + (int64_t)b * T, *S2 = tp->S2 + (int64_t)b * T;
    double *u = tp->u + (int64_t)b * T, *v = tp->v + (int64_t)b * T;
    const int logit = (c->param_space == 1);

    /* smoothing coefficients lie strictly between zero and one (Section 3.1):
     * in the logit space they are sigmoids of free parameters, the initial
     * seasonal factors exponentials of free parameters */
    double alpha = es[0 * B + b], g1 = 0.0, g2 = 0.0;
    if (logit) alpha = sigmoid(alpha);
    if (c->n_seas >= 1) { g1 = es[(int64_t)pl->row_gamma1 * B + b]; if (logit) g1 = sigmoid(g1); }
    if (c->n_seas >= 2) { g2 = es[(int64_t)pl->row_gamma2 * B + b]; if (logit) g2 = sigmoid(g2); }
    tp->alpha[b] = alpha; tp->gamma1[b] = g1; tp->gamma2[b] = g2;

    for (int t = 0; t < T; ++t) { l[t] = 0.0; S1[t] = 1.0; S2[t] = 1.0; u[t] = 0.0; v[t] = 0.0; }
    if (c->n_seas >= 1)
        for (int k = 0; k < c->m1 && k < len; ++k) {
            double s = es[(int64_t)(pl->row_s1 + k) * B + b];
            S1[k] = logit ? exp(s) : s;
        }
    if (c->n_seas >= 2)
        for (int k = 0; k < c->m2 && k < len; ++k) {
            double s = es[(int64_t)(pl->row_s2 + k) * B + b];
            S2[k] = logit ? exp(s) : s;
        }
    const int m1 = c->m1, m2 = c->m2;

    /* t = 0 */
    l[0] = y[0 * B + b] / (S1[0] * S2[0]);
    if (c->n_seas >= 1 && m1 <= len - 1) S1[m1] = S1[0];
    if (c->n_seas >= 2 && m2 <= len - 1) S2[m2] = S2[0];
    for (int t = 1; t < len; ++t) {
        double yt = y[(int64_t)t * B + b];
        /* Eq. (1): de-seasonalise by every active factor, one after the other */
        l[t] = alpha * (yt / (S1[t] * S2[t])) + (1.0 - alpha) * l[t - 1];
        /* Eq. (3): the observation is divided by the previous level and, with
         * two seasonalities, by the other factor as well */
        if (c->n_seas >= 1 && t + m1 <= len - 1)
            S1[t + m1] = g1 * yt / (l[t - 1] * S2[t]) + (1.0 - g1) * S1[t];
        if (c->n_seas >= 2 && t + m2 <= len - 1)
            S2[t + m2] = g2 * yt / (l[t - 1] * S1[t]) + (1.0 - g2) * S2[t];
    }
    for (int t = 0; t < len; ++t) {
        u[t] = log(l[t]);
        v[t] = log(y[(int64_t)t * B + b]) - log(S1[t] * S2[t]);
    }
}

/* Section 5.3 and Eq. (6): every input value is divided by the level at the
 * window's last time step and by its own seasonal factor; the targets are
 * treated the same way.  Reading: natural logarithm of these ratios, stride
 * one, every position whose input and target windows are complete. */
static void window_series(const eso_config *c, const plan_t *pl, int b, int len, eso_tape *tp)
{
    const int T = c->T, I = c->I, H = c->H, P = pl->P;
    const int Iw = I + c->n_cat;   /* width of the network input */
    const double *u = tp->u + (int64_t)b * T, *v = tp->v + (int64_t)b * T;
    double *X = tp->X + (int64_t)b * P * Iw, *Z = tp->Z + (int64_t)b * P * H;
    memset(X, 0, sizeof(double) * P * Iw);
    memset(Z, 0, sizeof(double) * P * H);
    const int Pb = len - I - H + 1;
    for (int p = 0; p < Pb; ++p) {
        const int t = p + I - 1;
        for (int i = 0; i < I; ++i) X[p * Iw + i] = v[p + i] - u[t];
        /* Section 5.3: a one-hot representation of the series' category follows the window */
        for (int k = 0; k < c->n_cat; ++k) X[p * Iw + I + k] = (c->categories[b] == k) ? 1.0 : 0.0;
        for (int j = 1; j <= H; ++j) Z[p * H + (j - 1)] = v[t + j] - u[t];
    }
}

/* Section 3.2, Table 1: stack of LSTM cells whose recurrent state (hidden and
 * cell) comes from `dilation` positions back, zero before the start; blocks
 * after the first add their input to their output (residual).  Textbook cell,
 * no peepholes, one bias.  Section 3.4: tanh layer, then linear layer. */
static void network_series(const eso_config *c, const plan_t *pl, int b, int Pb,
                           const double *w, eso_tape *tp)
{
    const int h = c->hidden, P = pl->P, H = c->H, B = c->B, Iw = c->I + c->n_cat;
    for (int layer = 0; layer < pl->L; ++layer) {
        const int in = pl->in_dim[layer], d = pl->dil[layer], k = pl->block_of[layer];
        const double *W = w + pl->W_off[layer], *bias = w + pl->b_off[layer];
        double *G = tp->gates + ((int64_t)layer * B + b) * P * 4 * h;
        double *C = tp->c + ((int64_t)layer * B + b) * P * h;
        double *Hh = tp->h + ((int64_t)layer * B + b) * P * h;
        memset(G, 0, sizeof(double) * P * 4 * h);
        memset(C, 0, sizeof(double) * P * h);
        memset(Hh, 0, sizeof(double) * P * h);
        for (int p = 0; p < Pb; ++p) {
            const double *x;
            if (layer == 0) x = tp->X + ((int64_t)b * P + p) * Iw;
            else if (pl->first_in_block[layer]) x = tp->blk + (((int64_t)(k - 1) * B + b) * P + p) * h;
            else x = tp->h + (((int64_t)(layer - 1) * B + b) * P + p) * h;
            const double *hprev = (p - d >= 0) ? Hh + (int64_t)(p - d) * h : NULL;
            const double *cprev = (p - d >= 0) ? C + (int64_t)(p - d) * h : NULL;
            double *g = G + (int64_t)p * 4 * h;
            for (int r = 0; r < 4 * h; ++r) {
                double acc = bias[r];
                const double *Wr = W + (int64_t)r * (in + h);
                for (int q = 0; q < in; ++q) acc += Wr[q] * x[q];
                if (hprev) for (int q = 0; q < h; ++q) acc += Wr[in + q] * hprev[q];
                g[r] = acc;
            }
            for (int j = 0; j < h; ++j) {
                double gi = sigmoid(g[0 * h + j]), gf = sigmoid(g[1 * h + j]);
                double gg = tanh(g[2 * h + j]), go = sigmoid(g[3 * h + j]);
                double cp = cprev ? cprev[j] : 0.0;
                double cn = gf * cp + gi * gg;
                g[0 * h + j] = gi; g[1 * h + j] = gf; g[2 * h + j] = gg; g[3 * h + j] = go;
                C[(int64_t)p * h + j] = cn;
                Hh[(int64_t)p * h + j] = go * tanh(cn);
            }
        }
        if (pl->last_in_block[layer]) {
            double *out = tp->blk + ((int64_t)k * B + b) * P * h;
            memset(out, 0, sizeof(double) * P * h);
            for (int p = 0; p < Pb; ++p)
                for (int j = 0; j < h; ++j) {
                    double val = Hh[(int64_t)p * h + j];
                    if (k >= 1) val += tp->blk[(((int64_t)(k - 1) * B + b) * P + p) * h + j];
                    out[(int64_t)p * h + j] = val;
                }
        }
    }
    const double *Wa = w + pl->Wa_off, *ba = w + pl->ba_off, *Wo = w + pl->Wo_off, *bo = w + pl->bo_off;
    const double *R = tp->blk + ((int64_t)(c->n_blocks - 1) * B + b) * P * h;
    double *A = tp->a + (int64_t)b * P * h, *O = tp->o + (int64_t)b * P * H;
    memset(A, 0, sizeof(double) * P * h);
    memset(O, 0, sizeof(double) * P * H);
    for (int p = 0; p < Pb; ++p) {
        for (int j = 0; j < h; ++j) {
            double acc = ba[j];
            for (int q = 0; q < h; ++q) acc += Wa[(int64_t)j * h + q] * R[(int64_t)p * h + q];
            A[(int64_t)p * h + j] = tanh(acc);
        }
        for (int j = 0; j < H; ++j) {
            double acc = bo[j];
            for (int q = 0; q < h; ++q) acc += Wo[(int64_t)j * h + q] * A[(int64_t)p * h + q];
            O[(int64_t)p * H + j] = acc;
        }
    }
}

/* Section 3.5: pinball loss between target and output in the normalised
 * space, summed over unmasked positions; at a tie the branch z >= o is taken.
 * Section 8.4: squared second difference of the log level.  Eq. (5): forecast
 * = exp(output) * level at the window end * seasonal factors of the target
 * times (those of the in-sample recursion). */
static void loss_series(const eso_config *c, const plan_t *pl, int b, int len,
                        const eso_tape *tp, double *sum_pin, double *sum_lv, double *forecasts)
{
    const int T = c->T, I = c->I, H = c->H, P = pl->P, B = c->B;
    const int Pb = len - I - H + 1;
    const double *u = tp->u + (int64_t)b * T;
    const double *S1 = tp->S1 + (int64_t)b * T, *S2 = tp->S2 + (int64_t)b * T;
    const double *l = tp->l + (int64_t)b * T;
    const double *Z = tp->Z + (int64_t)b * P * H, *O = tp->o + (int64_t)b * P * H;
    double sp = 0.0, sl = 0.0;
    for (int p = 0; p < Pb; ++p)
        for (int j = 0; j < H; ++j) {
            double d = Z[p * H + j] - O[p * H + j];
            sp += (d >= 0.0) ? c->tau * d : (c->tau - 1.0) * d;
        }
    for (int t = 2; t < len; ++t) {
        double e = u[t] - 2.0 * u[t - 1] + u[t - 2];
        sl += e * e;
    }
    *sum_pin = sp;
    *sum_lv = sl;
    if (forecasts)
        for (int p = 0; p < P; ++p)
            for (int j = 1; j <= H; ++j) {
                double f = 0.0;
                if (p < Pb) {
                    int t = p + I - 1;
                    f = exp(O[p * H + (j - 1)]) * l[t] * S1[t + j] * S2[t + j];
                }
                forecasts[((int64_t)p * B + b) * H + (j - 1)] = f;
            }
}

/* Section 8.4, second kind of penalty: the mean of the squared cell states of the first layer of
 * every block (the paper's word for a block is stack).  Reading: one average over those layers, the valid window positions
 * of all series and the hidden units; this returns one series' sum of squares. */
static double cell_state_sumsq(const eso_config *c, const plan_t *pl, int b, int Pb, const eso_tape *tp)
{
    const int h = c->hidden, P = pl->P, B = c->B;
    double s = 0.0;
    for (int layer = 0; layer < pl->L; ++layer) {
        if (!pl->first_in_block[layer]) continue;
        const double *C = tp->c + ((int64_t)layer * B + b) * P * h;
        for (int p = 0; p < Pb; ++p)
            for (int j = 0; j < h; ++j) s += C[(int64_t)p * h + j] * C[(int64_t)p * h + j];
    }
    return s;
}

/* number of terms of that average */
static double cell_state_count(const eso_config *c, const int32_t *lengths)
{
    double n = 0.0;
    for (int b = 0; b < c->B; ++b) {
        int Pb = lengths[b] - c->I - c->H + 1;
        if (Pb > 0) n += (double)Pb;
    }
    return n * c->hidden * c->n_blocks;
}

int eso_forward(const eso_config *cfg, const double *y, const int32_t *lengths,
                const double *es_params, const double *weights,
                eso_tape *tape, double *loss, double *forecasts)
{
    plan_t pl;
    if (make_plan(cfg, &pl)) return 1;
    for (int b = 0; b < cfg->B; ++b)
        if (lengths[b] < cfg->I + cfg->H || lengths[b] > cfg->T) return 2;
    double total_pin = 0.0, total_lv = 0.0, total_cs = 0.0;
#pragma omp parallel for schedule(dynamic, 1) reduction(+ : total_pin, total_lv, total_cs)
    for (int b = 0; b < cfg->B; ++b) {
        const int len = lengths[b];
        double sp, sl;
        es_forward_series(cfg, &pl, b, len, y, es_params, tape);
        window_series(cfg, &pl, b, len, tape);
        network_series(cfg, &pl, b, len - cfg->I - cfg->H + 1, weights, tape);
        loss_series(cfg, &pl, b, len, tape, &sp, &sl, forecasts);
        total_pin += sp;
        total_lv += sl;
        if (cfg->lambda_c != 0.0) total_cs += cell_state_sumsq(cfg, &pl, b, len - cfg->I - cfg->H + 1, tape);
    }
    loss_counts(cfg, lengths, &tape->n_pin, &tape->n_lv);
    tape->sum_pin = total_pin;
    tape->sum_lv = total_lv;
    double L = total_pin / tape->n_pin;
    if (cfg->lambda_lv != 0.0 && tape->n_lv > 0.0) L += cfg->lambda_lv * total_lv / tape->n_lv;
    tape->sum_cs = total_cs;
    tape->n_cs = cell_state_count(cfg, lengths);
    if (cfg->lambda_c != 0.0 && tape->n_cs > 0.0) L += cfg->lambda_c * total_cs / tape->n_cs;
    *loss = L;
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Reverse mode, one series                                                   */
/* ------------------------------------------------------------------------- */

/* Network part: derivative of the pinball loss with respect to the head
 * output, then linear layer, tanh layer, residual blocks and the LSTM layers
 * back through the window positions.  gw accumulates weight gradients. */
static void network_backward_series(const eso_config *c, const plan_t *pl, int b, int Pb,
                                    const double *w, const eso_tape *tp, double n_pin, double n_cs,
                                    double *gO, double *gR, double *gX, double *gw)
{
    const int h = c->hidden, P = pl->P, H = c->H, B = c->B, Iw = c->I + c->n_cat;
    const double *Z = tp->Z + (int64_t)b * P * H, *O = tp->o + (int64_t)b * P * H;
    const double *A = tp->a + (int64_t)b * P * h;
    const double *R = tp->blk + ((int64_t)(c->n_blocks - 1) * B + b) * P * h;
    const double *Wa = w + pl->Wa_off, *Wo = w + pl->Wo_off;
    double *gWa = gw + pl->Wa_off, *gba = gw + pl->ba_off, *gWo = gw + pl->Wo_off, *gbo = gw + pl->bo_off;

    memset(gO, 0, sizeof(double) * P * H);
    memset(gR, 0, sizeof(double) * P * h);
    memset(gX, 0, sizeof(double) * P * Iw);
    double *da = (double *)calloc(h, sizeof(double));
    for (int p = 0; p < Pb; ++p) {
        for (int j = 0; j < H; ++j) {
            double d = Z[p * H + j] - O[p * H + j];
            /* rho = tau*d (d >= 0) or (tau-1)*d; d = z - o */
            int right = (d >= 0.0);
            /* kink of the loss: the caller may name the one-sided derivative to take (see eso_config) */
            if (c->pin_side) {
                const int8_t side = c->pin_side[((int64_t)b * P + p) * H + j];
                if (side > 0) right = 1;
                if (side < 0) right = 0;
            }
            gO[p * H + j] = (right ? -c->tau : (1.0 - c->tau)) / n_pin;
        }
        for (int q = 0; q < h; ++q) da[q] = 0.0;
        for (int j = 0; j < H; ++j) {
            double g = gO[p * H + j];
            gbo[j] += g;
            for (int q = 0; q < h; ++q) {
                gWo[(int64_t)j * h + q] += g * A[(int64_t)p * h + q];
                da[q] += Wo[(int64_t)j * h + q] * g;
            }
        }
        for (int j = 0; j < h; ++j) {
            double a = A[(int64_t)p * h + j];
            double dpre = da[j] * (1.0 - a * a);
            gba[j] += dpre;
            for (int q = 0; q < h; ++q) {
                gWa[(int64_t)j * h + q] += dpre * R[(int64_t)p * h + q];
                gR[(int64_t)p * h + q] += Wa[(int64_t)j * h + q] * dpre;
            }
        }
    }
    free(da);

    /* g_out: gradient with respect to the output of the block being processed;
     * g_h: gradient arriving at the hidden output of the layer being processed */
    double *g_out = (double *)malloc(sizeof(double) * P * h);
    double *g_in = (double *)malloc(sizeof(double) * P * h);
    double *g_h = (double *)malloc(sizeof(double) * P * h);
    double *dh_rec = (double *)malloc(sizeof(double) * P * h);
    double *dc_rec = (double *)malloc(sizeof(double) * P * h);
    double *dx = (double *)malloc(sizeof(double) * P * (h > Iw ? h : Iw));
    double *dgate = (double *)malloc(sizeof(double) * 4 * h);
    memcpy(g_out, gR, sizeof(double) * P * h);

    for (int layer = pl->L - 1; layer >= 0; --layer) {
        const int in = pl->in_dim[layer], d = pl->dil[layer], k = pl->block_of[layer];
        const double *W = w + pl->W_off[layer];
        double *gW = gw + pl->W_off[layer], *gb = gw + pl->b_off[layer];
        const double *G = tp->gates + ((int64_t)layer * B + b) * P * 4 * h;
        const double *C = tp->c + ((int64_t)layer * B + b) * P * h;
        const double *Hh = tp->h + ((int64_t)layer * B + b) * P * h;
        if (pl->last_in_block[layer]) {
            /* block output = (block input, if not the first block) + hidden of its last layer */
            memcpy(g_h, g_out, sizeof(double) * P * h);
            if (k >= 1) memcpy(g_in, g_out, sizeof(double) * P * h);
            else memset(g_in, 0, sizeof(double) * P * h);
        }
        memset(dh_rec, 0, sizeof(double) * P * h);
        memset(dc_rec, 0, sizeof(double) * P * h);
        memset(dx, 0, sizeof(double) * P * in);
        for (int p = Pb - 1; p >= 0; --p) {
            const double *x;
            if (layer == 0) x = tp->X + ((int64_t)b * P + p) * Iw;
            else if (pl->first_in_block[layer]) x = tp->blk + (((int64_t)(k - 1) * B + b) * P + p) * h;
            else x = tp->h + (((int64_t)(layer - 1) * B + b) * P + p) * h;
            const double *hprev = (p - d >= 0) ? Hh + (int64_t)(p - d) * h : NULL;
            const double *cprev = (p - d >= 0) ? C + (int64_t)(p - d) * h : NULL;
            const double *g = G + (int64_t)p * 4 * h;
            for (int j = 0; j < h; ++j) {
                double gi = g[0 * h + j], gf = g[1 * h + j], gg = g[2 * h + j], go = g[3 * h + j];
                double dh = g_h[(int64_t)p * h + j] + dh_rec[(int64_t)p * h + j];
                double tc = tanh(C[(int64_t)p * h + j]);
                double dc = dc_rec[(int64_t)p * h + j] + dh * go * (1.0 - tc * tc);
                /* cell-state penalty of a block's first layer: d/dc of lambda_c * c^2 / n_cs */
                if (c->lambda_c != 0.0 && pl->first_in_block[layer] && n_cs > 0.0)
                    dc += 2.0 * c->lambda_c * C[(int64_t)p * h + j] / n_cs;
                double cp = cprev ? cprev[j] : 0.0;
                dgate[0 * h + j] = dc * gg * gi * (1.0 - gi);
                dgate[1 * h + j] = dc * cp * gf * (1.0 - gf);
                dgate[2 * h + j] = dc * gi * (1.0 - gg * gg);
                dgate[3 * h + j] = dh * tc * go * (1.0 - go);
                if (cprev) dc_rec[(int64_t)(p - d) * h + j] += dc * gf;
            }
            for (int r = 0; r < 4 * h; ++r) {
                const double da_r = dgate[r];
                const double *Wr = W + (int64_t)r * (in + h);
                double *gWr = gW + (int64_t)r * (in + h);
                gb[r] += da_r;
                for (int q = 0; q < in; ++q) {
                    gWr[q] += da_r * x[q];
                    dx[(int64_t)p * in + q] += Wr[q] * da_r;
                }
                if (hprev)
                    for (int q = 0; q < h; ++q) {
                        gWr[in + q] += da_r * hprev[q];
                        dh_rec[(int64_t)(p - d) * h + q] += Wr[in + q] * da_r;
                    }
            }
        }
        if (layer == 0) {
            memcpy(gX, dx, sizeof(double) * P * Iw);
        } else if (pl->first_in_block[layer]) {
            /* the block input feeds both the first layer and the residual sum */
            for (int64_t q = 0; q < (int64_t)P * h; ++q) g_out[q] = g_in[q] + dx[q];
        } else {
            memcpy(g_h, dx, sizeof(double) * P * h);
        }
    }
    free(g_out); free(g_in); free(g_h); free(dh_rec); free(dc_rec); free(dx); free(dgate);
}

/* Adjoints of u = ln l and v = ln y - ln(S1 S2) from the windows (every x and
 * z is a difference v[.] - u[t]) and from the level penalty. */
static void window_backward_series(const eso_config *c, const plan_t *pl, int b, int len,
                                   const eso_tape *tp, const double *gX, const double *gO,
                                   double n_lv, double *gu, double *gv)
{
    const int T = c->T, I = c->I, H = c->H, Iw = c->I + c->n_cat;
    const int Pb = len - I - H + 1;
    const double *u = tp->u + (int64_t)b * T;
    (void)pl;
    for (int t = 0; t < T; ++t) { gu[t] = 0.0; gv[t] = 0.0; }
    for (int p = 0; p < Pb; ++p) {
        const int t = p + I - 1;
        for (int i = 0; i < I; ++i) {
            gv[p + i] += gX[p * Iw + i];      /* the one-hot columns past I carry no gradient further */
            gu[t] -= gX[p * Iw + i];
        }
        for (int j = 1; j <= H; ++j) {
            double gz = -gO[p * H + (j - 1)];   /* the loss depends on z - o only */
            gv[t + j] += gz;
            gu[t] -= gz;
        }
    }
    if (c->lambda_lv != 0.0 && n_lv > 0.0)
        for (int t = 2; t < len; ++t) {
            double e = u[t] - 2.0 * u[t - 1] + u[t - 2];
            double ge = c->lambda_lv * 2.0 * e / n_lv;
            gu[t] += ge;
            gu[t - 1] -= 2.0 * ge;
            gu[t - 2] += ge;
        }
}

/* Reverse sweep through Eq. (1), (3): Lb[t], S1b[t], S2b[t] are the adjoints of
 * l[t], S1[t], S2[t].  Going down in t, the adjoint of the factor produced at
 * step t (for time t + m) is complete when step t is reached, because every
 * use of it lies at or after t + m. */
static void es_backward_series(const eso_config *c, const plan_t *pl, int b, int len,
                               const double *y, const double *es, const eso_tape *tp,
                               const double *gu, const double *gv, double *g_es)
{
    const int B = c->B, T = c->T, m1 = c->m1, m2 = c->m2, ns = c->n_seas;
    const double *l = tp->l + (int64_t)b * T, *S1 = tp->S1 + (int64_t)b * T, *S2 = tp->S2 + (int64_t)b * T;
    const double alpha = tp->alpha[b], g1 = tp->gamma1[b], g2 = tp->gamma2[b];
    double *Lb = (double *)calloc(T, sizeof(double));
    double *S1b = (double *)calloc(T, sizeof(double));
    double *S2b = (double *)calloc(T, sizeof(double));
    double ab = 0.0, g1b = 0.0, g2b = 0.0;
    (void)es;

    for (int t = 0; t < len; ++t) {
        Lb[t] = gu[t] / l[t];                  /* u = ln l */
        if (ns >= 1) S1b[t] = -gv[t] / S1[t];  /* v = ln y - ln S1 - ln S2 */
        if (ns >= 2) S2b[t] = -gv[t] / S2[t];
    }
    for (int t = len - 1; t >= 1; --t) {
        const double yt = y[(int64_t)t * B + b];
        const double lp = l[t - 1];
        if (ns >= 1 && t + m1 <= len - 1) {
            /* S1[t+m1] = g1 * yt / (lp * S2[t]) + (1 - g1) * S1[t] */
            const double A = S1b[t + m1];
            const double r = yt / (lp * S2[t]);
            g1b += A * (r - S1[t]);
            Lb[t - 1] += -A * g1 * r / lp;
            if (ns >= 2) S2b[t] += -A * g1 * r / S2[t];
            S1b[t] += A * (1.0 - g1);
        }
        if (ns >= 2 && t + m2 <= len - 1) {
            /* S2[t+m2] = g2 * yt / (lp * S1[t]) + (1 - g2) * S2[t] */
            const double A = S2b[t + m2];
            const double r = yt / (lp * S1[t]);
            g2b += A * (r - S2[t]);
            Lb[t - 1] += -A * g2 * r / lp;
            S1b[t] += -A * g2 * r / S1[t];
            S2b[t] += A * (1.0 - g2);
        }
        /* l[t] = alpha * q + (1 - alpha) * lp, q = yt / (S1[t] * S2[t]) */
        const double q = yt / (S1[t] * S2[t]);
        ab += Lb[t] * (q - lp);
        if (ns >= 1) S1b[t] += -Lb[t] * alpha * q / S1[t];
        if (ns >= 2) S2b[t] += -Lb[t] * alpha * q / S2[t];
        Lb[t - 1] += Lb[t] * (1.0 - alpha);
    }
    /* t = 0: l[0] = y0 / (S1[0] * S2[0]); S1[m1] = S1[0]; S2[m2] = S2[0] */
    if (ns >= 1) {
        if (m1 <= len - 1) S1b[0] += S1b[m1];
        S1b[0] += -Lb[0] * l[0] / S1[0];
    }
    if (ns >= 2) {
        if (m2 <= len - 1) S2b[0] += S2b[m2];
        S2b[0] += -Lb[0] * l[0] / S2[0];
    }
    const int logit = (c->param_space == 1);
    g_es[0 * B + b] = logit ? ab * alpha * (1.0 - alpha) : ab;
    if (ns >= 1) {
        g_es[(int64_t)pl->row_gamma1 * B + b] = logit ? g1b * g1 * (1.0 - g1) : g1b;
        for (int k = 0; k < m1; ++k) {
            double gs = (k < len) ? S1b[k] : 0.0;
            g_es[(int64_t)(pl->row_s1 + k) * B + b] = logit ? gs * S1[k] : gs;
        }
    }
    if (ns >= 2) {
        g_es[(int64_t)pl->row_gamma2 * B + b] = logit ? g2b * g2 * (1.0 - g2) : g2b;
        for (int k = 0; k < m2; ++k) {
            double gs = (k < len) ? S2b[k] : 0.0;
            g_es[(int64_t)(pl->row_s2 + k) * B + b] = logit ? gs * S2[k] : gs;
        }
    }
    free(Lb); free(S1b); free(S2b);
}

int eso_backward(const eso_config *cfg, const double *y, const int32_t *lengths,
                 const double *es_params, const double *weights,
                 const eso_tape *tape, eso_adjoint *adj,
                 double *grad_es_params, double *grad_weights)
{
    plan_t pl;
    if (make_plan(cfg, &pl)) return 1;
    const int P = pl.P, h = cfg->hidden, T = cfg->T, I = cfg->I, H = cfg->H, Iw = cfg->I + cfg->n_cat;
    double n_pin, n_lv;
    loss_counts(cfg, lengths, &n_pin, &n_lv);
    const double n_cs = cell_state_count(cfg, lengths);
    memset(grad_weights, 0, sizeof(double) * pl.n_weights);
    int nthreads = eso_max_threads();
    double *gw_all = (double *)calloc((size_t)nthreads * pl.n_weights, sizeof(double));
    if (!gw_all) return 3;
#pragma omp parallel
    {
#ifdef _OPENMP
        const int tid = omp_get_thread_num();
#else
        const int tid = 0;
#endif
        double *gw = gw_all + (size_t)tid * pl.n_weights;
        double *gO = (double *)malloc(sizeof(double) * P * H);
        double *gR = (double *)malloc(sizeof(double) * P * h);
        double *gX = (double *)malloc(sizeof(double) * P * Iw);
        double *gu = (double *)malloc(sizeof(double) * T);
        double *gv = (double *)malloc(sizeof(double) * T);
#pragma omp for schedule(dynamic, 1)
        for (int b = 0; b < cfg->B; ++b) {
            const int len = lengths[b];
            network_backward_series(cfg, &pl, b, len - I - H + 1, weights, tape, n_pin, n_cs, gO, gR, gX, gw);
            window_backward_series(cfg, &pl, b, len, tape, gX, gO, n_lv, gu, gv);
            es_backward_series(cfg, &pl, b, len, y, es_params, tape, gu, gv, grad_es_params);
            if (adj) {
                if (adj->gO) memcpy(adj->gO + (int64_t)b * P * H, gO, sizeof(double) * P * H);
                if (adj->gR) memcpy(adj->gR + (int64_t)b * P * h, gR, sizeof(double) * P * h);
                if (adj->gX) memcpy(adj->gX + (int64_t)b * P * Iw, gX, sizeof(double) * P * Iw);
                if (adj->gu) memcpy(adj->gu + (int64_t)b * T, gu, sizeof(double) * T);
                if (adj->gv) memcpy(adj->gv + (int64_t)b * T, gv, sizeof(double) * T);
            }
        }
        free(gO); free(gR); free(gX); free(gu); free(gv);
    }
    for (int t = 0; t < nthreads; ++t)
        for (int64_t q = 0; q < pl.n_weights; ++q) grad_weights[q] += gw_all[(size_t)t * pl.n_weights + q];
    free(gw_all);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Out-of-sample forecast, one series at a time                               */
/* ------------------------------------------------------------------------- */

/* Section 3.4 (forecasting from the end of a series) with Eq. (4) and (5): the smoothing
 * recursions run over the whole series; every position with a complete input
 * window goes through the network (no targets are needed); the output at the
 * last position, whose window ends at the last observation t = len-1, is
 * de-normalised with the level l_t and re-seasonalised.  The seasonal factor
 * of forecast step h is the one Eq. (4) names, s_{t-m+h_m^+} with
 * h_m^+ = ((h-1) mod m) + 1: the last m factors the recursion has produced,
 * repeated with period m.  In the indexing used here (S[t] is the factor that
 * applies at time t; Eq. (3) at step t produces S[t+m]) that is
 * S[t + ((h-1) mod m) + 1].  Written out on its own arrays, sized by the
 * series, so that it can be compared with the training pass rather than
 * derived from it. */
int eso_predict(const eso_config *cfg, const double *y, const int32_t *lengths,
                const double *es_params, const double *weights, double *forecasts)
{
    plan_t pl;
    if (make_plan(cfg, &pl)) return 1;
    const int B = cfg->B, I = cfg->I, H = cfg->H, h = cfg->hidden;
    const int m1 = cfg->n_seas >= 1 ? cfg->m1 : 0, m2 = cfg->n_seas >= 2 ? cfg->m2 : 0;
    const int logit = (cfg->param_space == 1);
    for (int b = 0; b < B; ++b)
        if (lengths[b] < I || lengths[b] > cfg->T) return 2;
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        const int len = lengths[b];
        const int Pp = len - I + 1;                 /* positions with a complete input window */
        const int ext = len + (m1 > m2 ? m1 : m2);  /* factors exist up to index len-1+m */
        double *l = (double *)malloc(sizeof(double) * len);
        double *S1 = (double *)malloc(sizeof(double) * (ext + 1));
        double *S2 = (double *)malloc(sizeof(double) * (ext + 1));
        const int Iw = I + cfg->n_cat;
        double *cur = (double *)malloc(sizeof(double) * Pp * (Iw > h ? Iw : h));   /* input of the current layer */
        double *blk_in = (double *)malloc(sizeof(double) * Pp * h);              /* input of the current block */
        double *hs = (double *)malloc(sizeof(double) * Pp * h);
        double *cs = (double *)malloc(sizeof(double) * Pp * h);
        double *g = (double *)malloc(sizeof(double) * 4 * h);
        double *a = (double *)malloc(sizeof(double) * h);
        if (!l || !S1 || !S2 || !cur || !blk_in || !hs || !cs || !g || !a) {
#pragma omp atomic write
            fail = 1;
        } else {
            double alpha = es_params[b], g1 = 0.0, g2 = 0.0;
            if (logit) alpha = sigmoid(alpha);
            if (m1) { g1 = es_params[(int64_t)pl.row_gamma1 * B + b]; if (logit) g1 = sigmoid(g1); }
            if (m2) { g2 = es_params[(int64_t)pl.row_gamma2 * B + b]; if (logit) g2 = sigmoid(g2); }
            for (int t = 0; t <= ext; ++t) { S1[t] = 1.0; S2[t] = 1.0; }
            for (int k = 0; k < m1; ++k) { double v0 = es_params[(int64_t)(pl.row_s1 + k) * B + b]; S1[k] = logit ? exp(v0) : v0; }
            for (int k = 0; k < m2; ++k) { double v0 = es_params[(int64_t)(pl.row_s2 + k) * B + b]; S2[k] = logit ? exp(v0) : v0; }
            /* Eq. (1), (3); state before the first observation as in the training pass */
            l[0] = y[b] / (S1[0] * S2[0]);
            if (m1) S1[m1] = S1[0];
            if (m2) S2[m2] = S2[0];
            for (int t = 1; t < len; ++t) {
                const double yt = y[(int64_t)t * B + b];
                l[t] = alpha * (yt / (S1[t] * S2[t])) + (1.0 - alpha) * l[t - 1];
                if (m1) S1[t + m1] = g1 * yt / (l[t - 1] * S2[t]) + (1.0 - g1) * S1[t];
                if (m2) S2[t + m2] = g2 * yt / (l[t - 1] * S1[t]) + (1.0 - g2) * S2[t];
            }
            /* Eq. (6) inputs: ln( y / (level at the window end * own seasonal factor) ) */
            for (int p = 0; p < Pp; ++p) {
                const int t = p + I - 1;
                for (int i = 0; i < I; ++i)
                    cur[p * Iw + i] = log(y[(int64_t)(p + i) * B + b] / (l[t] * S1[p + i] * S2[p + i]));
                for (int k = 0; k < cfg->n_cat; ++k) cur[p * Iw + I + k] = (cfg->categories[b] == k) ? 1.0 : 0.0;
            }
            /* Section 3.2: dilated LSTM layers, residual around every block but the first */
            int width = Iw;
            for (int layer = 0; layer < pl.L; ++layer) {
                const int in = pl.in_dim[layer], d = pl.dil[layer];
                const double *W = weights + pl.W_off[layer], *bias = weights + pl.b_off[layer];
                if (pl.first_in_block[layer] && layer > 0) memcpy(blk_in, cur, sizeof(double) * Pp * h);
                for (int p = 0; p < Pp; ++p) {
                    for (int r = 0; r < 4 * h; ++r) {
                        double acc = bias[r];
                        for (int q = 0; q < in; ++q) acc += W[(int64_t)r * (in + h) + q] * cur[p * width + q];
                        if (p - d >= 0)
                            for (int q = 0; q < h; ++q) acc += W[(int64_t)r * (in + h) + in + q] * hs[(p - d) * h + q];
                        g[r] = acc;
                    }
                    for (int j = 0; j < h; ++j) {
                        const double gi = sigmoid(g[j]), gf = sigmoid(g[h + j]), gg = tanh(g[2 * h + j]), go = sigmoid(g[3 * h + j]);
                        const double cn = gf * (p - d >= 0 ? cs[(p - d) * h + j] : 0.0) + gi * gg;
                        cs[p * h + j] = cn;
                        hs[p * h + j] = go * tanh(cn);
                    }
                }
                /* the layer's hidden sequence is the next layer's input; a block past the first adds its input */
                for (int p = 0; p < Pp; ++p)
                    for (int j = 0; j < h; ++j) {
                        double val = hs[p * h + j];
                        if (pl.last_in_block[layer] && pl.block_of[layer] >= 1) val += blk_in[p * h + j];
                        cur[p * h + j] = val;
                    }
                width = h;
            }
            /* Section 3.4 at the last position; Eq. (5) with the factors of Eq. (4) */
            const double *Wa = weights + pl.Wa_off, *ba = weights + pl.ba_off, *Wo = weights + pl.Wo_off, *bo = weights + pl.bo_off;
            const double *R = cur + (int64_t)(Pp - 1) * h;
            const int t = len - 1;
            for (int j = 0; j < h; ++j) {
                double acc = ba[j];
                for (int q = 0; q < h; ++q) acc += Wa[(int64_t)j * h + q] * R[q];
                a[j] = tanh(acc);
            }
            for (int hh = 1; hh <= H; ++hh) {
                double o = bo[hh - 1];
                for (int q = 0; q < h; ++q) o += Wo[(int64_t)(hh - 1) * h + q] * a[q];
                double seas = 1.0;
                if (m1) seas *= S1[t + ((hh - 1) % m1) + 1];
                if (m2) seas *= S2[t + ((hh - 1) % m2) + 1];
                forecasts[(int64_t)b * H + (hh - 1)] = exp(o) * l[t] * seas;
            }
        }
        free(l); free(S1); free(S2); free(cur); free(blk_in); free(hs); free(cs); free(g); free(a);
    }
    return fail ? 3 : 0;
}

