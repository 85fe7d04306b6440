/*
 * Float64 CPU oracle for one ES-RNN training step (forward and reverse mode).
 *
 * TEST INFRASTRUCTURE ONLY.  This is the plain, slow statement of what the
 * method computes, written from the paper (arXiv 1907.03329) one formula at a
 * time: scalar loops per series, per time step, per window position and per
 * hidden unit, with no blocking, fusion or reordering.  It shares nothing with
 * the HIP library (no header, helper, table or constant), and only the tests,
 * the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * Passages followed (paper sections / equations):
 *   - Section 3.1, Eq. (1) and Eq. (3) with the trend removed as stated after
 *     Eq. (4): level and multiplicative-seasonality recursions.
 *   - Section 3.1, Eq. (5), (6): normalised, de-seasonalised windows and the
 *     re-seasonalised, de-normalised forecast.
 *   - Section 3.2 and Table 1: dilated LSTM stack with residual connections.
 *   - Section 3.4: tanh layer followed by a linear layer.
 *   - Section 3.5: masking of padded outputs and the pinball loss.
 *   - Section 8.2 (multiple seasonality, no seasonality) and Section 8.4
 *     (penalty on changes of the level; penalty on the squared cell state of
 *     the first layer of every block).
 *   - Section 3.3: per-series smoothing coefficients and initial seasonality
 *     are trained jointly with the network, hence the reverse sweep through
 *     the smoothing recursions.
 *   - Section 3.4 with Eq. (4): out-of-sample forecasts from the last input
 *     window, seasonal factors repeated with their period (eso_predict).
 *
 * Readings taken where the paper is silent are stated next to the code that
 * takes them.  Pins: closed forms, invariants, a library LSTM, brute force and
 * central finite differences (tests/test_oracle_*.py).  Readings that no pin can
 * separate ("parity unpinned"): the seasonal update dividing by the previous
 * level (printed form of Eq. (3)), natural logarithm on the windows, in-sample
 * seasonal factors for the training targets, the form of the level penalty,
 * the placement of the residual connections.
 *
 * Layouts.  Arguments shared with the C-ABI of the HIP library keep its
 * layouts: y [T][B] time-major, es_params [K][B] (rows: alpha, gamma1, gamma2,
 * s1_init[0..m1), s2_init[0..m2); absent rows omitted), weights flat (per
 * layer W [4h][in+h] row-major with gate rows input, forget, candidate, output
 * and columns input-then-recurrent (first layer: window, category one-hot), then bias [4h]; then Wa [h][h], ba [h],
 * Wo [H][h], bo [H]), forecasts [P][B][H].  Tape arrays are series-major.
 */
#ifndef ESRNN_ORACLE_H
#define ESRNN_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t B, T;
    int32_t n_seas, m1, m2;   /* 0: level only; 1: period m1; 2: periods m1 and m2 */
    int32_t I, H;             /* input window, horizon */
    int32_t hidden;
    int32_t n_blocks;
    int32_t layers_in_block[4];
    int32_t dilation[4][4];
    int32_t param_space;      /* 0: alpha, gamma, s_init given directly; 1: logit / log */
    double tau;               /* pinball quantile */
    double lambda_lv;         /* weight of the level penalty */
    double n_pin, n_lv;       /* > 0: use as normalisers instead of the counts from lengths */
    int32_t n_cat;            /* 0: none; else the network input is the window followed by a one-hot block of
                                 this many entries for the series' category (Section 5.3) */
    const int32_t *categories; /* [B], values in [0, n_cat); NULL if n_cat == 0 */
    double lambda_c;          /* weight of the cell-state penalty (Section 8.4, second kind); 0 disables it */
    const int8_t *pin_side;   /* NULL, or [B][P][H]: which one-sided derivative of the pinball loss (Section 3.5)
                                 eso_backward takes at an output.  0: the side the sign of target - output
                                 gives (target == output counts as the target >= output side); +1: the
                                 target >= output side; -1: the other side.  The loss is not differentiable
                                 where target == output, and both one-sided values are valid results there:
                                 a checker sets +-1 only at outputs that are equal to their targets up to the
                                 rounding of the implementation under test.  eso_forward ignores it. */
} eso_config;

/* Forward intermediates; every array is caller-allocated and series-major.
 * P = T - I - H + 1, L = number of layers, h = hidden. */
typedef struct {
    double *alpha, *gamma1, *gamma2;  /* [B] coefficients after the transform */
    double *l, *S1, *S2;              /* [B][T] level, seasonal factor applying at t */
    double *u, *v;                    /* [B][T] ln l, ln y - ln(S1*S2) */
    double *X;                        /* [B][P][I + n_cat] */
    double *Z;                        /* [B][P][H] */
    double *gates;                    /* [L][B][P][4][h] activated i, f, g, o */
    double *c, *h;                    /* [L][B][P][h] */
    double *blk;                      /* [n_blocks][B][P][h] block outputs */
    double *a;                        /* [B][P][h] tanh layer */
    double *o;                        /* [B][P][H] head output */
    double sum_pin, sum_lv, n_pin, n_lv;
    double sum_cs, n_cs;              /* cell-state penalty: sum of squares and number of terms */
} eso_tape;

/* Reverse-mode intermediates (any pointer may be NULL). */
typedef struct {
    double *gO;        /* [B][P][H] dL/do  (dL/dz is its negative) */
    double *gR;        /* [B][P][h] dL/d(top block output) */
    double *gX;        /* [B][P][I + n_cat] */
    double *gu, *gv;   /* [B][T] */
} eso_adjoint;

int eso_es_param_rows(const eso_config *cfg);
int64_t eso_weight_count(const eso_config *cfg);
int eso_num_layers(const eso_config *cfg);
int eso_max_threads(void);
void eso_set_num_threads(int n);   /* host threads used by later calls (timing only) */

/* Returns 0 on success, nonzero on an invalid configuration. */
int eso_forward(const eso_config *cfg, const double *y, const int32_t *lengths,
                const double *es_params, const double *weights,
                eso_tape *tape, double *loss, double *forecasts);

int eso_backward(const eso_config *cfg, const double *y, const int32_t *lengths,
                 const double *es_params, const double *weights,
                 const eso_tape *tape, eso_adjoint *adj,
                 double *grad_es_params, double *grad_weights);

/* Out-of-sample forecasts of the H steps after each series' last observation
 * (Section 3.4, Eq. (4), (5)): forecasts [B][H], original scale.  Needs
 * lengths[b] >= I; targets play no part.  Returns 0 on success. */
int eso_predict(const eso_config *cfg, const double *y, const int32_t *lengths,
                const double *es_params, const double *weights, double *forecasts);

#ifdef __cplusplus
}
#endif
#endif
