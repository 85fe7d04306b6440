/*
 * esrnn.h - C ABI of the MI355X (gfx950) ES-RNN training-step library.
 *
 * One call of esrnn_forward followed by one call of esrnn_backward is one
 * batched training step of the hybrid exponential-smoothing / recurrent
 * network model of arXiv 1907.03329 over B series at once:
 *
 *   Section 3.1, Eq. (1), (3)   per-series multiplicative smoothing of level
 *                               and seasonality (no trend, text after Eq. (4)),
 *                               sequential in time, parallel over series;
 *                               Section 8.2: two seasonalities, or none
 *   Section 5.3, Eq. (6)        sliding input / target windows, divided by the
 *                               level at the window end and by the seasonal
 *                               factors (natural log of the ratios)
 *   Section 3.2, Table 1        blocks of dilated LSTM layers with residual
 *                               connections between blocks
 *   Section 3.4                 tanh layer and linear layer
 *   Section 3.5, Section 8.4    pinball loss over unmasked outputs plus a
 *                               penalty on second differences of the log level
 *   Eq. (5)                     forecasts = exp(output) * level * seasonality
 *   Section 3.3                 gradients with respect to the per-series
 *                               smoothing parameters and the shared weights
 *
 * Conventions
 *   - Every function returns an esrnn_status; 0 is success.  Nothing throws or
 *     aborts.  Configuration errors are reported before any kernel is launched.
 *   - All array arguments are DEVICE pointers owned by the caller; the library
 *     reads inputs and writes only outputs and the workspace.  It allocates no
 *     device memory.  All work is enqueued on `stream` (a hipStream_t passed as
 *     void*, NULL = the default stream); no call synchronises with the host.
 *   - fp32 throughout.  Series values must be strictly positive inside their
 *     length; values past the length are ignored.
 *   - A handle may be used by one thread at a time.  A workspace belongs to one
 *     forward/backward pair at a time.
 */
#ifndef ESRNN_H
#define ESRNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ESRNN_MAX_BLOCKS 4
#define ESRNN_MAX_LAYERS_PER_BLOCK 4
#define ESRNN_MAX_HIDDEN 64
#define ESRNN_MAX_WINDOW 64   /* limit for both I + n_categories and H */
#define ESRNN_MAX_CATEGORIES 16

typedef enum {
    ESRNN_OK = 0,
    ESRNN_ERR_NULL = 1,       /* a required pointer is NULL */
    ESRNN_ERR_CONFIG = 2,     /* configuration outside the supported range */
    ESRNN_ERR_WORKSPACE = 3,  /* workspace pointer misaligned (256 bytes required), or the built-in workspace of
                                 esrnn_predict_static too small for this configuration */
    ESRNN_ERR_ORDER = 4,      /* esrnn_backward without a preceding esrnn_forward on the handle */
    ESRNN_ERR_HIP = 5         /* a HIP runtime call or kernel launch failed */
} esrnn_status;

typedef enum {
    ESRNN_PARAMS_DIRECT = 0,  /* alpha, gamma in [0,1] and s_init > 0 are given as such; gradients are with respect to them */
    ESRNN_PARAMS_LOGIT = 1    /* alpha, gamma = sigmoid(theta), s_init = exp(theta); gradients are with respect to theta
                                 (Section 3.1: smoothing coefficients lie between zero and one) */
} esrnn_param_space;

typedef struct {
    int32_t B, T;             /* number of series; padded length (rows of y) */
    int32_t n_seas, m1, m2;   /* 0: level only; 1: one seasonality of period m1; 2: periods m1 and m2 (Section 8.2) */
    int32_t I, H;             /* input window and horizon (= output window), Section 3.1 */
    int32_t hidden;           /* LSTM state size (Table 1) */
    int32_t n_blocks;         /* 1..ESRNN_MAX_BLOCKS residual blocks */
    int32_t layers_in_block[ESRNN_MAX_BLOCKS];
    int32_t dilation[ESRNN_MAX_BLOCKS][ESRNN_MAX_LAYERS_PER_BLOCK];  /* Table 1 */
    float tau;                /* pinball quantile in (0,1) */
    float lambda_lv;          /* weight of the level penalty; 0 disables it */
    int32_t param_space;      /* esrnn_param_space */
    int32_t n_categories;     /* 0: none; else the network input is the window followed by a one-hot block of this
                                 many entries for the series' category (Section 5.3; the paper's data has 6), and the
                                 first layer's W is [4*hidden][I + n_categories + hidden].  See esrnn_set_categories */
    float lambda_cs;          /* weight of the cell-state penalty (Section 8.4: the average squared cell state of the
                                 first layer of every block, over valid window positions, units and those layers);
                                 0 disables it */
} esrnn_config;

typedef struct esrnn_handle esrnn_handle;

/* Validates the configuration (I + H <= T, periods <= T and m1 + m2 <= 448 (the seasonal rings of 64 series
 * and a 48 KB staging buffer must fit into the 160 KB of LDS), dilations >= 1, sizes within the ESRNN_MAX_* limits, 0 < tau < 1) and
 * builds the launch plan.
 * The plan picks, from the batch size, between two kernels each for the LSTM layers (4-series tiles at small
 * batches, 16-series tiles otherwise) and for the window adjoint (gather, or streaming at very many series);
 * the results agree to rounding.  Two environment variables, read here, override the choice for measurements:
 * ESRNN_NARROW_BELOW (16-series workgroups below which a layer uses 4-series tiles) and
 * ESRNN_WINDOW_STREAM_FROM (16-series tiles from which the window adjoint streams).
 * Host-only; touches no device. */
esrnn_status esrnn_create(const esrnn_config *cfg, esrnn_handle **out);
esrnn_status esrnn_destroy(esrnn_handle *h);

/* Category of every series (Section 5.3): device array [B] of int32 in [0, n_categories), read by every
 * later esrnn_forward, esrnn_predict and esrnn_es_window_forward on this handle; it must stay valid until
 * then.  Required before those calls when n_categories > 0 (they return ESRNN_ERR_NULL otherwise). */
esrnn_status esrnn_set_categories(esrnn_handle *h, const int32_t *categories);

/* Callers that only evaluate (loss and forecasts of esrnn_forward, no esrnn_backward): with on != 0 the output
 * stage of esrnn_forward skips its reverse pass (Sections 3.4, 3.5 forward only) and esrnn_backward returns
 * ESRNN_ERR_ORDER until it is switched off again.  Off by default.  esrnn_predict never runs that reverse pass. */
esrnn_status esrnn_set_forward_only(esrnn_handle *h, int32_t on);

/* Sizes the caller needs to allocate buffers. */
esrnn_status esrnn_workspace_bytes(const esrnn_handle *h, size_t *bytes);
/* The calls below take the workspace as a bare pointer and cannot see its size.  A caller can have both of its
 * properties checked here, on the host, once: ESRNN_OK if `workspace` is 256-byte aligned and `bytes` is at least
 * esrnn_workspace_bytes (with es_window_only != 0: at least esrnn_es_window_workspace_bytes, the prefix that the
 * esrnn_es_window_* calls use), ESRNN_ERR_WORKSPACE otherwise.  The pointer is not dereferenced. */
esrnn_status esrnn_check_workspace(const esrnn_handle *h, const void *workspace, size_t bytes, int32_t es_window_only);
esrnn_status esrnn_es_param_rows(const esrnn_handle *h, int32_t *K);   /* K = 1 + n_seas + m1 + m2 (Section 3.3) */
esrnn_status esrnn_weight_count(const esrnn_handle *h, size_t *n);     /* length of the flat weight vector */
const char *esrnn_status_string(esrnn_status s);

/*
 * Forward pass: smoothing recursions, windows, network, loss, forecasts.
 * The output stage (Sections 3.4, 3.5) also runs its own reverse pass here,
 * while its activations are on chip: the gradient of the pinball loss with
 * respect to an output needs only that output, its target and the count of
 * unmasked outputs.  Its results wait in the workspace for esrnn_backward.
 *
 *   y          [T][B] time-major.  Series b occupies t = 0 .. lengths[b]-1.
 *   lengths    [B] int32, I + H <= lengths[b] <= T (values outside are clamped).
 *   es_params  [K][B]; rows in this order, absent ones omitted: alpha, gamma1,
 *              gamma2, s1_init[0..m1), s2_init[0..m2).
 *   weights    flat.  Per LSTM layer, in stack order: W [4*hidden][in+hidden]
 *              row-major, gate rows in the order input, forget, candidate,
 *              output, columns first the layer input (in = I for the first
 *              layer, hidden otherwise) then the recurrent state; bias
 *              [4*hidden].  Then Wa [hidden][hidden], ba [hidden] (tanh layer),
 *              Wo [H][hidden], bo [H] (linear layer).
 *   workspace  >= esrnn_workspace_bytes, 256-byte aligned; afterwards holds
 *              everything esrnn_backward needs.
 *   loss       one float: mean pinball loss over unmasked outputs + lambda_lv *
 *              mean squared second difference of the log level + lambda_cs * mean
 *              squared cell state of the first layer of every block.
 *   forecasts  [P][B][H] with P = T - I - H + 1, original scale, zero where the
 *              window does not fit into the series; may be NULL.
 */
esrnn_status esrnn_forward(esrnn_handle *h, const float *y, const int32_t *lengths,
                           const float *es_params, const float *weights, void *workspace,
                           float *loss, float *forecasts, void *stream);

/*
 * Reverse pass for the forward pass last run on this handle with the same
 * inputs and workspace.  grad_es_params [K][B] and grad_weights (flat, packed
 * like weights) are overwritten, not accumulated into.
 */
esrnn_status esrnn_backward(esrnn_handle *h, const float *y, const int32_t *lengths,
                            const float *es_params, const float *weights, void *workspace,
                            float *grad_es_params, float *grad_weights, void *stream);

/*
 * Parameter update after esrnn_backward, for callers that train in a loop.
 * Section 3.3 trains the per-series smoothing parameters jointly with the
 * network weights; the paper does not name its optimiser.  This is the Adam
 * rule as published (Kingma & Ba 2015, Algorithm 1, with bias correction),
 * preceded by clipping of the gradient by its global L2 norm over both
 * parameter sets: g <- g * min(1, clip_norm / (||g|| + 1e-6)).
 *   m <- beta1 m + (1 - beta1) g,  v <- beta2 v + (1 - beta2) g^2,
 *   p <- p - lr * (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps)
 * step counts from 1.  weights, es_params and the four moment arrays (same
 * shapes as their parameters, zero before the first step) are updated in place;
 * the gradients are read only.  Uses a few KB of the workspace.
 */
typedef struct {
    float lr_weights, lr_es;  /* learning rates of the shared weights and of the per-series parameters */
    float beta1, beta2, eps;
    float clip_norm;          /* <= 0: no clipping */
} esrnn_adam_config;

esrnn_status esrnn_adam_update(esrnn_handle *h, const esrnn_adam_config *opt, int32_t step,
                               float *weights, const float *grad_weights, float *m_weights, float *v_weights,
                               float *es_params, const float *grad_es_params, float *m_es, float *v_es,
                               void *workspace, void *stream);

/*
 * Training over a store of N series, a batch of B at a time (Section 3.3: every series has its own smoothing
 * parameters, N (2 + S) in all, trained jointly with the shared weights; Table 5: training runs for epochs of
 * batches).  The store holds y_store [T][N], lengths_store [N], es_store [K][N], the Adam moments of the
 * per-series parameters m_es_store, v_es_store [K][N] (zero before the first step) and one update counter per
 * series counts_store [N] (int32, zero before the first step); index [B] (int32, distinct values in [0, N))
 * names the series of the batch.  All device pointers.
 *
 * esrnn_gather_batch copies the batch's series, lengths and parameters out of the store into the [T][B], [B]
 * and [K][B] arrays that esrnn_forward / esrnn_backward take.
 *
 * esrnn_adam_update_indexed is esrnn_adam_update for such a batch: the shared weights take the Adam step with
 * counter `step`; of the store only the columns named by index are touched, column index[b] with the gradient
 * grad_es_params[:, b] and, in the bias correction, its own counter counts_store[index[b]] + 1 (a series is
 * optimised as if on its own and simply has no step while it is not in a batch; a reading: the paper names
 * neither the optimiser nor the handling of per-series state between batches).  Clipping is by the global L2
 * norm over the weight gradient and the batch's per-series gradients.  The counters of the batch's series
 * are incremented.  Series outside the batch keep parameters, moments and counters bit for bit.
 */
esrnn_status esrnn_gather_batch(esrnn_handle *h, const float *y_store, const int32_t *lengths_store,
                                const float *es_store, const int32_t *index, int32_t N,
                                float *y, int32_t *lengths, float *es_params, void *stream);
esrnn_status esrnn_adam_update_indexed(esrnn_handle *h, const esrnn_adam_config *opt, int32_t step,
                                       float *weights, const float *grad_weights, float *m_weights, float *v_weights,
                                       float *es_store, const float *grad_es_params, float *m_es_store,
                                       float *v_es_store, int32_t *counts_store, const int32_t *index, int32_t N,
                                       void *workspace, void *stream);

/*
 * Out-of-sample forecasts (Section 3.4, the use of the trained network on a series' end; Eq. (4), (5)):
 * the H steps after each series' last observation, from the window of the last
 * I observations, de-normalised with the last level and re-seasonalised with
 * the last m factors of the recursion repeated with period m.
 *
 *   forecasts  [B][H], original scale.  A series with lengths[b] < I or
 *              lengths[b] + H > T gets zeros: the pass runs on lengths extended
 *              by H, so y needs H rows past every series to be forecast.  Those
 *              rows are read; their values do not reach the forecasts.
 *
 * Inputs and workspace as for esrnn_forward.  The workspace afterwards holds the
 * state of the extended problem: esrnn_backward must not follow (it returns
 * ESRNN_ERR_ORDER).
 */
esrnn_status esrnn_predict(esrnn_handle *h, const float *y, const int32_t *lengths, const float *es_params,
                           const float *weights, void *workspace, float *forecasts, void *stream);

/*
 * esrnn_predict for callers that cannot allocate device memory and have no workspace to pass: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs, same kernels and
 * same results as esrnn_predict, but the workspace is an array inside the library (device memory of
 * ESRNN_STATIC_SCRATCH_BYTES that every GPU the library runs on holds until the process ends).  The call
 * allocates nothing and frees nothing; its first call on a device looks the array's address up.
 * Returns ESRNN_ERR_WORKSPACE if esrnn_workspace_bytes of this handle exceeds ESRNN_STATIC_SCRATCH_BYTES
 * (batch too large for the built-in array: use esrnn_predict with a workspace of your own).
 * All calls on one GPU, from every handle, share the one array, which keeps the contents of the last
 * call (no part of it needs clearing: every kernel writes what it later reads): calls that overlap on
 * one GPU race, and esrnn_backward must not follow.
 */
#define ESRNN_STATIC_SCRATCH_BYTES (32u << 20)
esrnn_status esrnn_predict_static(esrnn_handle *h, const float *y, const int32_t *lengths, const float *es_params,
                                  const float *weights, float *forecasts, void *stream);

/*
 * Accuracy per series of forecasts [B][H] against actual values [B][H], with the
 * two metrics of the M4 competition that Section 3.5 names:
 *   smape [B]  mean over the horizon of 200 |a - f| / (|a| + |f|)   (percent)
 *   mase  [B]  mean |a - f| over the horizon, divided by the mean of
 *              |y_t - y_{t-m}| over t = m .. lengths[b]-1 (in-sample seasonal
 *              naive forecast; m = the seasonal period, 1 for none).
 * y [T][B] and lengths as for esrnn_forward; lengths[b] > m is required.
 */
esrnn_status esrnn_forecast_metrics(esrnn_handle *h, const float *forecasts, const float *actuals, const float *y,
                                    const int32_t *lengths, int32_t m, float *smape, float *mase, void *stream);

/*
 * The smoothing and window stages on their own (Section 3.1 Eq. (1), (3), Section
 * 5.3 Eq. (6), and their adjoints), for callers that fit or inspect the
 * exponential-smoothing part without the network, and for measuring these
 * stages at batch sizes whose network stash would not fit.  They use only the
 * first esrnn_es_window_workspace_bytes bytes of the workspace layout (a full
 * workspace works too).  esrnn_es_window_forward fills the level, seasonal
 * factors, u, v and the window tiles X, Z (see esrnn_workspace_buffer).
 * esrnn_es_window_backward takes the window gradients the caller has placed in
 * the ESRNN_BUF_GRAD_X and ESRNN_BUF_GRAD_O tiles of the workspace (every
 * element, padding rows included, must be finite), adds the gradient of the
 * level penalty, and writes grad_es_params [K][B].
 */
esrnn_status esrnn_es_window_workspace_bytes(const esrnn_handle *h, size_t *bytes);
esrnn_status esrnn_es_window_forward(esrnn_handle *h, const float *y, const int32_t *lengths,
                                     const float *es_params, void *workspace, void *stream);
esrnn_status esrnn_es_window_backward(esrnn_handle *h, const float *y, const int32_t *lengths,
                                      const float *es_params, void *workspace, float *grad_es_params, void *stream);

/*
 * Where an intermediate lives inside the workspace, for tests and profiling.
 * Layout kinds:
 *   ESRNN_LAYOUT_TIME_MAJOR  [T][Bt], Bt = 64 * ceil(B / 64)
 *   ESRNN_LAYOUT_TILE        [P][Bp/16][R][16], Bp = 16 * ceil(B / 16): element (p, b, r) at
 *                            ((p * Bp/16 + b/16) * R + r) * 16 + b%16; rows past
 *                            the logical count are padding
 *   ESRNN_LAYOUT_GATE_TILE   as TILE with a trailing [4] (activated input,
 *                            forget, candidate, output gate of hidden unit r)
 * dims = {T or P, Bt or Bp, R (padded rows), logical rows}.
 */
typedef enum {
    ESRNN_BUF_LEVEL = 0, ESRNN_BUF_S1, ESRNN_BUF_S2, ESRNN_BUF_U, ESRNN_BUF_V,   /* time-major */
    ESRNN_BUF_X, ESRNN_BUF_Z,                                                    /* tile */
    ESRNN_BUF_GATES,                                                             /* gate tile, index = layer */
    ESRNN_BUF_C, ESRNN_BUF_HID,                                                  /* tile, index = layer */
    ESRNN_BUF_BLOCK_OUT,                                                         /* tile, index = block */
    ESRNN_BUF_O,                                                                 /* tile: linear-layer outputs */
    ESRNN_BUF_GRAD_O, ESRNN_BUF_GRAD_TOP,                                        /* tile (filled by esrnn_forward) */
    ESRNN_BUF_GRAD_X,                                                            /* tile (after backward) */
    ESRNN_BUF_GRAD_U, ESRNN_BUF_GRAD_V,                                          /* time-major (after backward) */
    ESRNN_BUF_COUNT_
} esrnn_buffer;

typedef enum { ESRNN_LAYOUT_TIME_MAJOR = 0, ESRNN_LAYOUT_TILE = 1, ESRNN_LAYOUT_GATE_TILE = 2 } esrnn_layout;

typedef struct {
    size_t offset_bytes;
    int32_t layout;
    int32_t dims[4];
} esrnn_buffer_view;

esrnn_status esrnn_workspace_buffer(const esrnn_handle *h, int32_t which, int32_t index, esrnn_buffer_view *out);

/*
 * Per-stage timing for benchmarks.  While enabled, esrnn_forward and
 * esrnn_backward bracket every stage (one kernel launch, except the packing
 * and gradient-reduction stages, which launch one small kernel per layer) with
 * HIP events on the caller's stream.  esrnn_profile_collect waits for the
 * events of the last forward/backward pair (the only call here that blocks the
 * host) and adds their elapsed times to per-stage totals; call it once after
 * each pair.  esrnn_profile_read copies the totals in milliseconds and the
 * number of collected launches into host arrays of esrnn_profile_stage_count
 * entries.  Enabling resets the totals.
 */
esrnn_status esrnn_profile_enable(esrnn_handle *h, int32_t on);
esrnn_status esrnn_profile_stage_count(const esrnn_handle *h, int32_t *n);
esrnn_status esrnn_profile_stage_name(const esrnn_handle *h, int32_t i, const char **name);
esrnn_status esrnn_profile_collect(esrnn_handle *h);
esrnn_status esrnn_profile_read(const esrnn_handle *h, double *total_ms, int32_t *launches);

/*
 * Diagnostic, independent of any handle: a synthetic kernel that tells whether the fp32 matrix
 * instructions (v_mfma_f32_16x16x4_f32) and the ordinary vector instructions of one SIMD execute at the
 * same time on this device.  The bound of the LSTM kernels (Section 3.2 network at Table 1 sizes: gate
 * contraction on the matrix pipe, activations on the vector ALU of the same SIMD) depends on it.
 * Launches 256 x per_cu workgroups of four waves (per_cu = 1 or 2: workgroups that share a compute
 * unit); every wave runs `iterations` rounds of
 *   mode 0: 16 MFMAs;  mode 1: 64 vector FMAs;  mode 2: both, interleaved in every wave;
 *   mode 3 (per_cu = 2): workgroups of the first half MFMAs only, of the second half FMAs only.
 * The caller times the launch on `stream`.  If the two kinds overlapped, mode 2 would take the longer
 * of modes 0 and 1, not their sum.  out: device, 256 * per_cu * 256 floats, overwritten with values of
 * no meaning.  ESRNN_ERR_CONFIG for arguments outside these ranges (iterations 1 .. 1 << 20).
 */
esrnn_status esrnn_probe_issue_overlap(int32_t mode, int32_t iterations, int32_t per_cu, float *out, void *stream);

#ifdef __cplusplus
}
#endif
#endif
