// C ABI of the ES-RNN library (include/esrnn.h): handle management, argument
// checks and the order in which the kernels of one training step are enqueued.
#include <cstdio>
#include <new>

#include "esrnn_internal.h"

using namespace esrnn;

namespace {
constexpr int kMaxStages = 16 + 2 * kMaxLayers;
struct Stage {
    char name[32];
    hipEvent_t start, stop;
    bool recorded;
    double total_ms;
    int launches;
};
}  // namespace

struct esrnn_handle {
    Plan plan;
    bool forward_done;
    bool profiling;
    int n_stages;
    Stage stage[kMaxStages];
    // stage indices
    int st_setup, st_es_fwd, st_win_fwd, st_lstm_fwd[kMaxLayers], st_head, st_fc, st_loss;
    int st_lstm_bwd[kMaxLayers], st_win_bwd, st_es_bwd, st_reduce, st_tail;
    const int32_t *categories;   // device array of the caller, or null
    bool forward_only;           // esrnn_forward skips the reverse pass of the output stage; esrnn_backward is refused
};

namespace {
int add_stage(esrnn_handle *h, const char *fmt, int arg)
{
    Stage &s = h->stage[h->n_stages];
    snprintf(s.name, sizeof(s.name), fmt, arg);
    s.start = s.stop = nullptr;
    s.recorded = false;
    s.total_ms = 0.0;
    s.launches = 0;
    return h->n_stages++;
}

// Runs one stage; with profiling on, brackets it with events on the same stream.
template <class F>
hipError_t run_stage(esrnn_handle *h, int idx, hipStream_t st, F &&launch)
{
    if (!h->profiling) return launch();
    Stage &s = h->stage[idx];
    hipError_t e = hipEventRecord(s.start, st);
    if (e != hipSuccess) return e;
    e = launch();
    if (e != hipSuccess) return e;
    e = hipEventRecord(s.stop, st);
    s.recorded = true;
    return e;
}
}  // namespace

#define ESRNN_TRY(expr)                              \
    do {                                             \
        hipError_t e_ = (expr);                      \
        if (e_ != hipSuccess) return ESRNN_ERR_HIP;  \
    } while (0)

extern "C" {

esrnn_status esrnn_create(const esrnn_config *cfg, esrnn_handle **out)
{
    if (!cfg || !out) return ESRNN_ERR_NULL;
    *out = nullptr;
    esrnn_handle *h = new (std::nothrow) esrnn_handle;
    if (!h) return ESRNN_ERR_HIP;
    esrnn_status st = build_plan(*cfg, h->plan);
    if (st != ESRNN_OK) {
        delete h;
        return st;
    }
    h->forward_done = false;
    h->profiling = false;
    h->categories = nullptr;
    h->forward_only = false;
    h->n_stages = 0;
    const Plan &pl = h->plan;
    h->st_setup = add_stage(h, "setup", 0);
    h->st_es_fwd = add_stage(h, "es_forward", 0);
    h->st_win_fwd = add_stage(h, "window_forward", 0);
    for (int l = 0; l < pl.L; ++l) h->st_lstm_fwd[l] = add_stage(h, "lstm_forward_l%d", l);
    h->st_head = add_stage(h, "head_forward_backward", 0);
    h->st_fc = add_stage(h, "forecasts", 0);
    h->st_loss = add_stage(h, "loss_finalize", 0);
    for (int l = pl.L - 1; l >= 0; --l) h->st_lstm_bwd[l] = add_stage(h, "lstm_backward_l%d", l);
    h->st_win_bwd = add_stage(h, "window_backward", 0);
    h->st_es_bwd = add_stage(h, "es_backward", 0);
    h->st_reduce = add_stage(h, "reduce_weight_grads", 0);
    h->st_tail = add_stage(h, "forecast_tail", 0);
    *out = h;
    return ESRNN_OK;
}

esrnn_status esrnn_destroy(esrnn_handle *h)
{
    if (!h) return ESRNN_ERR_NULL;
    for (int i = 0; i < h->n_stages; ++i) {
        if (h->stage[i].start) (void)hipEventDestroy(h->stage[i].start);
        if (h->stage[i].stop) (void)hipEventDestroy(h->stage[i].stop);
    }
    delete h;
    return ESRNN_OK;
}

esrnn_status esrnn_set_categories(esrnn_handle *h, const int32_t *categories)
{
    if (!h) return ESRNN_ERR_NULL;
    if (h->plan.C == 0 && categories) return ESRNN_ERR_CONFIG;
    h->categories = categories;
    return ESRNN_OK;
}

esrnn_status esrnn_set_forward_only(esrnn_handle *h, int32_t on)
{
    if (!h) return ESRNN_ERR_NULL;
    h->forward_only = on != 0;
    h->forward_done = false;
    return ESRNN_OK;
}

esrnn_status esrnn_workspace_bytes(const esrnn_handle *h, size_t *bytes)
{
    if (!h || !bytes) return ESRNN_ERR_NULL;
    *bytes = h->plan.total_floats * sizeof(float);
    return ESRNN_OK;
}

esrnn_status esrnn_check_workspace(const esrnn_handle *h, const void *workspace, size_t bytes, int32_t es_window_only)
{
    if (!h || !workspace) return ESRNN_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return ESRNN_ERR_WORKSPACE;
    const size_t need = (es_window_only ? h->plan.es_window_floats : h->plan.total_floats) * sizeof(float);
    return bytes >= need ? ESRNN_OK : ESRNN_ERR_WORKSPACE;
}

esrnn_status esrnn_es_param_rows(const esrnn_handle *h, int32_t *K)
{
    if (!h || !K) return ESRNN_ERR_NULL;
    *K = h->plan.K;
    return ESRNN_OK;
}

esrnn_status esrnn_weight_count(const esrnn_handle *h, size_t *n)
{
    if (!h || !n) return ESRNN_ERR_NULL;
    *n = h->plan.n_weights;
    return ESRNN_OK;
}

const char *esrnn_status_string(esrnn_status s)
{
    switch (s) {
    case ESRNN_OK: return "ok";
    case ESRNN_ERR_NULL: return "null pointer argument";
    case ESRNN_ERR_CONFIG: return "unsupported configuration";
    case ESRNN_ERR_WORKSPACE: return "workspace pointer not 256-byte aligned, or built-in workspace too small";
    case ESRNN_ERR_ORDER: return "backward called without a preceding forward";
    case ESRNN_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

esrnn_status esrnn_forward(esrnn_handle *h, const float *y, const int32_t *lengths,
                           const float *es_params, const float *weights, void *workspace,
                           float *loss, float *forecasts, void *stream)
{
    if (!h || !y || !lengths || !es_params || !weights || !workspace || !loss) return ESRNN_ERR_NULL;
    if (h->plan.C > 0 && !h->categories) return ESRNN_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return ESRNN_ERR_WORKSPACE;
    const Plan &pl = h->plan;
    float *ws = static_cast<float *>(workspace);
    hipStream_t st = static_cast<hipStream_t>(stream);
    h->forward_done = false;
    ESRNN_TRY(run_stage(h, h->st_setup, st, [&] { return launch_setup(pl, lengths, weights, ws, st); }));
    ESRNN_TRY(run_stage(h, h->st_es_fwd, st, [&] { return launch_es_forward(pl, y, lengths, es_params, ws, st); }));
    ESRNN_TRY(run_stage(h, h->st_win_fwd, st, [&] { return launch_window_forward(pl, h->categories, ws, st); }));
    for (int l = 0; l < pl.L; ++l)
        ESRNN_TRY(run_stage(h, h->st_lstm_fwd[l], st, [&] { return launch_lstm_forward(pl, l, lengths, weights, ws, st); }));
    // the output stage runs its reverse pass in the same launch: the loss gradient needs nothing beyond it
    ESRNN_TRY(run_stage(h, h->st_head, st, [&] { return launch_head(pl, lengths, ws, !h->forward_only, st); }));
    if (forecasts)
        ESRNN_TRY(run_stage(h, h->st_fc, st, [&] { return launch_forecasts(pl, lengths, ws, forecasts, st); }));
    ESRNN_TRY(run_stage(h, h->st_loss, st, [&] { return launch_loss_finalize(pl, ws, loss, st); }));
    h->forward_done = !h->forward_only;
    return ESRNN_OK;
}

esrnn_status esrnn_backward(esrnn_handle *h, const float *y, const int32_t *lengths,
                            const float *es_params, const float *weights, void *workspace,
                            float *grad_es_params, float *grad_weights, void *stream)
{
    if (!h || !y || !lengths || !es_params || !weights || !workspace || !grad_es_params || !grad_weights)
        return ESRNN_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return ESRNN_ERR_WORKSPACE;
    if (!h->forward_done) return ESRNN_ERR_ORDER;
    const Plan &pl = h->plan;
    float *ws = static_cast<float *>(workspace);
    hipStream_t st = static_cast<hipStream_t>(stream);
    for (int l = pl.L - 1; l >= 0; --l)
        ESRNN_TRY(run_stage(h, h->st_lstm_bwd[l], st, [&] { return launch_lstm_backward(pl, l, lengths, ws, st); }));
    ESRNN_TRY(run_stage(h, h->st_win_bwd, st, [&] { return launch_window_backward(pl, lengths, ws, st); }));
    ESRNN_TRY(run_stage(h, h->st_es_bwd, st,
                        [&] { return launch_es_backward(pl, y, lengths, es_params, ws, grad_es_params, st); }));
    ESRNN_TRY(run_stage(h, h->st_reduce, st, [&] { return launch_reduce_weight_grads(pl, ws, grad_weights, st); }));
    return ESRNN_OK;
}

esrnn_status esrnn_adam_update(esrnn_handle *h, const esrnn_adam_config *opt, int32_t step,
                               float *weights, const float *grad_weights, float *m_weights, float *v_weights,
                               float *es_params, const float *grad_es_params, float *m_es, float *v_es,
                               void *workspace, void *stream)
{
    if (!h || !opt || !weights || !grad_weights || !m_weights || !v_weights || !es_params || !grad_es_params ||
        !m_es || !v_es || !workspace)
        return ESRNN_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return ESRNN_ERR_WORKSPACE;
    if (step < 1 || !(opt->beta1 >= 0.0f && opt->beta1 < 1.0f) || !(opt->beta2 >= 0.0f && opt->beta2 < 1.0f) ||
        !(opt->eps > 0.0f))
        return ESRNN_ERR_CONFIG;
    ESRNN_TRY(launch_adam_update(h->plan, *opt, step, weights, grad_weights, m_weights, v_weights, es_params,
                                 grad_es_params, m_es, v_es, static_cast<float *>(workspace),
                                 static_cast<hipStream_t>(stream)));
    h->forward_done = false;    // the parameters have changed: a new forward pass comes before the next backward
    return ESRNN_OK;
}

esrnn_status esrnn_gather_batch(esrnn_handle *h, const float *y_store, const int32_t *lengths_store,
                                const float *es_store, const int32_t *index, int32_t N,
                                float *y, int32_t *lengths, float *es_params, void *stream)
{
    if (!h || !y_store || !lengths_store || !es_store || !index || !y || !lengths || !es_params) return ESRNN_ERR_NULL;
    if (N < 1) return ESRNN_ERR_CONFIG;
    ESRNN_TRY(launch_gather_batch(h->plan, y_store, lengths_store, es_store, index, N, y, lengths, es_params,
                                  static_cast<hipStream_t>(stream)));
    return ESRNN_OK;
}

esrnn_status esrnn_adam_update_indexed(esrnn_handle *h, const esrnn_adam_config *opt, int32_t step,
                                       float *weights, const float *grad_weights, float *m_weights, float *v_weights,
                                       float *es_store, const float *grad_es_params, float *m_es_store,
                                       float *v_es_store, int32_t *counts_store, const int32_t *index, int32_t N,
                                       void *workspace, void *stream)
{
    if (!h || !opt || !weights || !grad_weights || !m_weights || !v_weights || !es_store || !grad_es_params ||
        !m_es_store || !v_es_store || !counts_store || !index || !workspace)
        return ESRNN_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return ESRNN_ERR_WORKSPACE;
    if (step < 1 || N < 1 || !(opt->beta1 >= 0.0f && opt->beta1 < 1.0f) || !(opt->beta2 >= 0.0f && opt->beta2 < 1.0f) ||
        !(opt->eps > 0.0f))
        return ESRNN_ERR_CONFIG;
    ESRNN_TRY(launch_adam_update_indexed(h->plan, *opt, step, weights, grad_weights, m_weights, v_weights, es_store,
                                         grad_es_params, m_es_store, v_es_store, counts_store, index, N,
                                         static_cast<float *>(workspace), static_cast<hipStream_t>(stream)));
    h->forward_done = false;
    return ESRNN_OK;
}

esrnn_status esrnn_predict(esrnn_handle *h, const float *y, const int32_t *lengths, const float *es_params,
                           const float *weights, void *workspace, float *forecasts, void *stream)
{
    if (!h || !y || !lengths || !es_params || !weights || !workspace || !forecasts) return ESRNN_ERR_NULL;
    if (h->plan.C > 0 && !h->categories) return ESRNN_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return ESRNN_ERR_WORKSPACE;
    const Plan &pl = h->plan;
    float *ws = static_cast<float *>(workspace);
    hipStream_t st = static_cast<hipStream_t>(stream);
    h->forward_done = false;    // the workspace now holds the state of the extended problem, not of a training pass
    const int32_t *ext = reinterpret_cast<const int32_t *>(ws + pl.len_ext);
    ESRNN_TRY(launch_extend_lengths(pl, lengths, ws, st));
    ESRNN_TRY(run_stage(h, h->st_setup, st, [&] { return launch_setup(pl, ext, weights, ws, st); }));
    ESRNN_TRY(run_stage(h, h->st_es_fwd, st, [&] { return launch_es_forward(pl, y, ext, es_params, ws, st); }));
    ESRNN_TRY(run_stage(h, h->st_win_fwd, st, [&] { return launch_window_forward(pl, h->categories, ws, st); }));
    for (int l = 0; l < pl.L; ++l)
        ESRNN_TRY(run_stage(h, h->st_lstm_fwd[l], st, [&] { return launch_lstm_forward(pl, l, ext, weights, ws, st); }));
    ESRNN_TRY(run_stage(h, h->st_head, st, [&] { return launch_head(pl, ext, ws, false, st); }));
    ESRNN_TRY(run_stage(h, h->st_tail, st, [&] { return launch_forecast_tail(pl, lengths, ws, forecasts, st); }));
    return ESRNN_OK;
}

esrnn_status esrnn_predict_static(esrnn_handle *h, const float *y, const int32_t *lengths, const float *es_params,
                                  const float *weights, float *forecasts, void *stream)
{
    if (!h || !y || !lengths || !es_params || !weights || !forecasts) return ESRNN_ERR_NULL;
    if (h->plan.total_floats * sizeof(float) > (size_t)ESRNN_STATIC_SCRATCH_BYTES) return ESRNN_ERR_WORKSPACE;
    void *ws = nullptr;
    size_t bytes = 0;
    ESRNN_TRY(static_scratch(&ws, &bytes));
    if (h->plan.total_floats * sizeof(float) > bytes) return ESRNN_ERR_WORKSPACE;
    return esrnn_predict(h, y, lengths, es_params, weights, ws, forecasts, stream);
}

esrnn_status esrnn_forecast_metrics(esrnn_handle *h, const float *forecasts, const float *actuals, const float *y,
                                    const int32_t *lengths, int32_t m, float *smape, float *mase, void *stream)
{
    if (!h || !forecasts || !actuals || !y || !lengths || !smape || !mase) return ESRNN_ERR_NULL;
    if (m < 1 || m >= h->plan.T) return ESRNN_ERR_CONFIG;
    ESRNN_TRY(launch_forecast_metrics(h->plan, forecasts, actuals, y, lengths, m, smape, mase,
                                      static_cast<hipStream_t>(stream)));
    return ESRNN_OK;
}

esrnn_status esrnn_es_window_workspace_bytes(const esrnn_handle *h, size_t *bytes)
{
    if (!h || !bytes) return ESRNN_ERR_NULL;
    *bytes = h->plan.es_window_floats * sizeof(float);
    return ESRNN_OK;
}

esrnn_status esrnn_es_window_forward(esrnn_handle *h, const float *y, const int32_t *lengths,
                                     const float *es_params, void *workspace, void *stream)
{
    if (!h || !y || !lengths || !es_params || !workspace) return ESRNN_ERR_NULL;
    if (h->plan.C > 0 && !h->categories) return ESRNN_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return ESRNN_ERR_WORKSPACE;
    const Plan &pl = h->plan;
    float *ws = static_cast<float *>(workspace);
    hipStream_t st = static_cast<hipStream_t>(stream);
    ESRNN_TRY(run_stage(h, h->st_setup, st, [&] { return launch_setup(pl, lengths, nullptr, ws, st); }));
    ESRNN_TRY(run_stage(h, h->st_es_fwd, st, [&] { return launch_es_forward(pl, y, lengths, es_params, ws, st); }));
    ESRNN_TRY(run_stage(h, h->st_win_fwd, st, [&] { return launch_window_forward(pl, h->categories, ws, st); }));
    return ESRNN_OK;
}

esrnn_status esrnn_es_window_backward(esrnn_handle *h, const float *y, const int32_t *lengths,
                                      const float *es_params, void *workspace, float *grad_es_params, void *stream)
{
    if (!h || !y || !lengths || !es_params || !workspace || !grad_es_params) return ESRNN_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return ESRNN_ERR_WORKSPACE;
    const Plan &pl = h->plan;
    float *ws = static_cast<float *>(workspace);
    hipStream_t st = static_cast<hipStream_t>(stream);
    ESRNN_TRY(run_stage(h, h->st_win_bwd, st, [&] { return launch_window_backward(pl, lengths, ws, st); }));
    ESRNN_TRY(run_stage(h, h->st_es_bwd, st,
                        [&] { return launch_es_backward(pl, y, lengths, es_params, ws, grad_es_params, st); }));
    return ESRNN_OK;
}

esrnn_status esrnn_profile_enable(esrnn_handle *h, int32_t on)
{
    if (!h) return ESRNN_ERR_NULL;
    if (on) {
        for (int i = 0; i < h->n_stages; ++i) {
            Stage &s = h->stage[i];
            if (!s.start) ESRNN_TRY(hipEventCreate(&s.start));
            if (!s.stop) ESRNN_TRY(hipEventCreate(&s.stop));
            s.recorded = false;
            s.total_ms = 0.0;
            s.launches = 0;
        }
    }
    h->profiling = on != 0;
    return ESRNN_OK;
}

esrnn_status esrnn_profile_stage_count(const esrnn_handle *h, int32_t *n)
{
    if (!h || !n) return ESRNN_ERR_NULL;
    *n = h->n_stages;
    return ESRNN_OK;
}

esrnn_status esrnn_profile_stage_name(const esrnn_handle *h, int32_t i, const char **name)
{
    if (!h || !name) return ESRNN_ERR_NULL;
    if (i < 0 || i >= h->n_stages) return ESRNN_ERR_CONFIG;
    *name = h->stage[i].name;
    return ESRNN_OK;
}

esrnn_status esrnn_profile_collect(esrnn_handle *h)
{
    if (!h) return ESRNN_ERR_NULL;
    for (int i = 0; i < h->n_stages; ++i) {
        Stage &s = h->stage[i];
        if (!s.recorded) continue;
        ESRNN_TRY(hipEventSynchronize(s.stop));
        float ms = 0.0f;
        ESRNN_TRY(hipEventElapsedTime(&ms, s.start, s.stop));
        s.total_ms += ms;
        s.launches += 1;
        s.recorded = false;
    }
    return ESRNN_OK;
}

esrnn_status esrnn_profile_read(const esrnn_handle *h, double *total_ms, int32_t *launches)
{
    if (!h || !total_ms || !launches) return ESRNN_ERR_NULL;
    for (int i = 0; i < h->n_stages; ++i) {
        total_ms[i] = h->stage[i].total_ms;
        launches[i] = h->stage[i].launches;
    }
    return ESRNN_OK;
}

esrnn_status esrnn_probe_issue_overlap(int32_t mode, int32_t iterations, int32_t per_cu, float *out, void *stream)
{
    if (!out) return ESRNN_ERR_NULL;
    if (mode < 0 || mode > 3 || per_cu < 1 || per_cu > 2 || (mode == 3 && per_cu != 2) || iterations < 1 ||
        iterations > (1 << 20))
        return ESRNN_ERR_CONFIG;
    return esrnn::launch_probe_issue_overlap(mode, iterations, per_cu, out, static_cast<hipStream_t>(stream)) == hipSuccess
               ? ESRNN_OK : ESRNN_ERR_HIP;
}

esrnn_status esrnn_workspace_buffer(const esrnn_handle *h, int32_t which, int32_t index, esrnn_buffer_view *out)
{
    if (!h || !out) return ESRNN_ERR_NULL;
    const Plan &pl = h->plan;
    size_t off = 0;
    int layout = ESRNN_LAYOUT_TILE, rows = 0, logical = 0, lead = pl.P;
    auto layer_ok = [&](int i) { return i >= 0 && i < pl.L; };
    switch (which) {
    case ESRNN_BUF_LEVEL: off = pl.lvl; layout = ESRNN_LAYOUT_TIME_MAJOR; break;
    case ESRNN_BUF_S1: off = pl.S1; layout = ESRNN_LAYOUT_TIME_MAJOR; break;
    case ESRNN_BUF_S2: off = pl.S2; layout = ESRNN_LAYOUT_TIME_MAJOR; break;
    case ESRNN_BUF_U: off = pl.u; layout = ESRNN_LAYOUT_TIME_MAJOR; break;
    case ESRNN_BUF_V: off = pl.v; layout = ESRNN_LAYOUT_TIME_MAJOR; break;
    case ESRNN_BUF_GRAD_U: off = pl.gu; layout = ESRNN_LAYOUT_TIME_MAJOR; break;
    case ESRNN_BUF_GRAD_V: off = pl.gv; layout = ESRNN_LAYOUT_TIME_MAJOR; break;
    case ESRNN_BUF_X: off = pl.X; rows = 4 * pl.IT; logical = pl.I + pl.C; break;
    case ESRNN_BUF_GRAD_X: off = pl.gX; rows = 4 * pl.IT; logical = pl.I + pl.C; break;
    case ESRNN_BUF_Z: off = pl.Z; rows = pl.OP; logical = pl.H; break;
    case ESRNN_BUF_O: off = pl.O; rows = pl.OP; logical = pl.H; break;
    case ESRNN_BUF_GRAD_O: off = pl.gO; rows = pl.OP; logical = pl.H; break;
    case ESRNN_BUF_GRAD_TOP: off = pl.gTop; rows = pl.HP; logical = pl.h; break;
    case ESRNN_BUF_GATES:
        if (!layer_ok(index)) return ESRNN_ERR_CONFIG;
        off = pl.layer[index].gates; layout = ESRNN_LAYOUT_GATE_TILE; rows = pl.HP; logical = pl.h; break;
    case ESRNN_BUF_C:
        if (!layer_ok(index)) return ESRNN_ERR_CONFIG;
        off = pl.layer[index].c; rows = pl.HP; logical = pl.h; break;
    case ESRNN_BUF_HID:
        if (!layer_ok(index)) return ESRNN_ERR_CONFIG;
        off = pl.layer[index].hid; rows = pl.HP; logical = pl.h; break;
    case ESRNN_BUF_BLOCK_OUT:
        if (index < 0 || index >= pl.cfg.n_blocks) return ESRNN_ERR_CONFIG;
        off = pl.blk_out[index]; rows = pl.HP; logical = pl.h; break;
    default: return ESRNN_ERR_CONFIG;
    }
    if (layout == ESRNN_LAYOUT_TIME_MAJOR) { lead = pl.T; rows = 1; logical = 1; }
    out->offset_bytes = off * sizeof(float);
    out->layout = layout;
    out->dims[0] = lead;
    out->dims[1] = layout == ESRNN_LAYOUT_TIME_MAJOR ? pl.Bt : pl.Bp;
    out->dims[2] = rows;
    out->dims[3] = logical;
    return ESRNN_OK;
}

}  // extern "C"
