// Internal declarations of the ES-RNN HIP library: launch plan, workspace map
// and kernel launchers.  Not part of the public ABI (see include/esrnn.h).
#pragma once

#include <hip/hip_runtime.h>
#include <algorithm>
#include <cmath>
#include <stddef.h>
#include <stdint.h>

#include "esrnn.h"

namespace esrnn {

constexpr int kTileN = 16;       // series per tile (N of the 16x16x4 fp32 MFMA)
constexpr int kMaxLayers = ESRNN_MAX_BLOCKS * ESRNN_MAX_LAYERS_PER_BLOCK;
constexpr int kLstmWaves = 4;    // waves per workgroup in the LSTM kernels
constexpr int kSinkLines = 256;  // 256-byte lines of the store sink
constexpr int kSplitBwdFromHT = 13;   // hidden unit tiles from which the 16-series reverse kernel always puts the weight gradient on waves of its own
constexpr int kReduceSplits = 16; // subsets of producers in the first stage of the weight-gradient reduction
// Row stride of the LDS arrays [row][16 series] that are read transposed (lane = row n, column 4k + g).  With 18
// the 32 lanes of a half wave (16 rows x 2 columns) hit 32 different banks: (18 n + g) mod 32 takes every value
// once.  (17, the usual odd padding, leaves one two-way conflict in every such read.)
constexpr int kLdsPad = 18;
constexpr int kNarrowSeries = 4; // series per workgroup in the small-batch LSTM kernels

// Tile layout TL(R): [P][NB][R][16]; element (p, b, r) at ((p*NB + b/16)*R + r)*16 + b%16.
// A "unit tile" is 4 consecutive rows (64 floats = one float per lane).

struct LayerPlan {
    int dil, block, first_in_block, last_in_block;
    int in_dim;          // logical width of the layer input
    int KXT;             // unit tiles of the layer input (x part of the contraction)
    size_t w_off, b_off; // offsets into the caller's flat weight vector
    // forward operands (offsets in floats into the workspace)
    size_t wpack_fwd;    // [HT][KXT+HT][64]  A operands of the gate contraction
    size_t bias_pack;    // [HT][4][4]        bias of (unit tile, unit, gate)
    size_t xsrc;         // TL(4*KXT) input
    size_t gates, c, hid;
    size_t resid, out;   // out = resid + hid for the last layer of a block >= 1 (0 = none)
    // backward operands
    size_t wpack_bwd;    // [MB][4*HT][64]    A operands of the transposed contraction
    size_t gsrc[4];      // TL(HP): the gradient arriving at this layer's hidden output is the sum of these
    int n_gsrc;
    size_t gdst;         // TL(4*KXT) gradient with respect to the layer input
    int chains;          // workgroups per series tile (per 4 series if narrow); each walks the residue classes r, r+chains, ... (mod dil)
    int chains_bwd;      // the same for the reverse kernel
    int split_bwd;       // 1: reverse kernel with eight waves, the weight gradient on waves of its own, one workgroup per compute unit
    int narrow;          // 1: the layer runs on the 4-series kernels (lstm_narrow_fwd.h, lstm_narrow_bwd.h): wpack_fwd is
                         // [4][4*(KXT+HT)][64], wpack_bwd [4][NG][4*HT][64], bias_pack unused, and the
                         // weight-gradient partials are indexed by 4*NB*chains workgroups
    size_t dw_partial;   // [NB*chains][HT*MB][4][64] per-workgroup weight-gradient tiles
    size_t db_partial;   // [NB*chains][HT][4][4]
    size_t dw_reduced, db_reduced;   // [kReduceSplits][...] first reduction stage
    size_t cs_partial;   // [NB*chains] sums of squared cell states (first layer of a block, penalty on)
};

struct Plan {
    esrnn_config cfg;
    int B, T, I, H, h, P;
    int C;               // entries of the category one-hot block that follows the input window (0: none)
    int NB, Bp;          // series tiles, padded batch (16 * NB)
    int Bt;              // row stride of the time-major arrays: the batch padded to whole waves of 64 series
    int HT, HP;          // hidden unit tiles, padded hidden (4*HT)
    int IT;              // unit tiles of the network input (window + one-hot block) as used by layer 0
    int OT, MO, OP;      // horizon: unit tiles, 16-row MFMA tiles, rows of the Z / O / gO tiles (4*OT)
    int MA;              // 16-row tiles of the hidden dimension in "unit-tile" order: ceil(HT/4)
    int window_stream;   // window adjoint: 1 = streaming kernel (many series tiles), 0 = gather kernel
    int L;
    int K;               // rows of es_params
    int row_gamma1, row_gamma2, row_s1, row_s2;
    LayerPlan layer[kMaxLayers];
    size_t Wa_off, ba_off, Wo_off, bo_off, n_weights;
    // workspace map (offsets in floats)
    size_t scalars;      // float[16]: see Scalars
    size_t sink;         // float[kSinkLines][64]: target of stores whose value nothing reads (a workgroup uses line id % kSinkLines)
    size_t len_ext;      // int32[B]: lengths extended by the horizon (out-of-sample forecasts)
    size_t pmax;         // int32[NB]: window positions the series of a 16-series tile need (max over the tile), by setup
    size_t opt_partial;  // float[512]: sums of squares of the gradients, per workgroup (parameter update)
    size_t lvl, S1, S2, u, v, gu, gv;   // [T][Bt]
    size_t X, Z;         // TL(4*IT), TL(OP)
    size_t blk_out[ESRNN_MAX_BLOCKS];
    size_t O, gO, gTop, gX;
    size_t dx[kMaxLayers];              // gradient with respect to the input of layer l (layer 0: gX)
    size_t gsum;                        // TL(HP) sum of gradient sources (three or more blocks only)
    size_t head_fwd_pack, head_bwd_pack; // packed head operands
    size_t loss_partial; int n_loss_partial;   // [head_blocks] pinball sums, then [es_blocks] level-penalty sums
    size_t cs_partial; int n_cs_partial;       // sums of squared cell states of all penalised layers, contiguous
    int head_blocks;                           // workgroups of the output-stage kernel
    size_t head_dw_partial; int n_head_waves;  // [n_head_waves][head_dw_stride]; 4 waves per workgroup
    int head_dw_stride;
    size_t head_dw_reduced;
    int es_blocks;
    int partial_groups(const LayerPlan &lp) const { return (lp.narrow ? 4 * NB : NB) * lp.chains_bwd; }   // producers of weight-gradient partials
    int forward_groups(const LayerPlan &lp) const { return (lp.narrow ? 4 * NB : NB) * lp.chains; }        // workgroups of the forward kernel
    size_t es_window_floats;   // prefix of the workspace used by the smoothing and window stages alone
    size_t total_floats;
};

// device-side scalars computed from lengths
struct Scalars {
    float inv_n_pin;   // 1 / number of unmasked head outputs
    float inv_n_lv;    // 1 / number of second differences of the log level (0 if none)
    float inv_n_cs;    // 1 / number of cell-state values in the cell-state penalty (0 if none)
};

// offsets inside the packed head operand blocks (floats), filled by plan.cpp
struct HeadPack {
    // forward: Wa as A operand in unit-tile order [MA][HT][64], ba [MA][4][4],
    //          Wo as A operand in unit-tile order [MO][HT][64], bo [MO][4][4]
    size_t WaF, baF, WoF, boF, fwd_total;
    // backward: Wo^T [MA][OT][64], Wa^T [MA][HT][64]
    size_t WoT, WaT, bwd_total;
};
HeadPack head_pack_layout(const Plan &pl);
hipError_t launch_probe_issue_overlap(int mode, int iterations, int per_cu, float *out, hipStream_t st);

esrnn_status build_plan(const esrnn_config &cfg, Plan &pl);

// ---- kernel launchers (each returns hipGetLastError()) -----------------------------------
hipError_t launch_setup(const Plan &pl, const int32_t *lengths, const float *weights, float *ws, hipStream_t st);
hipError_t launch_es_forward(const Plan &pl, const float *y, const int32_t *lengths, const float *es,
                             float *ws, hipStream_t st);
hipError_t launch_window_forward(const Plan &pl, const int32_t *categories, float *ws, hipStream_t st);
hipError_t launch_lstm_forward(const Plan &pl, int layer, const int32_t *lengths, const float *weights, float *ws,
                               hipStream_t st);
// 4-series kernels for layers with few workgroups (called by the two launchers above and below)
hipError_t launch_lstm_forward_narrow(const Plan &pl, int layer, const int32_t *lengths, const float *weights,
                                      float *ws, hipStream_t st);
hipError_t launch_lstm_forward_narrow_residual(const Plan &pl, int layer, const int32_t *lengths, const float *weights,
                                      float *ws, hipStream_t st);
hipError_t launch_lstm_backward_narrow(const Plan &pl, int layer, const int32_t *lengths, float *ws, hipStream_t st);
hipError_t launch_lstm_backward_narrow_split(const Plan &pl, int layer, const int32_t *lengths, float *ws, hipStream_t st);
// output stage, forward and reverse in one launch (needs the loss normalisers of launch_setup)
hipError_t launch_head(const Plan &pl, const int32_t *lengths, float *ws, bool reverse, hipStream_t st);
hipError_t launch_forecasts(const Plan &pl, const int32_t *lengths, float *ws, float *forecasts, hipStream_t st);
hipError_t launch_loss_finalize(const Plan &pl, float *ws, float *loss, hipStream_t st);

hipError_t launch_lstm_backward(const Plan &pl, int layer, const int32_t *lengths, float *ws, hipStream_t st);
hipError_t launch_window_backward(const Plan &pl, const int32_t *lengths, float *ws, hipStream_t st);
hipError_t launch_es_backward(const Plan &pl, const float *y, const int32_t *lengths, const float *es,
                              float *ws, float *grad_es, hipStream_t st);
hipError_t launch_reduce_weight_grads(const Plan &pl, float *ws, float *grad_weights, hipStream_t st);

hipError_t launch_adam_update(const Plan &pl, const esrnn_adam_config &opt, int step, float *weights,
                              const float *grad_weights, float *m_w, float *v_w, float *es_params,
                              const float *grad_es, float *m_es, float *v_es, float *ws, hipStream_t st);
hipError_t launch_gather_batch(const Plan &pl, const float *store_y, const int32_t *store_len, const float *store_es,
                               const int32_t *index, int N, float *y, int32_t *len, float *es, hipStream_t st);
hipError_t launch_adam_update_indexed(const Plan &pl, const esrnn_adam_config &opt, int step, float *weights,
                                      const float *grad_weights, float *m_w, float *v_w, float *es_store,
                                      const float *grad_es, float *m_es, float *v_es, int32_t *counts,
                                      const int32_t *index, int N, float *ws, hipStream_t st);
hipError_t launch_extend_lengths(const Plan &pl, const int32_t *lengths, float *ws, hipStream_t st);
hipError_t launch_forecast_tail(const Plan &pl, const int32_t *lengths, float *ws, float *out, hipStream_t st);
hipError_t launch_forecast_metrics(const Plan &pl, const float *forecasts, const float *actuals, const float *y,
                                   const int32_t *lengths, int m, float *smape, float *mase, hipStream_t st);

// Device address and size of the library's own scratch array on the current device (static_scratch.hip).
hipError_t static_scratch(void **ptr, size_t *bytes);

// Supported (HT, KXT) instantiations of the LSTM kernels.
bool lstm_shape_supported(int HT, int KXT);

}  // namespace esrnn
