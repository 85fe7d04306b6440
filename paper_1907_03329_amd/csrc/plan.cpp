// Host-side launch plan: validates a configuration, lays out the workspace and
// the packed operand blocks.  No device work happens here.
#include <algorithm>
#include <cstdlib>
#include <cstring>

#include "esrnn_internal.h"

namespace esrnn {

namespace {

struct Bump {
    size_t at = 0;
    size_t take(size_t n_floats)
    {
        size_t r = at;
        at += (n_floats + 63) & ~size_t(63);   // keep every block 256-byte aligned
        return r;
    }
};

int ceil_div(int a, int b) { return (a + b - 1) / b; }

constexpr int kNarrowBelowDefault = 160;
// Series tiles from which the window adjoint streams (one wave per tile) instead of gathering (one thread per
// time step and series).  Measured on the quarterly shape: gather 0.026 / 0.118 / 0.476 ms at 1024 / 4096 /
// 16384 tiles, streaming 0.053 / 0.079 / 0.25 ms; a wave of the streaming kernel is a chain of dependent memory
// round trips and needs about sixteen waves per SIMD to hide them.
constexpr int kWindowStreamFromDefault = 4096;

// hidden sizes are padded to one of the instantiated unit-tile counts
int pick_ht(int hidden)
{
    const int need = ceil_div(hidden, 4);
    const int avail[] = {2, 8, 10, 13, 16};
    for (int v : avail)
        if (need <= v) return v;
    return -1;
}

}  // namespace

bool lstm_shape_supported(int HT, int KXT)
{
    static const int pairs[][2] = {{2, 1}, {2, 2}, {8, 2}, {8, 3}, {8, 8}, {10, 1}, {10, 3}, {10, 6}, {10, 8}, {10, 10},
                                   {13, 3}, {13, 5}, {13, 13}, {16, 16}};
    for (auto &p : pairs)
        if (p[0] == HT && p[1] == KXT) return true;
    return false;
}

HeadPack head_pack_layout(const Plan &pl)
{
    HeadPack hp{};
    Bump b;
    hp.WaF = b.take((size_t)pl.MA * pl.HT * 64);
    hp.baF = b.take((size_t)pl.MA * 16);
    hp.WoF = b.take((size_t)pl.MO * pl.HT * 64);
    hp.boF = b.take((size_t)pl.MO * 16);
    hp.fwd_total = b.at;
    Bump c;
    hp.WoT = c.take((size_t)pl.MA * pl.OT * 64);
    hp.WaT = c.take((size_t)pl.MA * pl.HT * 64);
    hp.bwd_total = c.at;
    return hp;
}

esrnn_status build_plan(const esrnn_config &cfg, Plan &pl)
{
    std::memset(&pl, 0, sizeof(pl));
    // Layers whose 16-series grid has fewer workgroups than this run on the 4-series kernels.
    // ESRNN_NARROW_BELOW overrides the threshold (0: never, a large number: always), for measurements.
    int narrow_below = kNarrowBelowDefault;
    if (const char *env = std::getenv("ESRNN_NARROW_BELOW")) narrow_below = std::atoi(env);
    // The window adjoint streams tile by tile from this many series tiles on (one wave per tile needs enough
    // tiles to hide memory latency); ESRNN_WINDOW_STREAM_FROM overrides, for measurements.
    int window_stream_from = kWindowStreamFromDefault;
    if (const char *env = std::getenv("ESRNN_WINDOW_STREAM_FROM")) window_stream_from = std::atoi(env);
    pl.cfg = cfg;
    if (cfg.B < 1 || cfg.T < 1 || cfg.I < 1 || cfg.H < 1 || cfg.hidden < 1) return ESRNN_ERR_CONFIG;
    if (cfg.hidden > ESRNN_MAX_HIDDEN || cfg.I > ESRNN_MAX_WINDOW || cfg.H > ESRNN_MAX_WINDOW) return ESRNN_ERR_CONFIG;
    if (cfg.n_seas < 0 || cfg.n_seas > 2) return ESRNN_ERR_CONFIG;
    if (cfg.n_seas >= 1 && (cfg.m1 < 1 || cfg.m1 > cfg.T)) return ESRNN_ERR_CONFIG;
    if (cfg.n_seas >= 2 && (cfg.m2 < 1 || cfg.m2 > cfg.T)) return ESRNN_ERR_CONFIG;
    // the smoothing kernels keep the seasonal rings of 64 series in LDS: (m1 + m2) * 64 floats, which with the
    // 48 KB staging buffer of the reverse recursion must fit into 160 KB
    if ((long long)(cfg.n_seas >= 1 ? cfg.m1 : 0) + (cfg.n_seas >= 2 ? cfg.m2 : 0) > 448) return ESRNN_ERR_CONFIG;
    if ((long long)cfg.I + cfg.H > cfg.T) return ESRNN_ERR_CONFIG;
    if (cfg.n_blocks < 1 || cfg.n_blocks > ESRNN_MAX_BLOCKS) return ESRNN_ERR_CONFIG;
    if (!(cfg.tau > 0.0f && cfg.tau < 1.0f)) return ESRNN_ERR_CONFIG;
    if (!(cfg.lambda_lv >= 0.0f)) return ESRNN_ERR_CONFIG;
    if (!(cfg.lambda_cs >= 0.0f)) return ESRNN_ERR_CONFIG;
    if (cfg.param_space != ESRNN_PARAMS_DIRECT && cfg.param_space != ESRNN_PARAMS_LOGIT) return ESRNN_ERR_CONFIG;
    if ((long long)cfg.B * cfg.T > (1LL << 30)) return ESRNN_ERR_CONFIG;
    if (cfg.n_categories < 0 || cfg.n_categories > ESRNN_MAX_CATEGORIES) return ESRNN_ERR_CONFIG;
    if (cfg.I + cfg.n_categories > ESRNN_MAX_WINDOW) return ESRNN_ERR_CONFIG;

    pl.B = cfg.B; pl.T = cfg.T; pl.I = cfg.I; pl.H = cfg.H; pl.h = cfg.hidden; pl.C = cfg.n_categories;
    pl.P = cfg.T - cfg.I - cfg.H + 1;
    pl.NB = ceil_div(cfg.B, kTileN);
    pl.window_stream = pl.NB >= window_stream_from ? 1 : 0;
    pl.Bp = pl.NB * kTileN;
    pl.Bt = ceil_div(cfg.B, 64) * 64;
    pl.HT = pick_ht(cfg.hidden);
    if (pl.HT < 0) return ESRNN_ERR_CONFIG;
    pl.HP = 4 * pl.HT;
    pl.OT = ceil_div(cfg.H, 4);
    pl.MO = ceil_div(cfg.H, 16);
    pl.OP = 4 * pl.OT;
    pl.MA = ceil_div(pl.HT, 4);
    // layer 0 input tiles: exact if that kernel shape is instantiated, else padded to HT
    pl.IT = ceil_div(cfg.I + pl.C, 4);
    if (!lstm_shape_supported(pl.HT, pl.IT)) {
        if (cfg.I + pl.C > pl.HP) return ESRNN_ERR_CONFIG;
        pl.IT = pl.HT;
    }

    int r = 1;
    pl.row_gamma1 = pl.row_gamma2 = pl.row_s1 = pl.row_s2 = -1;
    if (cfg.n_seas >= 1) pl.row_gamma1 = r++;
    if (cfg.n_seas >= 2) pl.row_gamma2 = r++;
    if (cfg.n_seas >= 1) { pl.row_s1 = r; r += cfg.m1; }
    if (cfg.n_seas >= 2) { pl.row_s2 = r; r += cfg.m2; }
    pl.K = r;

    // user weight offsets
    size_t off = 0;
    int L = 0;
    const int h = cfg.hidden;
    for (int k = 0; k < cfg.n_blocks; ++k) {
        const int nl = cfg.layers_in_block[k];
        if (nl < 1 || nl > ESRNN_MAX_LAYERS_PER_BLOCK) return ESRNN_ERR_CONFIG;
        for (int j = 0; j < nl; ++j) {
            LayerPlan &lp = pl.layer[L];
            lp.dil = cfg.dilation[k][j];
            if (lp.dil < 1) return ESRNN_ERR_CONFIG;
            lp.block = k;
            lp.first_in_block = (j == 0);
            lp.last_in_block = (j == nl - 1);
            lp.in_dim = (L == 0) ? cfg.I + pl.C : h;
            lp.KXT = (L == 0) ? pl.IT : pl.HT;
            lp.w_off = off; off += (size_t)4 * h * (lp.in_dim + h);
            lp.b_off = off; off += (size_t)4 * h;
            ++L;
        }
    }
    pl.L = L;
    pl.Wa_off = off; off += (size_t)h * h;
    pl.ba_off = off; off += h;
    pl.Wo_off = off; off += (size_t)cfg.H * h;
    pl.bo_off = off; off += cfg.H;
    pl.n_weights = off;

    // workspace
    Bump ws;
    const size_t TB = (size_t)pl.T * pl.Bt;
    const size_t PN = (size_t)pl.P * pl.NB;
    const size_t tileH = (size_t)pl.HT * 64;         // floats of one (p, series-tile) block with HP rows
    // output stage: every wave leaves a block of weight-gradient partials, so no more waves than fill the chip
    const size_t n_tiles = PN;
    const int head_blocks = (int)std::min<size_t>((n_tiles + 3) / 4, 256);
    pl.head_blocks = head_blocks;
    pl.n_head_waves = 4 * head_blocks;
    pl.es_blocks = pl.Bt / 64;
    // first everything the smoothing and window stages touch (their own entry points need only this prefix)
    pl.scalars = ws.take(64);
    pl.sink = ws.take(64 * kSinkLines);
    pl.len_ext = ws.take((size_t)pl.B);
    pl.pmax = ws.take((size_t)pl.NB);
    pl.opt_partial = ws.take(512);
    pl.n_loss_partial = head_blocks + pl.es_blocks;
    pl.loss_partial = ws.take((size_t)pl.n_loss_partial);
    pl.lvl = ws.take(TB); pl.S1 = ws.take(TB); pl.S2 = ws.take(TB);
    pl.u = ws.take(TB); pl.v = ws.take(TB); pl.gu = ws.take(TB); pl.gv = ws.take(TB);
    pl.X = ws.take(PN * (size_t)pl.IT * 64);
    pl.Z = ws.take(PN * (size_t)pl.OP * 16);
    pl.gX = ws.take(PN * (size_t)pl.IT * 64);
    pl.gO = ws.take(PN * (size_t)pl.OP * 16);
    pl.es_window_floats = ws.at;
    pl.O = ws.take(PN * (size_t)pl.OP * 16);
    pl.gTop = ws.take(PN * tileH);
    for (int l = 0; l < L; ++l) {
        LayerPlan &lp = pl.layer[l];
        const int KT = lp.KXT + pl.HT;
        const int MB = ceil_div(KT, 4);
        // Few workgroups (small batch, small dilation): four series per workgroup instead of sixteen.
        // `narrow_below`: use the 4-series kernels when the 16-series grid would have fewer workgroups.
        const int wide_chains = std::min(std::min(lp.dil, pl.P), std::max(1, ceil_div(512, pl.NB)));
        lp.narrow = pl.NB * wide_chains < narrow_below ? 1 : 0;
        const int groups = lp.narrow ? 4 * pl.NB : pl.NB;
        // enough workgroups to put several on every compute unit, without more
        // weight-gradient partials than the reduction can read cheaply
        const int max_chains = std::max(1, ceil_div(512, groups));
        lp.chains = std::min(std::min(lp.dil, pl.P), max_chains);
        // Reverse kernels with eight waves, the weight gradient on waves of its own: one workgroup per compute
        // unit.  The faster kind where the grid has at most one workgroup per compute unit anyway, and for the
        // 16-series kernel with the larger hidden sizes (whose four-wave workgroup would be alone on its
        // compute unit for its registers).
        const bool one_per_cu = groups * lp.chains <= 256;
        lp.split_bwd = (one_per_cu || (!lp.narrow && pl.HT >= kSplitBwdFromHT)) ? 1 : 0;
        lp.chains_bwd = (lp.split_bwd && !lp.narrow) ? std::min(std::min(lp.dil, pl.P), std::max(1, ceil_div(256, groups)))
                                                      : lp.chains;
        if (lp.narrow) {
            const int KT4 = 4 * KT, NG = ceil_div(KT4, 64);
            lp.wpack_fwd = ws.take((size_t)4 * KT4 * 64);
            lp.bias_pack = lp.wpack_fwd;                       // unused: the kernels read the caller's bias
            lp.wpack_bwd = ws.take((size_t)4 * NG * 4 * pl.HT * 64);
        } else {
            lp.wpack_fwd = ws.take((size_t)pl.HT * KT * 64);
            lp.bias_pack = ws.take((size_t)pl.HT * 16);
            lp.wpack_bwd = ws.take((size_t)MB * 4 * pl.HT * 64);
        }
        lp.gates = ws.take(PN * tileH * 4);
        lp.c = ws.take(PN * tileH);
        lp.hid = ws.take(PN * tileH);
        lp.dw_partial = ws.take((size_t)groups * lp.chains_bwd * pl.HT * MB * 256);
        lp.db_partial = ws.take((size_t)groups * lp.chains_bwd * pl.HT * 16);
        lp.dw_reduced = ws.take((size_t)kReduceSplits * pl.HT * MB * 256);
        lp.db_reduced = ws.take((size_t)kReduceSplits * pl.HT * 16);
        pl.dx[l] = l > 0 ? ws.take(PN * tileH) : pl.gX;
    }
    // cell-state penalty: one partial sum per forward workgroup of every block's first layer, contiguous
    pl.cs_partial = ws.at;
    pl.n_cs_partial = 0;
    if (cfg.lambda_cs != 0.0f)
        for (int l = 0; l < L; ++l) {
            LayerPlan &lp = pl.layer[l];
            if (!lp.first_in_block) continue;
            lp.cs_partial = pl.cs_partial + pl.n_cs_partial;
            pl.n_cs_partial += pl.forward_groups(lp);
        }
    ws.take((size_t)pl.n_cs_partial);
    // block outputs: block 0's is the hidden state of its last layer
    for (int l = 0; l < L; ++l) {
        LayerPlan &lp = pl.layer[l];
        if (lp.last_in_block) {
            if (lp.block == 0) pl.blk_out[0] = lp.hid;
            else pl.blk_out[lp.block] = ws.take(PN * tileH);
        }
    }
    for (int l = 0; l < L; ++l) {
        LayerPlan &lp = pl.layer[l];
        // forward wiring
        if (l == 0) lp.xsrc = pl.X;
        else if (lp.first_in_block) lp.xsrc = pl.blk_out[lp.block - 1];
        else lp.xsrc = pl.layer[l - 1].hid;
        if (lp.last_in_block && lp.block >= 1) { lp.resid = pl.blk_out[lp.block - 1]; lp.out = pl.blk_out[lp.block]; }
        // backward wiring.  The output of block k feeds the first layer of every
        // later block through the residual sums, and the head: the gradient
        // arriving at its last layer is the sum of those input gradients.
        lp.gdst = pl.dx[l];
        lp.n_gsrc = 0;
        if (lp.last_in_block) {
            lp.gsrc[lp.n_gsrc++] = pl.gTop;
            for (int m = l + 1; m < L; ++m)
                if (pl.layer[m].first_in_block) lp.gsrc[lp.n_gsrc++] = pl.dx[m];
        } else {
            lp.gsrc[lp.n_gsrc++] = pl.dx[l + 1];
        }
    }
    if (cfg.n_blocks >= 3) pl.gsum = ws.take(PN * tileH);
    const HeadPack hp = head_pack_layout(pl);
    pl.head_fwd_pack = ws.take(hp.fwd_total);
    pl.head_bwd_pack = ws.take(hp.bwd_total);
    pl.head_dw_stride = (pl.MO * pl.MA + pl.MA * pl.MA) * 256 + 4 * pl.OT + 4 * pl.HT;
    pl.head_dw_stride = (pl.head_dw_stride + 63) & ~63;
    pl.head_dw_partial = ws.take((size_t)pl.n_head_waves * pl.head_dw_stride);
    pl.head_dw_reduced = ws.take((size_t)kReduceSplits * pl.head_dw_stride);
    pl.total_floats = ws.at;
    return ESRNN_OK;
}

}  // namespace esrnn
