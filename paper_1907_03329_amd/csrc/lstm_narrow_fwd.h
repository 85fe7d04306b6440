// Forward pass of a dilated LSTM layer on the 4-series kernels (see lstm_narrow_common.h for the tiling): the
// kernel template and its launcher, included by one translation unit per residual wiring (plain layer / last layer
// of a residual block) so that the two compile side by side.
#pragma once

#include "lstm_narrow_common.h"

namespace esrnn {

namespace {

struct NarrowFwdArgs {
    const float *wpack;   // [4][KT4][64]  weight operands: wave, input column, lane (gate l%4 of unit l/4 of the wave)
    const float *bias;    // caller's bias vector [4h]
    const float *xsrc;    // TL(4*KXT)
    float *gates;         // TL(HP) x [4]
    float *c, *hid;       // TL(HP)
    const float *resid;   // TL(HP) or null
    float *out;           // TL(HP) or null: resid + hid
    int P, NB, d, h;
    const int32_t *pmax;  // [NB] positions the longest series of a 16-series tile has: its chains stop there
    const int32_t *lengths;
    float *cs_partial;    // [4*NB * gridDim.y] (cell-state penalty, CP instantiations only)
    int B, T, I, H;
};

// CP: the layer's cell states enter the cell-state penalty; OUT: the layer ends a residual block (reads the
// block input, writes the block output).
template <int HT, int KXT, bool CP, bool OUT>
__global__ void __launch_bounds__(kNT) lstm_forward_narrow_kernel(NarrowFwdArgs a)
{
    constexpr int KX = 4 * KXT, HP = 4 * HT;
    constexpr int CH = 8;                       // positions per chunk of staged inputs
    constexpr int XG = (KX + 15) / 16, HG = (HP + 15) / 16;   // groups of 16 columns (one register each)
    // inputs x_p of a chunk of positions [column][series], by chunk parity (+ 64 floats that take the writes of
    // the threads with no input row, so that staging is the same instruction stream in every thread)
    __shared__ float xc[2][CH][XG * 64 + 64];
    __shared__ float rc[CH][kNT];               // residual input of this thread's (unit, series)
    __shared__ float hb[2][HG * 64];            // h_{p-d} [unit][series], by position parity

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int blk = lane >> 2, j = lane & 3;
    // The four workgroups of a 16-series tile share every 64-byte row of the tile.  Consecutive workgroup
    // ids go round the 8 XCDs, each with its own L2: ids x, x+8, x+16, x+24 of a group of 32 are the four
    // quarters of ONE tile, so they land on the same XCD at about the same time and a row is fetched from
    // HBM once, not four times (measured before: 2.3-2.8 times the algorithmic bytes).
    const int bt = (blockIdx.x >> 5) * 8 + (blockIdx.x & 7), q = (blockIdx.x >> 3) & 3;
    if (bt >= a.NB) return;     // the grid is padded to whole groups of 32 (before any barrier)
    // All four workgroups of a 16-series tile stop at the tile's longest series: what lies beyond is
    // neither computed here nor read by any later kernel.
    const int Pt = a.pmax[bt];
    const bool valid = blk < HT;
    const int unit = w * HT + min(blk, HT - 1);     // blocks past HT repeat the last unit

    float wx[KX], wh[HP];
#pragma unroll
    for (int k = 0; k < KX; ++k) wx[k] = a.wpack[((size_t)w * (KX + HP) + k) * 64 + lane];
#pragma unroll
    for (int k = 0; k < HP; ++k) wh[k] = a.wpack[((size_t)w * (KX + HP) + KX + k) * 64 + lane];
    // before the transpose a lane holds gate j of its unit for the four series
    const float bias = unit < a.h ? a.bias[j * a.h + unit] : 0.0f;

    // element of this lane inside the TL(HP) block of one (position, series tile)
    const int lane_off = unit * 16 + 4 * q + j;
    // cooperative input load: thread t < 4*KX brings row t/4 of series t%4 (the others repeat row 0)
    const bool x_thread = (int)threadIdx.x < 4 * KX;
    const int x_off = (x_thread ? (int)threadIdx.x >> 2 : 0) * 16 + 4 * q + (threadIdx.x & 3);
    const int x_slot = x_thread ? (int)threadIdx.x : XG * 64 + lane;

    int n_valid = 0;
    float csq = 0.0f;
    if constexpr (CP) {
        const int col = bt * kTileN + 4 * q + j;
        const int len = col < a.B ? min(max(a.lengths[col], 0), a.T) : 0;
        n_valid = len - a.I - a.H + 1;
    }
    // columns past KX / HP in the last group of 16 are never written: zero once (their weights do not exist)
    for (int e = threadIdx.x; e < 2 * CH * (XG * 64 + 64); e += kNT) (&xc[0][0][0])[e] = 0.0f;
    for (int e = threadIdx.x; e < 2 * HG * 64; e += kNT) (&hb[0][0])[e] = 0.0f;

    for (int r = blockIdx.y; r < a.d && r < Pt; r += gridDim.y) {
        const int n = (Pt - r + a.d - 1) / a.d;            // positions of this chain: r, r+d, ...
        float xs[CH], rs[CH];
        auto load_chunk = [&](int c) {
#pragma unroll
            for (int ii = 0; ii < CH; ++ii) {
                const size_t tile = (size_t)(r + min(c * CH + ii, n - 1) * a.d) * a.NB + bt;
                xs[ii] = (a.xsrc + tile * (KX * 16))[x_off];
                rs[ii] = OUT ? (a.resid + tile * (HP * 16))[lane_off] : 0.0f;
            }
        };
        auto flush_chunk = [&](int c) {
#pragma unroll
            for (int ii = 0; ii < CH; ++ii) {
                xc[c & 1][ii][x_slot] = xs[ii];
                if (OUT) rc[ii][threadIdx.x] = rs[ii];
            }
        };
        float creg = 0.0f;
        // One position.  `staged` runs after the recurrent state is published and before the position's
        // stores are issued (the staging of the next chunk goes there).
        auto position = [&](int i, int ii, int cpar, auto staged) {
            const int p = r + i * a.d;
            // [x_p ; h_{p-d}] of the four series: lane (b, s) of register m holds column 16m + b of series s
            float vh[HG], vx[XG];
#pragma unroll
            for (int m = 0; m < HG; ++m) vh[m] = hb[i & 1][64 * m + lane];
#pragma unroll
            for (int m = 0; m < XG; ++m) vx[m] = xc[cpar][ii][64 * m + lane];
            const float res = OUT ? rc[ii][threadIdx.x] : 0.0f;
            // two accumulators: consecutive instructions never depend on each other (measured: one is
            // slower, four are slower too)
            f32x4 acc0 = f32x4{bias, bias, bias, bias}, acc1 = f32x4{0.f, 0.f, 0.f, 0.f};
            static_for<0, KX / 2>([&](auto ic) {
                constexpr int k = 2 * decltype(ic)::value;
                acc0 = mfma4_bcast<k % 16>(vx[k / 16], wx[k], acc0);
                acc1 = mfma4_bcast<(k + 1) % 16>(vx[k / 16], wx[k + 1], acc1);
            });
            static_for<0, HP / 2>([&](auto ic) {
                constexpr int k = 2 * decltype(ic)::value;
                acc0 = mfma4_bcast<k % 16>(vh[k / 16], wh[k], acc0);
                acc1 = mfma4_bcast<(k + 1) % 16>(vh[k / 16], wh[k + 1], acc1);
            });
            f32x4 pre = acc0 + acc1;        // gate j of the unit, series 0..3
            quad_transpose(pre, j);         // gates 0..3 of the unit, series j
            const float gi = sigmoid_f(pre[0]);
            const float gf = sigmoid_f(pre[1]);
            const float gg = tanh_f(pre[2]);
            const float go = sigmoid_f(pre[3]);
            const float cn = gf * creg + gi * gg;
            const float hn = go * tanh_f(cn);
            creg = cn;
            if constexpr (CP) csq += (valid && p < n_valid) ? cn * cn : 0.0f;
            hb[(i + 1) & 1][4 * unit + j] = hn;
            staged();
            // wave-uniform tile base plus the lane's element: scalar address arithmetic
            const size_t tile = ((size_t)p * a.NB + bt) * (HP * 16);
            __builtin_nontemporal_store(f32x4{gi, gf, gg, go}, reinterpret_cast<f32x4 *>(a.gates) + tile + lane_off);
            (a.c + tile)[lane_off] = cn;     // (a plain store: the four quarter-row writes of a tile then merge in L2)
            (a.hid + tile)[lane_off] = hn;
            if (OUT) (a.out + tile)[lane_off] = res + hn;
            lds_barrier();
        };
        // start of a chain: zero state, inputs of the first chunk staged
        load_chunk(0);
        __syncthreads();            // LDS free: initial clearing, or the last position of the previous chain
        for (int e = threadIdx.x; e < 4 * HP; e += kNT) hb[0][e] = 0.0f;
        flush_chunk(0);
        lds_barrier();

        // Whole chunks: the body of a chunk is one straight run of instructions.  The inputs of the next chunk
        // are requested at its start and staged at its end, before the stores of its last position: memory
        // operations complete in order, and with request and use in the same run the wait for a request is a
        // count of the stores issued since (those of seven positions), never a wait for the newest stores.
        int c = 0;
        for (; (c + 1) * CH <= n; ++c) {
            load_chunk(c + 1);              // (row indices stop at the chain's last position)
            static_for<0, CH>([&](auto iic) {
                constexpr int ii = decltype(iic)::value;
                position(c * CH + ii, ii, c & 1, [&] {
                    if constexpr (ii == CH - 1) flush_chunk(c + 1);
                });
            });
        }
        // the last, partial chunk (staged by the run before it, or by the start of the chain)
        for (int i = c * CH; i < n; ++i) position(i, i - c * CH, c & 1, [] {});
    }
    if constexpr (CP) {
        __shared__ float s_cs[kNW];
        const float tot = wave_sum(csq);
        if (lane == 0) s_cs[w] = tot;
        __syncthreads();
        if (threadIdx.x == 0)
            a.cs_partial[(4 * bt + q) * gridDim.y + blockIdx.y] = (s_cs[0] + s_cs[1]) + (s_cs[2] + s_cs[3]);
    }
}

template <int HT, int KXT, bool OUT>
hipError_t run_nfwd(const NarrowFwdArgs &a, int chains, hipStream_t st)
{
    const dim3 grid(narrow_grid_x(a.NB), chains);
    if (a.cs_partial) lstm_forward_narrow_kernel<HT, KXT, true, OUT><<<grid, 64 * kNW, 0, st>>>(a);
    else lstm_forward_narrow_kernel<HT, KXT, false, OUT><<<grid, 64 * kNW, 0, st>>>(a);
    return hipGetLastError();
}

template <bool OUT>
hipError_t launch_narrow_fwd(const Plan &pl, int layer, const int32_t *lengths, const float *weights, float *ws,
                             hipStream_t st)
{
    const LayerPlan &lp = pl.layer[layer];
    const bool cp = lp.first_in_block && pl.cfg.lambda_cs != 0.0f;
    NarrowFwdArgs a{ws + lp.wpack_fwd, weights + lp.b_off, ws + lp.xsrc, ws + lp.gates, ws + lp.c, ws + lp.hid,
                    lp.out ? ws + lp.resid : nullptr, lp.out ? ws + lp.out : nullptr, pl.P, pl.NB, lp.dil, pl.h,
                    reinterpret_cast<const int32_t *>(ws + pl.pmax), lengths, cp ? ws + lp.cs_partial : nullptr, pl.B, pl.T, pl.I, pl.H};
#define X(HT_, KXT_) if (pl.HT == HT_ && lp.KXT == KXT_) return run_nfwd<HT_, KXT_, OUT>(a, lp.chains, st);
    ESRNN_LSTM_SHAPES(X)
#undef X
    return hipErrorInvalidValue;
}

}  // namespace

}  // namespace esrnn
