// Reverse pass of a dilated LSTM layer on the 4-series kernels: the kernel template and its launcher, included by
// one translation unit per kind of workgroup (four waves / eight waves) so that the two compile side by side.
#pragma once

#include "lstm_narrow_common.h"

namespace esrnn {

namespace {

// ---------------------------------------------------------------------------
// Reverse pass.  Per position p of a chain, descending:
//   A. every lane turns (dh, dc) of its (unit, series) into the four gate
//      pre-activation gradients da (registers; a copy goes to LDS for step C);
//   B. a wave multiplies W^T by the da of the units it owns: 4x4x1 MFMA with da
//      as the broadcast A operand, taken from the registers of the four lanes
//      that hold unit u, and the weights as B (a block is four consecutive
//      columns of [x ; h]); the four partial results meet in LDS (part);
//   -- barrier --
//   every lane sums the four partials of its own (unit, series): the recurrent
//      dh of the next position; the threads sum and store the input gradient;
//   C. dW += da (x) [x_p ; h_{p-d}]: one 16x16x4 MFMA per 16x16 tile of dW, k =
//      the four series; row tiles dealt to the waves round-robin.
// da_all and part alternate between two copies by position parity: what a
// position writes was last read two positions earlier, one barrier ago.  The
// staged operands of a chunk of positions: per-thread values (gates, cell
// states, arriving gradient) in a buffer every thread reads only where it wrote;
// [x ; h] rows, which the whole workgroup reads, in two buffers by chunk parity.
// ---------------------------------------------------------------------------
struct NarrowBwdArgs {
    const float *wpack;   // [4][NG][4*HT][64]  operands of W^T: wave, column group, k-step (unit, gate), lane = column
    const float *xsrc;    // TL(4*KXT)
    const float *gates, *c;
    ptrdiff_t hid_minus_xsrc;   // hidden states TL(HP), as an offset in floats from xsrc (both lie in the workspace)
    const float *gsrc[2];
    int n_gsrc;
    float *gdst;          // TL(4*KXT)
    float *dw_partial;    // [4*NB*chains][HT*CT][4][64]
    float *db_partial;    // [4*NB*chains][HT][4][4]
    int P, NB, d;
    const int32_t *pmax;  // [NB] positions the longest series of a 16-series tile has: its chains stop there
    const int32_t *lengths;
    const Scalars *sc;
    float two_lambda_cs;
    int B, T, I, H;
};

// (up to hidden 40 the kernel is held to 256 registers: two workgroups per compute unit, which the chains of a
// dilated layer need to run side by side)
// SPLIT: eight waves.  Waves 0-3 carry the recurrence (steps A and B and the sums); waves 4-7 do step C, the
// weight gradient, which only consumes what step A leaves in LDS, one barrier behind them.  Both kinds take the
// same barriers (one per position).  For grids of at most one workgroup per compute unit: the chain waves then
// have half the matrix work per position, and the SIMDs have the weight-gradient waves' work while a chain wave
// waits.
template <int HT, int KXT, bool CP, bool SPLIT>
__global__ void __launch_bounds__(SPLIT ? 2 * kNT : kNT, (!SPLIT && HT <= 10) ? 2 : 1) lstm_backward_narrow_kernel(NarrowBwdArgs a)
{
    constexpr int KX = 4 * KXT, HP = 4 * HT, KT4 = KX + HP;
    constexpr int CH = 4;                        // positions per chunk of staged operands
    constexpr int NG = (KT4 + 63) / 64;          // groups of 64 columns of [x ; h]
    constexpr int CT = (KT4 + 15) / 16;          // 16-column tiles of dW
    constexpr int MTW = (HT + kNW - 1) / kNW;    // 16-row tiles of dW per wave (a row tile = 4 units x 4 gates)
    constexpr int XH_PER = (4 * KT4 + kNT - 1) / kNT;
    __shared__ __align__(16) float da_all[2][HP * 16];           // [unit][series][gate]
    __shared__ __align__(16) float part[2][kNW][NG * 64 * 4];    // partial W^T da of every wave [column][series]
    __shared__ __align__(16) f32x4 lc[CH][2][kNT];               // per thread: activated gates; c, c_{p-d}, two gradient sources
    __shared__ float xhc[2][CH][CT * 64];                        // [column of x_p ; h_{p-d}][series]

    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int w = SPLIT ? (wv & (kNW - 1)) : wv;
    const bool dw_wave = SPLIT && wv >= kNW;
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
    const int lane_off = unit * 16 + 4 * q + j;
    // input gradient: thread t sums and stores element t mod 4*KX (threads past 4*KX repeat earlier ones)
    const int dx_el = (int)threadIdx.x % (4 * KX);
    // operands of the weight-gradient tiles inside 64 consecutive floats of da_all / xhc
    const int ar_off = 16 * (lane & 3) + 4 * (lane >> 4) + ((lane & 15) >> 2);   // unit l%4, series l/16, gate (l%16)/4
    const int xb_off = 4 * (lane & 15) + (lane >> 4);                            // column l%16, series l/16

    float wreg[NG][4 * HT];
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
        for (int k = 0; k < 4 * HT; ++k) wreg[g][k] = a.wpack[(((size_t)w * NG + g) * (4 * HT) + k) * 64 + lane];
    f32x4 dw[MTW][CT];
#pragma unroll
    for (int t = 0; t < MTW; ++t)
#pragma unroll
        for (int nb = 0; nb < CT; ++nb) dw[t][nb] = f32x4{0.f, 0.f, 0.f, 0.f};
    f32x4 dbacc = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int e = threadIdx.x; e < 2 * CH * CT * 64; e += kNT) (&xhc[0][0][0])[e] = 0.0f;   // columns past KT4 stay zero

    auto store_dw = [&]() {
        const size_t partix = (size_t)(4 * bt + q) * gridDim.y + blockIdx.y;
#pragma unroll
        for (int t = 0; t < MTW; ++t) {
            const int mt = w + kNW * t;
            if (mt < HT) {
#pragma unroll
                for (int nb = 0; nb < CT; ++nb) {
                    float *dst = a.dw_partial + (partix * (HT * CT) + mt * CT + nb) * 256 + lane;
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) dst[rr * 64] = dw[t][nb][rr];
                }
            }
        }
    };
    if constexpr (SPLIT) {
        if (dw_wave) {
            // ---- C: weight gradient of one position, k = the four series; da in da_all[par], [x ; h] in xhc[cpar][ii]
            auto step_c = [&](int par, int cpar, int ii) {
                float xb[CT];
#pragma unroll
                for (int nb = 0; nb < CT; ++nb) xb[nb] = xhc[cpar][ii][64 * nb + xb_off];
#pragma unroll
                for (int t = 0; t < MTW; ++t) {
                    const int mt = w + kNW * t;
                    if (mt < HT) {
                        // row 4*gate + u of the tile is gate `gate` of unit 4*mt + u
                        const float ar = da_all[par][64 * mt + ar_off];
#pragma unroll
                        for (int nb = 0; nb < CT; ++nb) dw[t][nb] = mfma16(ar, xb[nb], dw[t][nb]);
                    }
                }
            };
            // the same barriers as the chain waves below: start of a chain, first staging, one per position
            for (int r0 = blockIdx.y; r0 < a.d && r0 < Pt; r0 += gridDim.y) {
                const int n = (Pt - r0 + a.d - 1) / a.d;
                __syncthreads();
                lds_barrier();
                for (int i = 0; i < n; ++i) {
                    lds_barrier();
                    step_c(i & 1, (i / CH) & 1, i % CH);
                }
            }
            store_dw();
            return;
        }
    }

    const float g2_scale = a.n_gsrc >= 2 ? 1.0f : 0.0f;
    int n_valid = 0;
    float pen = 0.0f;
    if constexpr (CP) {
        const int col = bt * kTileN + 4 * q + j;
        const int len = col < a.B ? min(max(a.lengths[col], 0), a.T) : 0;
        n_valid = len - a.I - a.H + 1;
        pen = a.two_lambda_cs * a.sc->inv_n_cs;
    }

    for (int r0 = blockIdx.y; r0 < a.d && r0 < Pt; r0 += gridDim.y) {
        const int n = (Pt - r0 + a.d - 1) / a.d;
        const int p_last = r0 + (n - 1) * a.d;
        // operands of the i-th position from the end of the chain (requests past the chain repeat the last)
        f32x4 s_gt[CH], s_o[CH];     // (native vectors: arrays of the HIP float4 class do not stay in registers)
        float s_xh[CH][XH_PER];
        auto load_chunk = [&](int c) {
#pragma unroll
            for (int ii = 0; ii < CH; ++ii) {
                const int p = p_last - min(c * CH + ii, n - 1) * a.d;
                const size_t pb = (size_t)p * a.NB + bt;
                const size_t pbd = (size_t)(p >= a.d ? p - a.d : p) * a.NB + bt;
                const size_t e = pb * (HP * 16) + lane_off;
                s_gt[ii] = reinterpret_cast<const f32x4 *>(a.gates)[e];
                s_o[ii] = f32x4{a.c[e], a.c[pbd * (HP * 16) + lane_off], a.gsrc[0][e], a.gsrc[1][e]};
#pragma unroll
                for (int k = 0; k < XH_PER; ++k) {
                    const int el = min((int)threadIdx.x + k * kNT, 4 * KT4 - 1);
                    const int col = el >> 2, jj = el & 3;
                    // one base pointer and a per-lane offset (a per-lane choice between two pointers would be
                    // fetched from the argument block in memory, with a wait, before every request)
                    const ptrdiff_t off = col < KX ? (ptrdiff_t)((pb * KX + col) * 16)
                                                   : a.hid_minus_xsrc + (ptrdiff_t)((pbd * HP + (col - KX)) * 16);
                    s_xh[ii][k] = a.xsrc[off + 4 * q + jj];
                }
            }
        };
        auto flush_chunk = [&](int c) {
#pragma unroll
            for (int ii = 0; ii < CH; ++ii) {
                const bool has_prev = p_last - min(c * CH + ii, n - 1) * a.d >= a.d;
                lc[ii][0][threadIdx.x] = s_gt[ii];
                lc[ii][1][threadIdx.x] = s_o[ii];
#pragma unroll
                for (int k = 0; k < XH_PER; ++k) {
                    const int el = (int)threadIdx.x + k * kNT;
                    if (el < 4 * KT4) xhc[c & 1][ii][el] = (el < 4 * KX || has_prev) ? s_xh[ii][k] : 0.0f;
                }
            }
        };
        load_chunk(0);
        float dcreg = 0.0f, dhreg = 0.0f;
        __syncthreads();            // LDS free: initial clearing, or the last position of the previous chain
        flush_chunk(0);
        lds_barrier();

        // per-thread operands of the first position; those of position i+1 are read before the barrier
        // that ends position i
        f32x4 gt = lc[0][0][threadIdx.x];      // activated input, forget, candidate, output gate
        f32x4 o = lc[0][1][threadIdx.x];       // c, c_{p-d}, gradient sources
        // One position: the i-th from the end of the chain, staged in slot ii of the chunk buffers of parity
        // cpar; the per-thread operands of the next position are in slot `next`.  `staged` runs after they
        // have been read and before the barrier (the staging of the next chunk goes there).
        auto position = [&](int i, int ii, int cpar, int next, auto staged) {
            const int par = i & 1;
            const int p = p_last - i * a.d;
            const bool has_prev = p >= a.d;
            // ---- A: gate gradients of (unit, series)
            const float dh = o[2] + g2_scale * o[3] + dhreg;
            const float tc = tanh_f(o[0]);
            const float dh_o = dh * gt[3];          // (shared products formed once)
            float dc = dcreg + dh_o * (1.0f - tc * tc);
            if constexpr (CP) dc += p < n_valid ? pen * o[0] : 0.0f;
            const float cp = has_prev ? o[1] : 0.0f;
            const float dc_i = dc * gt[0], dc_f = dc * gt[1];
            f32x4 da;
            da[0] = dc_i * gt[2] * (1.0f - gt[0]);
            da[1] = dc_f * cp * (1.0f - gt[1]);
            da[2] = dc_i * (1.0f - gt[2] * gt[2]);
            da[3] = dh_o * tc * (1.0f - gt[3]);
            dcreg = dc_f;
            if (valid) dbacc += da;
            *reinterpret_cast<f32x4 *>(&da_all[par][16 * unit + 4 * j]) = da;    // for step C
            // ---- B: partial W^T da over the k-steps (unit, gate) of this wave; da of unit u is
            // broadcast from the registers of block u.  Two chains of dependent instructions: the two
            // column groups, or with one group two accumulators (more would cost the second resident
            // workgroup its registers at hidden 40).
            constexpr int kBwdAcc = NG == 1 ? 2 : 1;
            f32x4 acc[NG][4];
#pragma unroll
            for (int g = 0; g < NG; ++g) acc[g][0] = acc[g][1] = acc[g][2] = acc[g][3] = f32x4{0.f, 0.f, 0.f, 0.f};
            static_for<0, HT>([&](auto ic) {
                constexpr int ul = decltype(ic)::value;
#pragma unroll
                for (int g = 0; g < NG; ++g) {
                    acc[g][0] = mfma4_bcast<ul>(da[0], wreg[g][4 * ul + 0], acc[g][0]);
                    acc[g][1 % kBwdAcc] = mfma4_bcast<ul>(da[1], wreg[g][4 * ul + 1], acc[g][1 % kBwdAcc]);
                }
#pragma unroll
                for (int g = 0; g < NG; ++g) {
                    acc[g][2 % kBwdAcc] = mfma4_bcast<ul>(da[2], wreg[g][4 * ul + 2], acc[g][2 % kBwdAcc]);
                    acc[g][3 % kBwdAcc] = mfma4_bcast<ul>(da[3], wreg[g][4 * ul + 3], acc[g][3 % kBwdAcc]);
                }
            });
            // lane l of group g holds column 64g + l for the four series
#pragma unroll
            for (int g = 0; g < NG; ++g)
                *reinterpret_cast<f32x4 *>(&part[par][w][(64 * g + lane) * 4]) =
                    kBwdAcc == 4 ? (acc[g][0] + acc[g][1]) + (acc[g][2] + acc[g][3]) : kBwdAcc == 2 ? acc[g][0] + acc[g][1] : acc[g][0];
            // per-thread operands of the next position (staged at least one barrier ago)
            gt = lc[next][0][threadIdx.x];
            o = lc[next][1][threadIdx.x];
            staged();
            lds_barrier();
            // ---- sums of the four partials: recurrent dh of this lane; input gradient
            {
                const int e = 4 * (KX + unit) + j;
                dhreg = (part[par][0][e] + part[par][1][e]) + (part[par][2][e] + part[par][3][e]);
            }
            const float dxv = (part[par][0][dx_el] + part[par][1][dx_el]) + (part[par][2][dx_el] + part[par][3][dx_el]);
            (a.gdst + ((size_t)p * a.NB + bt) * (KX * 16))[(dx_el >> 2) * 16 + 4 * q + (dx_el & 3)] = dxv;
            // ---- C: weight gradient, k = the four series (on the waves of its own where there are some)
            if constexpr (!SPLIT) {
                float xb[CT];
#pragma unroll
                for (int nb = 0; nb < CT; ++nb) xb[nb] = xhc[cpar][ii][64 * nb + xb_off];
#pragma unroll
                for (int t = 0; t < MTW; ++t) {
                    const int mt = w + kNW * t;
                    if (mt < HT) {
                        // row 4*gate + u of the tile is gate `gate` of unit 4*mt + u
                        const float ar = da_all[par][64 * mt + ar_off];
#pragma unroll
                        for (int nb = 0; nb < CT; ++nb) dw[t][nb] = mfma16(ar, xb[nb], dw[t][nb]);
                    }
                }
            }
        };
        // Whole chunks: one straight run of instructions each.  The operands of the next chunk are requested
        // at its start and staged one position before its end (after this thread has read its operands of the
        // chunk's last position): request and use in the same run, so the wait for a request counts the
        // memory operations issued since instead of waiting for all of them.
        int c = 0;
        for (; (c + 1) * CH <= n; ++c) {
            load_chunk(c + 1);              // (requests past the chain repeat its last position)
            static_for<0, CH>([&](auto iic) {
                constexpr int ii = decltype(iic)::value;
                position(c * CH + ii, ii, c & 1, (ii + 1) % CH, [&] {
                    if constexpr (ii == CH - 2) flush_chunk(c + 1);
                });
            });
        }
        // the last, partial chunk (staged by the run before it, or by the start of the chain)
        for (int i = c * CH; i < n; ++i) position(i, i - c * CH, c & 1, min(i + 1, n - 1) - c * CH, [] {});
    }

    if constexpr (!SPLIT) store_dw();
    const size_t partix = (size_t)(4 * bt + q) * gridDim.y + blockIdx.y;
    // bias gradient: sum over the four series (the lanes of a quad)
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
        float v = dbacc[rr];
        v += quad_perm<0xB1>(v);
        v += quad_perm<0x4E>(v);
        dbacc[rr] = v;
    }
    if (valid && j == 0) {
        float *dst = a.db_partial + partix * (HT * 16) + (size_t)unit * 4;
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) dst[rr] = dbacc[rr];
    }
}

template <int HT, int KXT, bool SPLIT>
hipError_t run_nbwd(const NarrowBwdArgs &a, int chains, hipStream_t st)
{
    const dim3 grid(narrow_grid_x(a.NB), chains);
    if (a.sc) lstm_backward_narrow_kernel<HT, KXT, true, SPLIT><<<grid, SPLIT ? 2 * kNT : kNT, 0, st>>>(a);
    else lstm_backward_narrow_kernel<HT, KXT, false, SPLIT><<<grid, SPLIT ? 2 * kNT : kNT, 0, st>>>(a);
    return hipGetLastError();
}

template <bool SPLIT>
hipError_t launch_narrow_bwd(const Plan &pl, int layer, const int32_t *lengths, float *ws, hipStream_t st)
{
    const LayerPlan &lp = pl.layer[layer];
    NarrowBwdArgs a{};
    const bool cp = lp.first_in_block && pl.cfg.lambda_cs != 0.0f;
    a.lengths = lengths;
    a.sc = cp ? reinterpret_cast<const Scalars *>(ws + pl.scalars) : nullptr;
    a.two_lambda_cs = 2.0f * pl.cfg.lambda_cs;
    a.B = pl.B; a.T = pl.T; a.I = pl.I; a.H = pl.H;
    a.wpack = ws + lp.wpack_bwd; a.xsrc = ws + lp.xsrc; a.gates = ws + lp.gates; a.c = ws + lp.c;
    a.hid_minus_xsrc = (ptrdiff_t)lp.hid - (ptrdiff_t)lp.xsrc;
    a.n_gsrc = lp.n_gsrc < 2 ? lp.n_gsrc : 2;
    a.gsrc[0] = ws + lp.gsrc[0];
    a.gsrc[1] = ws + (lp.n_gsrc > 2 ? pl.gsum : lp.gsrc[lp.n_gsrc >= 2 ? 1 : 0]);
    a.gdst = ws + lp.gdst; a.dw_partial = ws + lp.dw_partial; a.db_partial = ws + lp.db_partial;
    a.P = pl.P; a.NB = pl.NB; a.d = lp.dil;
    a.pmax = reinterpret_cast<const int32_t *>(ws + pl.pmax);
#define X(HT_, KXT_) if (pl.HT == HT_ && lp.KXT == KXT_) return run_nbwd<HT_, KXT_, SPLIT>(a, lp.chains, st);
    ESRNN_LSTM_SHAPES(X)
#undef X
    return hipErrorInvalidValue;
}

}  // namespace

}  // namespace esrnn
