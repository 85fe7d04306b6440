// Dilated LSTM layer, forward and reverse (Section 3.2, Table 1), one launch per
// layer.  A workgroup of four waves owns 16 series and walks the window
// positions in order; series never interact, so there is no grid-level
// synchronisation.  The gate contraction runs on the 16x16x4 fp32 MFMA with the
// weights as the A operand, held in registers for the whole launch, and the
// activations [x_p ; h_{p-d}] of 16 series as the B operand.
//
// Row order of the A operand: row 4g+r of unit tile mt is gate r of hidden unit
// 4mt+g.  With that order a lane ends up holding the four gate pre-activations
// of one unit for one series (cell update without any cross-lane traffic), and
// the hidden state it produces for unit tile mt is, as it stands, the B operand
// of k-step mt of a later position.
#include "device_utils.h"
#include "esrnn_internal.h"

namespace esrnn {

namespace {

struct LstmFwdArgs {
    const float *wpack;   // [HT][KT][64]
    const float *bpack;   // [HT][4][4]
    const float *xsrc;    // TL(4*KXT)
    float *gates;         // [P][NB][HT][64][4]
    float *c, *hid;       // TL(HP)
    const float *resid;   // TL(HP) or null
    float *out;           // TL(HP) or null: resid + hid
    int P, NB, d;
};

template <int HT, int KXT>
__global__ void __launch_bounds__(64 * kLstmWaves) lstm_forward_kernel(LstmFwdArgs a)
{
    constexpr int KT = KXT + HT;
    constexpr int MTW = (HT + kLstmWaves - 1) / kLstmWaves;   // unit tiles per wave
    __shared__ float hbuf[2][HT * 64];

    const int lane = threadIdx.x & 63, s = threadIdx.x >> 6, bt = blockIdx.x;
    const bool d1 = (a.d == 1);

    float wreg[MTW][KT];
    f32x4 bias[MTW];
    float creg[MTW];
#pragma unroll
    for (int j = 0; j < MTW; ++j) {
        const int mt = s + kLstmWaves * j;
        const bool valid = mt < HT;
#pragma unroll
        for (int ks = 0; ks < KT; ++ks) wreg[j][ks] = valid ? a.wpack[((size_t)mt * KT + ks) * 64 + lane] : 0.0f;
        const float4 bv = valid ? *reinterpret_cast<const float4 *>(a.bpack + (mt * 4 + (lane >> 4)) * 4)
                                : make_float4(0.f, 0.f, 0.f, 0.f);
        bias[j] = f32x4{bv.x, bv.y, bv.z, bv.w};
        creg[j] = 0.0f;
    }
    for (int i = threadIdx.x; i < HT * 64; i += 64 * kLstmWaves) hbuf[0][i] = 0.0f;
    __syncthreads();

    const size_t xtile = (size_t)KXT * 64, htile = (size_t)HT * 64;
    float bx[KXT], bh[HT], cpv[MTW];
#pragma unroll
    for (int ks = 0; ks < KXT; ++ks) bx[ks] = a.xsrc[(size_t)bt * xtile + ks * 64 + lane];
#pragma unroll
    for (int ks = 0; ks < HT; ++ks) bh[ks] = 0.0f;
#pragma unroll
    for (int j = 0; j < MTW; ++j) cpv[j] = 0.0f;

    for (int p = 0; p < a.P; ++p) {
        const size_t pb = (size_t)p * a.NB + bt;
        if (d1) {
#pragma unroll
            for (int ks = 0; ks < HT; ++ks) bh[ks] = hbuf[p & 1][ks * 64 + lane];
        }
        f32x4 acc[MTW];
#pragma unroll
        for (int j = 0; j < MTW; ++j) acc[j] = bias[j];
#pragma unroll
        for (int ks = 0; ks < KXT; ++ks)
#pragma unroll
            for (int j = 0; j < MTW; ++j) acc[j] = mfma16(wreg[j][ks], bx[ks], acc[j]);
#pragma unroll
        for (int ks = 0; ks < HT; ++ks)
#pragma unroll
            for (int j = 0; j < MTW; ++j) acc[j] = mfma16(wreg[j][KXT + ks], bh[ks], acc[j]);

        // operands of the next position (the input never depends on this layer)
        if (p + 1 < a.P) {
            const size_t nb = ((size_t)(p + 1) * a.NB + bt) * xtile;
#pragma unroll
            for (int ks = 0; ks < KXT; ++ks) bx[ks] = a.xsrc[nb + ks * 64 + lane];
        }

#pragma unroll
        for (int j = 0; j < MTW; ++j) {
            const int mt = s + kLstmWaves * j;
            if (mt < HT) {
                const float gi = sigmoid_f(acc[j][0]);
                const float gf = sigmoid_f(acc[j][1]);
                const float gg = tanh_f(acc[j][2]);
                const float go = sigmoid_f(acc[j][3]);
                const float cprev = d1 ? creg[j] : cpv[j];
                const float cn = gf * cprev + gi * gg;
                const float hn = go * tanh_f(cn);
                const size_t e = (pb * HT + mt) * 64 + lane;
                reinterpret_cast<float4 *>(a.gates)[e] = make_float4(gi, gf, gg, go);
                a.c[e] = cn;
                a.hid[e] = hn;
                if (a.out) a.out[e] = a.resid[e] + hn;
                creg[j] = cn;
                if (d1) hbuf[(p + 1) & 1][mt * 64 + lane] = hn;
            }
        }
        if (d1) {
            lds_barrier();
        } else {
            // the state of position p+1-d was written by all four waves: make
            // those stores visible before anyone reads them back
            __syncthreads();
            if (p + 1 < a.P) {
                if (p + 1 >= a.d) {
                    const size_t rb = ((size_t)(p + 1 - a.d) * a.NB + bt) * htile;
#pragma unroll
                    for (int ks = 0; ks < HT; ++ks) bh[ks] = a.hid[rb + ks * 64 + lane];
#pragma unroll
                    for (int j = 0; j < MTW; ++j) {
                        const int mt = s + kLstmWaves * j;
                        cpv[j] = mt < HT ? a.c[rb + mt * 64 + lane] : 0.0f;
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Reverse pass of one layer.  Per position p (descending):
//   A. every lane turns (dh, dc) of its hidden unit into the four gate
//      pre-activation gradients da and leaves them in LDS;
//   B. transposed contraction d[x_p ; h_{p-d}] = W^T da on the MFMA, with W^T
//      register-resident; the row order of its output tiles is chosen so that
//      the result is again laid out one unit tile per 64 lanes;
//   C. weight gradient dW += da (x) [x_p ; h_{p-d}]: contraction over the 16
//      series on the MFMA, both operands read transposed from LDS; the tiles
//      stay in accumulators for the whole launch.
// ---------------------------------------------------------------------------
struct LstmBwdArgs {
    const float *wpack;   // [MB][4*HT][64]
    const float *xsrc;    // TL(4*KXT)
    const float *gates, *c, *hid;
    const float *gsrc;    // TL(HP) gradient arriving at the hidden output
    float *gdst;          // TL(4*KXT)
    const float *gadd;    // TL(HP) or null
    float *dhr, *dcr;     // TL(HP) recurrent gradients, dilation >= 2
    float *dw_partial;    // [NB][HT*MB][4][64]
    float *db_partial;    // [NB][HT][4][4]
    int P, NB, d;
};

template <int HT, int KXT>
__global__ void __launch_bounds__(64 * kLstmWaves) lstm_backward_kernel(LstmBwdArgs a)
{
    constexpr int KT = KXT + HT;
    constexpr int MB = (KT + 3) / 4;                                    // 16-row tiles of [x ; h]
    constexpr int MTW = (HT + kLstmWaves - 1) / kLstmWaves;             // unit tiles per wave (step A)
    constexpr int MBW = (MB + kLstmWaves - 1) / kLstmWaves;             // output tiles per wave (step B)
    constexpr int NDW = HT * MB;                                        // weight-gradient tiles
    constexpr int DWW = (NDW + kLstmWaves - 1) / kLstmWaves;            // ... per wave (step C)
    constexpr int XH_ROWS = 16 * MB;
    constexpr int NT = 64 * kLstmWaves;

    __shared__ float da_lds[HT * 16 * kLdsPad];        // [mt][4*gate + unit][series]
    __shared__ float xh_lds[XH_ROWS * kLdsPad];        // [row of x ; h][series]
    __shared__ float dh_lds[HT * 64];                  // recurrent dh for the next position (dilation 1)

    const int lane = threadIdx.x & 63, s = threadIdx.x >> 6, bt = blockIdx.x;
    const int g = lane >> 4, n = lane & 15;
    const bool d1 = (a.d == 1);

    float wreg[MBW][4 * HT];
#pragma unroll
    for (int j = 0; j < MBW; ++j) {
        const int mb = s + kLstmWaves * j;
#pragma unroll
        for (int ks = 0; ks < 4 * HT; ++ks)
            wreg[j][ks] = mb < MB ? a.wpack[((size_t)mb * 4 * HT + ks) * 64 + lane] : 0.0f;
    }
    f32x4 dw[DWW];
#pragma unroll
    for (int j = 0; j < DWW; ++j) dw[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    f32x4 dbacc[MTW];
    float dcreg[MTW];
#pragma unroll
    for (int j = 0; j < MTW; ++j) { dbacc[j] = f32x4{0.f, 0.f, 0.f, 0.f}; dcreg[j] = 0.0f; }
    for (int i = threadIdx.x; i < HT * 64; i += NT) dh_lds[i] = 0.0f;
    for (int i = threadIdx.x; i < XH_ROWS * kLdsPad; i += NT) xh_lds[i] = 0.0f;
    __syncthreads();

    const size_t xtile = (size_t)KXT * 64, htile = (size_t)HT * 64;
    constexpr int XH_PER_THREAD = (KT * 64 + NT - 1) / NT;

    for (int p = a.P - 1; p >= 0; --p) {
        const size_t pb = (size_t)p * a.NB + bt;
        const bool has_prev = p >= a.d;
        const size_t pbd = has_prev ? (size_t)(p - a.d) * a.NB + bt : 0;

        // [x_p ; h_{p-d}] into LDS, row-major with padded rows
#pragma unroll
        for (int i = 0; i < XH_PER_THREAD; ++i) {
            const int e = threadIdx.x + i * NT;
            if (e < KT * 64) {
                float val;
                if (e < KXT * 64) val = a.xsrc[pb * xtile + e];
                else val = has_prev ? a.hid[pbd * htile + (e - KXT * 64)] : 0.0f;
                xh_lds[(e >> 4) * kLdsPad + (e & 15)] = val;
            }
        }

        // A: gate gradients of this wave's units
#pragma unroll
        for (int j = 0; j < MTW; ++j) {
            const int mt = s + kLstmWaves * j;
            if (mt < HT) {
                const size_t e = (pb * HT + mt) * 64 + lane;
                const float4 gt = reinterpret_cast<const float4 *>(a.gates)[e];
                const float cn = a.c[e];
                const float cp = has_prev ? a.c[(pbd * HT + mt) * 64 + lane] : 0.0f;
                float dh = a.gsrc[e];
                float dc;
                if (d1) {
                    dh += dh_lds[mt * 64 + lane];
                    dc = dcreg[j];
                } else {
                    const bool has_next = p + a.d < a.P;
                    dh += has_next ? a.dhr[e] : 0.0f;
                    dc = has_next ? a.dcr[e] : 0.0f;
                }
                const float tc = tanh_f(cn);
                dc += dh * gt.w * (1.0f - tc * tc);
                const float dai = dc * gt.z * gt.x * (1.0f - gt.x);
                const float daf = dc * cp * gt.y * (1.0f - gt.y);
                const float dag = dc * gt.x * (1.0f - gt.z * gt.z);
                const float dao = dh * tc * gt.w * (1.0f - gt.w);
                const float dcp = dc * gt.y;
                if (d1) dcreg[j] = dcp;
                else if (has_prev) a.dcr[(pbd * HT + mt) * 64 + lane] = dcp;
                float *dst = da_lds + (mt * 16 + g) * kLdsPad + n;
                dst[0 * 4 * kLdsPad] = dai;
                dst[1 * 4 * kLdsPad] = daf;
                dst[2 * 4 * kLdsPad] = dag;
                dst[3 * 4 * kLdsPad] = dao;
                dbacc[j][0] += dai; dbacc[j][1] += daf; dbacc[j][2] += dag; dbacc[j][3] += dao;
            }
        }
        lds_barrier();

        // B: d[x ; h] = W^T da
        f32x4 acc[MBW];
#pragma unroll
        for (int j = 0; j < MBW; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 4 * HT; ++ks) {
            // k-step 4mt+gate, contraction index = unit within the tile
            const float bv = da_lds[((ks >> 2) * 16 + (ks & 3) * 4 + g) * kLdsPad + n];
#pragma unroll
            for (int j = 0; j < MBW; ++j) acc[j] = mfma16(wreg[j][ks], bv, acc[j]);
        }
#pragma unroll
        for (int j = 0; j < MBW; ++j) {
            const int mb = s + kLstmWaves * j;
            if (mb < MB) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int q = 4 * mb + r;           // unit tile of [x ; h]
                    if (q < KXT) {
                        const size_t e = pb * xtile + q * 64 + lane;
                        float val = acc[j][r];
                        if (a.gadd) val += a.gadd[e];
                        a.gdst[e] = val;
                    } else if (q < KT) {
                        const int mt = q - KXT;
                        if (d1) dh_lds[mt * 64 + lane] = acc[j][r];   // read after the closing barrier
                        else if (has_prev) a.dhr[(pbd * HT + mt) * 64 + lane] = acc[j][r];
                    }
                }
            }
        }

        // C: dW tiles of this wave
#pragma unroll
        for (int j = 0; j < DWW; ++j) {
            const int tix = s + kLstmWaves * j;
            if (tix < NDW) {
                const int mt = tix / MB, nbk = tix % MB;
                const float *ap = da_lds + (mt * 16 + n) * kLdsPad + g;
                const float *bp = xh_lds + (nbk * 16 + n) * kLdsPad + g;
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) dw[j] = mfma16(ap[4 * ks], bp[4 * ks], dw[j]);
            }
        }
        if (d1) lds_barrier();
        else __syncthreads();   // recurrent gradients go through global memory
    }

    // per-workgroup partial results
#pragma unroll
    for (int j = 0; j < DWW; ++j) {
        const int tix = s + kLstmWaves * j;
        if (tix < NDW) {
            float *dst = a.dw_partial + ((size_t)bt * NDW + tix) * 256 + lane;
#pragma unroll
            for (int r = 0; r < 4; ++r) dst[r * 64] = dw[j][r];
        }
    }
#pragma unroll
    for (int j = 0; j < MTW; ++j) {
        const int mt = s + kLstmWaves * j;
        if (mt < HT) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float tot = group16_sum(dbacc[j][r]);
                if (n == 0) a.db_partial[((size_t)bt * HT + mt) * 16 + g * 4 + r] = tot;
            }
        }
    }
}

template <int HT, int KXT>
hipError_t run_fwd(const LstmFwdArgs &a, hipStream_t st)
{
    lstm_forward_kernel<HT, KXT><<<a.NB, 64 * kLstmWaves, 0, st>>>(a);
    return hipGetLastError();
}

template <int HT, int KXT>
hipError_t run_bwd(const LstmBwdArgs &a, hipStream_t st)
{
    lstm_backward_kernel<HT, KXT><<<a.NB, 64 * kLstmWaves, 0, st>>>(a);
    return hipGetLastError();
}

#define ESRNN_LSTM_SHAPES(X) X(2, 1) X(2, 2) X(8, 2) X(8, 8) X(10, 1) X(10, 6) X(10, 10) X(13, 3) X(13, 13) X(16, 16)

}  // namespace

hipError_t launch_lstm_forward(const Plan &pl, int layer, float *ws, hipStream_t st)
{
    const LayerPlan &lp = pl.layer[layer];
    LstmFwdArgs a{ws + lp.wpack_fwd, ws + lp.bias_pack, ws + lp.xsrc, ws + lp.gates, ws + lp.c, ws + lp.hid,
                  lp.out ? ws + lp.resid : nullptr, lp.out ? ws + lp.out : nullptr, pl.P, pl.NB, lp.dil};
#define X(HT_, KXT_) if (pl.HT == HT_ && lp.KXT == KXT_) return run_fwd<HT_, KXT_>(a, st);
    ESRNN_LSTM_SHAPES(X)
#undef X
    return hipErrorInvalidValue;
}

hipError_t launch_lstm_backward(const Plan &pl, int layer, float *ws, hipStream_t st)
{
    const LayerPlan &lp = pl.layer[layer];
    LstmBwdArgs a{ws + lp.wpack_bwd, ws + lp.xsrc, ws + lp.gates, ws + lp.c, ws + lp.hid, ws + lp.gsrc, ws + lp.gdst,
                  lp.gadd ? ws + lp.gadd : nullptr, lp.dil >= 2 ? ws + lp.dhr : nullptr,
                  lp.dil >= 2 ? ws + lp.dcr : nullptr, ws + lp.dw_partial, ws + lp.db_partial, pl.P, pl.NB, lp.dil};
#define X(HT_, KXT_) if (pl.HT == HT_ && lp.KXT == KXT_) return run_bwd<HT_, KXT_>(a, st);
    ESRNN_LSTM_SHAPES(X)
#undef X
    return hipErrorInvalidValue;
}

}  // namespace esrnn
