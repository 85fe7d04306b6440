// Dilated LSTM layer, forward and reverse (Section 3.2, Table 1), one launch per
// layer.
//
// Parallel structure.  Series never interact, and a layer with dilation d is d
// independent recurrences over the interleaved position classes p = r (mod d).
// A workgroup of four waves (eight in one variant of the reverse pass, see
// there) therefore owns 16 series and one or more residue classes r (grid =
// series tiles x chains) and walks each class in order with the recurrent state
// on chip: h through LDS, c in registers.  There is no grid-level
// synchronisation and no recurrent traffic through global memory.
//
// Arithmetic.  The gate contraction runs on the 16x16x4 fp32 MFMA with the
// weights as the A operand, held in registers for the whole launch, and the
// activations [x_p ; h_{p-d}] of 16 series as the B operand.  Row order of the
// A operand: row 4g+r of unit tile mt is gate r of hidden unit 4mt+g.  A lane
// then holds the four gate pre-activations of one unit for one series (cell
// update without cross-lane traffic), and the hidden state it produces for unit
// tile mt is, as it stands, the B operand of k-step mt of the next position.
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
    const int32_t *pmax;  // [NB] positions the longest series of a tile has: the tile's chains stop there
    // cell-state penalty (Section 8.4) of a block's first layer, kernels instantiated with CP only
    const int32_t *lengths;
    float *cs_partial;    // [NB * gridDim.y] sums of squared cell states over valid window positions
    int B, T, I, H;
};

template <int HT, int KXT, bool CP>
__global__ void __launch_bounds__(64 * kLstmWaves, 2) lstm_forward_kernel(LstmFwdArgs a)
{
    constexpr int KT = KXT + HT;
    constexpr int MTW = (HT + kLstmWaves - 1) / kLstmWaves;   // unit tiles per wave
    // Waves 0 .. NX-1 own one unit tile more than the others.  Where that is at most two waves, wave s + 2
    // takes over the input part of the last tile of wave s (bias included) and hands the accumulators over
    // through LDS one position ahead: the input part does not depend on the recurrence, and the matrix work
    // per position becomes (nearly) the same on every wave.
    constexpr int NX = HT - kLstmWaves * (MTW - 1);
    constexpr bool kHelp = kLstmWaves == 4 && KXT >= 2 && MTW >= 2 && NX <= 2;
    __shared__ float hbuf[2][HT * 64];
    __shared__ f32x4 xfer[2][kHelp ? 2 : 1][64];

    const int lane = threadIdx.x & 63, bt = blockIdx.x;
    const int s = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave index, known to be uniform
    const int Pt = a.pmax[bt];      // positions past the tile's longest series are never computed (nor read later)
    const bool last_tile = s < NX;                              // this wave's last tile exists
    const bool helper = kHelp && s >= 2 && s - 2 < NX;          // its last slot holds the input part of wave s-2's last tile
    const bool last_x = kHelp ? helper : true;                  // input part of the last slot computed here

    float wreg[MTW][KT];
    f32x4 bias[MTW];
#pragma unroll
    for (int j = 0; j < MTW; ++j) {
        const int mt = (helper && j == MTW - 1 ? s - 2 : s) + kLstmWaves * j;
        const bool valid = mt < HT;
#pragma unroll
        for (int ks = 0; ks < KT; ++ks) wreg[j][ks] = valid ? a.wpack[((size_t)mt * KT + ks) * 64 + lane] : 0.0f;
        const float4 bv = valid ? *reinterpret_cast<const float4 *>(a.bpack + (mt * 4 + (lane >> 4)) * 4)
                                : make_float4(0.f, 0.f, 0.f, 0.f);
        bias[j] = f32x4{bv.x, bv.y, bv.z, bv.w};
    }
    const size_t xtile = (size_t)KXT * 64;
    // positions below this take part in the loss for this lane's series (CP only)
    int n_valid = 0;
    float csq = 0.0f;
    if constexpr (CP) {
        const int col = bt * kTileN + (lane & 15);
        const int len = col < a.B ? min(max(a.lengths[col], 0), a.T) : 0;
        n_valid = len - a.I - a.H + 1;
    }

    for (int r = blockIdx.y; r < a.d && r < Pt; r += gridDim.y) {
        // start of a chain: zero state
        float creg[MTW];
#pragma unroll
        for (int j = 0; j < MTW; ++j) creg[j] = 0.0f;
        for (int i = threadIdx.x; i < HT * 64; i += 64 * kLstmWaves) hbuf[0][i] = 0.0f;

        // input part of the first position
        float bx[KXT];
#pragma unroll
        for (int ks = 0; ks < KXT; ++ks) bx[ks] = (a.xsrc + ((size_t)r * a.NB + bt) * xtile + ks * 64)[lane];
        const unsigned lane4 = 4 * lane, lane16 = 16 * lane;   // this lane's bytes inside a tile
        f32x4 acc[MTW];
        // input part (with the bias) of one position; a helper's share first, so that it is complete when it
        // goes to LDS after the rest
        auto input_part = [&](int buf) {
#pragma unroll
            for (int j = 0; j < MTW; ++j) acc[j] = bias[j];
            if (last_x) {
#pragma unroll
                for (int ks = 0; ks < KXT; ++ks) acc[MTW - 1] = mfma16(wreg[MTW - 1][ks], bx[ks], acc[MTW - 1]);
            }
#pragma unroll
            for (int ks = 0; ks < KXT; ++ks)
#pragma unroll
                for (int j = 0; j < MTW - 1; ++j) acc[j] = mfma16(wreg[j][ks], bx[ks], acc[j]);
            if (helper) xfer[buf][kHelp ? s - 2 : 0][lane] = acc[MTW - 1];
        };
        input_part(0);
        {
            const buf_rsrc rx = make_rsrc(a.xsrc + ((size_t)min(r + a.d, Pt - 1) * a.NB + bt) * xtile);
#pragma unroll
            for (int ks = 0; ks < KXT; ++ks) bx[ks] = buf_load(rx, lane4, ks * 256);
        }
        // residual input of the block (last layer of a block >= 1), one position ahead like the input
        float res[MTW];
#pragma unroll
        for (int j = 0; j < MTW; ++j)
            res[j] = a.out ? (a.resid + (((size_t)r * a.NB + bt) * HT + min(s + kLstmWaves * j, HT - 1)) * 64)[lane] : 0.0f;
        lds_barrier();

        int it = 0;
        for (int p = r; p < Pt; p += a.d, ++it) {
            const size_t pb = (size_t)p * a.NB + bt;
            // this position's tiles of the stash and the outputs: scalar bases, scalar tile offsets
            const buf_rsrc r_gates = make_rsrc(a.gates + pb * HT * 256), r_c = make_rsrc(a.c + pb * HT * 64);
            const buf_rsrc r_hid = make_rsrc(a.hid + pb * HT * 64), r_out = make_rsrc(a.out + (a.out ? pb * HT * 64 : 0));
            float res_next[MTW];
            if (a.out) {
                const buf_rsrc rr = make_rsrc(a.resid + ((size_t)min(p + a.d, Pt - 1) * a.NB + bt) * HT * 64);
#pragma unroll
                for (int j = 0; j < MTW; ++j) res_next[j] = buf_load(rr, lane4, min(s + kLstmWaves * j, HT - 1) * 256);
            }
            // recurrent part
            const float *hb = hbuf[it & 1];
            float bh[HT];
#pragma unroll
            for (int ks = 0; ks < HT; ++ks) bh[ks] = hb[ks * 64 + lane];
            if (kHelp && last_tile) acc[MTW - 1] = xfer[it & 1][kHelp ? s : 0][lane];
            float *hn_buf = hbuf[(it + 1) & 1];
            // Tile by tile, one tile ahead on the matrix pipe: the MFMAs of tile j+1 are issued before the
            // activations of tile j, whose accumulator is complete by then (no drain of the pipe per tile).
            auto tile_mfma = [&](int j) {
#pragma unroll
                for (int ks = 0; ks < HT; ++ks) acc[j] = mfma16(wreg[j][KXT + ks], bh[ks], acc[j]);
            };
            auto tile_act = [&](int j) {
                const int mt = s + kLstmWaves * j;
                const float gi = sigmoid_f(acc[j][0]);
                const float gf = sigmoid_f(acc[j][1]);
                const float gg = tanh_f(acc[j][2]);
                const float go = sigmoid_f(acc[j][3]);
                const float cn = gf * creg[j] + gi * gg;
                const float hn = go * tanh_f(cn);
                creg[j] = cn;
                if constexpr (CP) csq += p < n_valid ? cn * cn : 0.0f;
                hn_buf[mt * 64 + lane] = hn;
                // gates and cell state are read again only by the reverse pass: streaming stores
                buf_store4<true>(r_gates, lane16, mt * 1024, f32x4{gi, gf, gg, go});
                buf_store<true>(r_c, lane4, mt * 256, cn);
                buf_store(r_hid, lane4, mt * 256, hn);
                if (a.out) buf_store(r_out, lane4, mt * 256, res[j] + hn);
            };
            // (with a one-tile input, KXT = 1, the plain order measured faster and is kept)
            constexpr bool kAhead = KXT >= 2;
            if (kAhead) tile_mfma(0);
#pragma unroll
            for (int j = 0; j < MTW; ++j) {
                if (kAhead) {
                    if (j + 1 < MTW - 1 || (j + 1 == MTW - 1 && last_tile)) tile_mfma(j + 1);
                } else {
                    if (j < MTW - 1 || last_tile) tile_mfma(j);
                }
                if (j < MTW - 1 || last_tile) tile_act(j);
            }
            // input part of the next position of the chain: independent of the
            // recurrence, so it runs on the matrix pipe while the waves meet at
            // the barrier
            if (p + a.d < Pt) {
                input_part((it + 1) & 1);
                const buf_rsrc rx = make_rsrc(a.xsrc + ((size_t)min(p + 2 * a.d, Pt - 1) * a.NB + bt) * xtile);
#pragma unroll
                for (int ks = 0; ks < KXT; ++ks) bx[ks] = buf_load(rx, lane4, ks * 256);
            }
            if (a.out) {
#pragma unroll
                for (int j = 0; j < MTW; ++j) res[j] = res_next[j];
            }
            lds_barrier();
        }
    }
    if constexpr (CP) {
        __shared__ float s_cs[kLstmWaves];
        const float tot = wave_sum(csq);
        if (lane == 0) s_cs[s] = tot;
        __syncthreads();
        if (threadIdx.x == 0)
            a.cs_partial[blockIdx.x * gridDim.y + blockIdx.y] = (s_cs[0] + s_cs[1]) + (s_cs[2] + s_cs[3]);
    }
}

// ---------------------------------------------------------------------------
// Reverse pass of one layer.  Per position p of a chain (descending):
//   A. every lane turns (dh, dc) of its hidden unit into the four gate
//      pre-activation gradients da (registers), and leaves them in LDS next to
//      [x_p ; h_{p-d}] for step C;
//   B. transposed contraction d[x_p ; h_{p-d}] = W^T da on the MFMA, split over
//      the waves along the contraction: a wave multiplies the k-steps of the
//      units it owns, whose da it has just computed, so no operand crosses
//      waves; the four partial results meet in LDS and every wave sums the
//      output tiles it needs next (the recurrent dh of its own units) in a
//      fixed order.  The row order of the output tiles (row 4g+r of tile mb is
//      row g of input unit tile 4mb+r) keeps the result one unit tile per 64
//      lanes;
//   C. weight gradient dW += da (x) [x_p ; h_{p-d}]: contraction over the 16
//      series on the MFMA, both operands read transposed from LDS; whole rows
//      of tiles per wave, in accumulators for the whole launch.  Rows go to the
//      waves in reverse order of unit ownership, which evens out the MFMA
//      count of B plus C.
// The loop is software-pipelined: the MFMAs of C(p) are issued together with
// the elementwise work of A(p-d), whose global operands were requested one
// position earlier.  fp32 MFMAs and vector instructions of a SIMD do not run at
// the same time on this chip (esrnn_probe_issue_overlap measures it): what the
// elementwise work and the address arithmetic cost is taken from the matrix
// pipe, so both are kept short.
// ---------------------------------------------------------------------------
struct LstmBwdArgs {
    const float *wpack;   // [MB][4*HT][64]
    const float *xsrc;    // TL(4*KXT)
    const float *gates, *c, *hid;
    const float *gsrc[2]; // TL(HP): the gradient arriving at the hidden output is the sum of these
    int n_gsrc;           // 1 or 2; gsrc[1] repeats gsrc[0] when there is one
    float *gdst;          // TL(4*KXT)
    float *sink;          // [kSinkLines][64] floats that nothing reads: target of the stores a wave has no input tile for
    float *dw_partial;    // [NB*chains][HT*MB][4][64]
    float *db_partial;    // [NB*chains][HT][4][4]
    int P, NB, d;
    const int32_t *pmax;  // [NB] positions the longest series of a tile has: the tile's chains stop there
    // cell-state penalty (Section 8.4) of a block's first layer, kernels instantiated with CP only
    const int32_t *lengths;
    const Scalars *sc;
    float two_lambda_cs;
    int B, T, I, H;
};

template <int HT, int KXT, bool CP>
__global__ void __launch_bounds__(64 * kLstmWaves, (HT <= 10 ? 2 : 1)) lstm_backward_kernel(LstmBwdArgs a)
{
    constexpr int W = kLstmWaves;
    constexpr int KT = KXT + HT;
    constexpr int MB = (KT + 3) / 4;                 // 16-row tiles of [x ; h]
    constexpr int MTW = (HT + W - 1) / W;            // unit tiles per wave
    constexpr int QXW = (KXT + W - 1) / W;           // input unit tiles finalised per wave
    constexpr int NT = 64 * W;
    constexpr int DA_ROWS = 16 * W * MTW;            // includes dummy rows for tiles past HT
    constexpr int XH_PER_THREAD = (KT * 64 + NT - 1) / NT;
    constexpr int XH_ROWS = (16 * MB > 16 * XH_PER_THREAD) ? 16 * MB : 16 * XH_PER_THREAD;

    __shared__ float da_lds[DA_ROWS * kLdsPad];      // [mt][4*gate + unit][series]
    __shared__ float xh_lds[XH_ROWS * kLdsPad];      // [row of x ; h][series]; rows past 4*KT are scratch
    __shared__ float part_lds[W][MB * 4][64];        // partial d[x ; h] of every wave
    static_assert((DA_ROWS * kLdsPad + XH_ROWS * kLdsPad + W * MB * 4 * 64) * 4 <= 128 * 1024, "LDS budget of the reverse kernel");

    const int lane = threadIdx.x & 63, bt = blockIdx.x;
    const int s = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave index, known to be uniform
    const int Pt = a.pmax[bt];      // the chains of this tile stop at its longest series
    const int g = lane >> 4, n = lane & 15;
    const bool last_own_valid = s + W * (MTW - 1) < HT;           // unit tile s + 4(MTW-1)
    const bool last_row_valid = (W - 1 - s) + W * (MTW - 1) < HT; // dW row (3-s) + 4(MTW-1)
    const bool last_qx_valid = s + W * (QXW - 1) < KXT;
    float *sink_line = a.sink + ((bt + blockIdx.y * 61) % kSinkLines) * 64;

    // W^T operands of the k-steps this wave owns: k-step 4*mt + gate, mt = s + 4j
    float wreg[MB][4 * MTW];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int j = 0; j < MTW; ++j) {
            const int mt = s + W * j;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float w = a.wpack[((size_t)mb * 4 * HT + 4 * min(mt, HT - 1) + r) * 64 + lane];
                wreg[mb][4 * j + r] = mt < HT ? w : 0.0f;
            }
        }
    f32x4 dw[MTW][MB];
    f32x4 dbacc[MTW];
#pragma unroll
    for (int j = 0; j < MTW; ++j) {
        dbacc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int nbk = 0; nbk < MB; ++nbk) dw[j][nbk] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    for (int i = threadIdx.x; i < XH_ROWS * kLdsPad; i += NT) xh_lds[i] = 0.0f;
    for (int i = threadIdx.x; i < DA_ROWS * kLdsPad; i += NT) da_lds[i] = 0.0f;

    const size_t xtile = (size_t)KXT * 64, htile = (size_t)HT * 64;

    // ---- operands of one position, requested one position ahead.  Branch-free:
    // tiles past HT alias the last tile, a missing predecessor aliases p itself,
    // elements past the end of [x ; h] alias its last element.
    float4 pf_gt[MTW];
    float pf_c[MTW], pf_cp[MTW], pf_g[MTW], pf_g2[MTW], pf_xh[XH_PER_THREAD];
    // `first`: the chain's first request.  Later ones follow a request for position p + d, whose predecessor
    // cell state c[p] is still in registers: it is not read from memory a second time.
    // The requests of a position go out piece by piece, each as soon as the registers it fills are free:
    // [x ; h] after it has gone to LDS, the operands of unit tile j after the elementwise step of tile j.
    // Buffer addressing: the tiles of a position sit behind scalar bases, a tile is a scalar byte offset, the
    // lane's share a fixed 32-bit offset - no address arithmetic on the vector ALU.
    const unsigned lane4 = 4 * lane, lane16 = 16 * lane;
    auto fetch_xh = [&](int p) {
        const size_t pb = (size_t)p * a.NB + bt;
        const size_t pbd = (size_t)(p >= a.d ? p - a.d : p) * a.NB + bt;
#pragma unroll
        for (int i = 0; i < XH_PER_THREAD; ++i) {
            // unit tile s + W*i of [x ; h]; tiles past the end alias the last one.  One request whichever array
            // the tile is in (a scalar choice of the base, no branch around the request)
            const int q = min(s + W * i, KT - 1);
            const float *src = q < KXT ? a.xsrc + pb * xtile + q * 64 : a.hid + pbd * htile + (q - KXT) * 64;
            pf_xh[i] = buf_load(make_rsrc(src), lane4, 0);
        }
    };
    auto fetch_tile = [&](int j, int p, bool first) {
        const size_t pb = (size_t)p * a.NB + bt;
        const size_t pbd = (size_t)(p >= a.d ? p - a.d : p) * a.NB + bt;
        const int mt = __builtin_amdgcn_readfirstlane(min(s + W * j, HT - 1));   // (known to be uniform)
        const f32x4 gt = buf_load4(make_rsrc(a.gates + pb * htile * 4), lane16, mt * 1024);
        pf_gt[j] = make_float4(gt[0], gt[1], gt[2], gt[3]);
        pf_c[j] = first ? buf_load(make_rsrc(a.c + pb * htile), lane4, mt * 256) : pf_cp[j];
        pf_cp[j] = buf_load(make_rsrc(a.c + pbd * htile), lane4, mt * 256);
        pf_g[j] = buf_load(make_rsrc(a.gsrc[0] + pb * htile), lane4, mt * 256);
        pf_g2[j] = buf_load(make_rsrc(a.gsrc[1] + pb * htile), lane4, mt * 256);   // gsrc[1] repeats gsrc[0] when there is one source (ignored then)
    };
    auto fetch = [&](int p, bool first) {
        fetch_xh(p);
#pragma unroll
        for (int j = 0; j < MTW; ++j) fetch_tile(j, p, first);
    };

    const float g2_scale = a.n_gsrc >= 2 ? 1.0f : 0.0f;
    // d/dc of lambda * c^2 / n over the valid window positions of this lane's series (CP only)
    int n_valid = 0;
    float pen = 0.0f;
    if constexpr (CP) {
        const int col = bt * kTileN + n;
        const int len = col < a.B ? min(max(a.lengths[col], 0), a.T) : 0;
        n_valid = len - a.I - a.H + 1;
        pen = a.two_lambda_cs * a.sc->inv_n_cs;
    }
    float dcreg[MTW], dhreg[MTW];
    float da[MTW][4];
    // ---- step A, tile j of the fetched position: gate gradients to registers and LDS
    auto step_a_tile = [&](int j, bool has_prev, int p_cur) {
        const float4 gt = pf_gt[j];
        const float dh = pf_g[j] + g2_scale * pf_g2[j] + dhreg[j];
        const float tc = tanh_f(pf_c[j]);
        // (products shared between the terms are formed once: the vector ALU's cycles are the matrix pipe's)
        const float dh_o = dh * gt.w;
        float dc = dcreg[j] + dh_o * (1.0f - tc * tc);
        if constexpr (CP) dc += p_cur < n_valid ? pen * pf_c[j] : 0.0f;
        const float cp = has_prev ? pf_cp[j] : 0.0f;
        const float dc_i = dc * gt.x, dc_f = dc * gt.y;
        da[j][0] = dc_i * gt.z * (1.0f - gt.x);
        da[j][1] = dc_f * cp * (1.0f - gt.y);
        da[j][2] = dc_i * (1.0f - gt.z * gt.z);
        da[j][3] = dh_o * tc * (1.0f - gt.w);
        dcreg[j] = dc_f;
        float *dst = da_lds + ((s + W * j) * 16 + g) * kLdsPad + n;   // dummy rows for tiles past HT
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            dst[r * 4 * kLdsPad] = da[j][r];
            dbacc[j][r] += da[j][r];
        }
    };
    auto store_xh = [&](bool has_prev) {
#pragma unroll
        for (int i = 0; i < XH_PER_THREAD; ++i) {
            const int e = threadIdx.x + i * NT;
            xh_lds[(e >> 4) * kLdsPad + (e & 15)] = (e < KXT * 64 || has_prev) ? pf_xh[i] : 0.0f;
        }
    };
    // ---- step B: partial W^T da over this wave's k-steps, into LDS
    auto step_b = [&]() {
        f32x4 acc[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) acc[mb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < MTW - 1; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) acc[mb] = mfma16(wreg[mb][4 * j + r], da[j][r], acc[mb]);
        if (last_own_valid) {
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
                    acc[mb] = mfma16(wreg[mb][4 * (MTW - 1) + r], da[MTW - 1][r], acc[mb]);
        }
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int r = 0; r < 4; ++r) part_lds[s][mb * 4 + r][lane] = acc[mb][r];
    };
    // ---- end of position p: sum the partials this wave needs (recurrent dh of its
    // units) or stores (input gradient), and pull the operands of step C into registers
    float xb[MB][4], ar[MTW][4], dxv[QXW];
    auto finish = [&](int p) {
        lds_barrier();              // partials, da, [x ; h] of position p complete
#pragma unroll
        for (int j = 0; j < MTW; ++j) {
            const int q = min(KXT + s + W * j, KT - 1);   // row of part_lds = unit tile of [x ; h]
            dhreg[j] = (part_lds[0][q][lane] + part_lds[1][q][lane]) + (part_lds[2][q][lane] + part_lds[3][q][lane]);
        }
#pragma unroll
        for (int j = 0; j < QXW; ++j) {
            const int q = min(s + W * j, KXT - 1);
            dxv[j] = (part_lds[0][q][lane] + part_lds[1][q][lane]) + (part_lds[2][q][lane] + part_lds[3][q][lane]);
        }
#pragma unroll
        for (int nbk = 0; nbk < MB; ++nbk)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) xb[nbk][ks] = xh_lds[(nbk * 16 + n) * kLdsPad + 4 * ks + g];
#pragma unroll
        for (int j = 0; j < MTW; ++j)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
                ar[j][ks] = da_lds[(((W - 1 - s) + W * j) * 16 + n) * kLdsPad + 4 * ks + g];
        lds_barrier();              // everything of position p has been read
    };
    // Memory operations complete in order, and the compiler's wait for the operands requested one
    // position ahead counts the stores issued since with the smallest number any wave issues.  Every
    // wave therefore issues the same number of stores: one without an input tile for its last store
    // writes to a sink.  The stores go out right after the sums, behind the requests already in flight
    // (which then do not wait for them) and a whole position ahead of the next wait.
    auto store_dx = [&](int p) {
        const size_t pb = (size_t)p * a.NB + bt;
        const buf_rsrc r_dx = make_rsrc(a.gdst + pb * xtile), r_sink = make_rsrc(sink_line);
#pragma unroll
        for (int j = 0; j < QXW; ++j) {
            if (j < QXW - 1 || last_qx_valid) buf_store(r_dx, lane4, (s + W * j) * 256, dxv[j]);
            else buf_store(r_sink, lane4, 0, dxv[j]);
        }
    };
    auto dw_row = [&](int j) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int nbk = 0; nbk < MB; ++nbk) dw[j][nbk] = mfma16(ar[j][ks], xb[nbk][ks], dw[j][nbk]);
    };

    for (int r0 = blockIdx.y; r0 < a.d && r0 < Pt; r0 += gridDim.y) {
        const int p_last = r0 + ((Pt - 1 - r0) / a.d) * a.d;
        // start of a chain: no gradient arrives from later positions
#pragma unroll
        for (int j = 0; j < MTW; ++j) { dcreg[j] = 0.0f; dhreg[j] = 0.0f; }
        __syncthreads();            // LDS free (previous chain / initial clearing)
        fetch(p_last, true);
        store_xh(p_last >= a.d);
#pragma unroll
        for (int j = 0; j < MTW; ++j) step_a_tile(j, p_last >= a.d, p_last);
        fetch(max(p_last - a.d, r0), false);
        step_b();

        for (int p = p_last; p >= a.d; p -= a.d) {
            finish(p);
            store_dx(p);
            // gate gradients of position p - d (elementwise) interleaved with the dW MFMAs of p and with
            // the requests for position p - 2d
            const bool has_prev = p >= 2 * a.d;
            const int p_next = max(p - 2 * a.d, r0);
            store_xh(has_prev);
            fetch_xh(p_next);
#pragma unroll
            for (int j = 0; j < MTW - 1; ++j) {
                step_a_tile(j, has_prev, p - a.d);
                fetch_tile(j, p_next, false);
                dw_row(j);
            }
            step_a_tile(MTW - 1, has_prev, p - a.d);
            fetch_tile(MTW - 1, p_next, false);
            if (last_row_valid) dw_row(MTW - 1);
            step_b();
        }
        finish(r0);
        store_dx(r0);
#pragma unroll
        for (int j = 0; j < MTW - 1; ++j) dw_row(j);
        if (last_row_valid) dw_row(MTW - 1);
    }

    // per-workgroup partial results
    const size_t part = (size_t)bt * gridDim.y + blockIdx.y;
#pragma unroll
    for (int j = 0; j < MTW; ++j) {
        const int row = (W - 1 - s) + W * j;
        if (row < HT) {
#pragma unroll
            for (int nbk = 0; nbk < MB; ++nbk) {
                float *dst = a.dw_partial + (part * (HT * MB) + row * MB + nbk) * 256 + lane;
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) dst[rr * 64] = dw[j][nbk][rr];
            }
        }
    }
#pragma unroll
    for (int j = 0; j < MTW; ++j) {
        const int mt = s + W * j;
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            const float tot = group16_sum(dbacc[j][rr]);
            if (n == 0 && mt < HT) a.db_partial[(part * HT + mt) * 16 + g * 4 + rr] = tot;
        }
    }
}

// ---------------------------------------------------------------------------
// Reverse pass with the weight gradient on waves of its own.  Steps A and B are
// the recurrence: position p - d cannot start before the recurrent dh of p is
// summed.  Step C only consumes what A leaves in LDS.  Here four "chain" waves
// do A and B exactly as above, and four "dW" waves do C one position behind
// them: after the barrier that completes position p they read da and [x ; h] of
// p from one LDS copy while the chain waves fill the other copy with p - d.
// The matrix pipe of a SIMD then has the dW wave's work whenever its chain wave
// waits (barrier, LDS round trip, accumulator read-out), and the chain waves
// carry half the MFMAs per position.  One workgroup of eight waves per compute
// unit; one barrier per position, taken by all eight waves.
// ---------------------------------------------------------------------------
template <int HT, int KXT, bool CP>
__global__ void __launch_bounds__(128 * kLstmWaves, 1) lstm_backward_split_kernel(LstmBwdArgs a)
{
    constexpr int W = kLstmWaves;
    constexpr int KT = KXT + HT;
    constexpr int MB = (KT + 3) / 4;                 // 16-row tiles of [x ; h]
    constexpr int MTW = (HT + W - 1) / W;            // unit tiles per wave
    constexpr int QXW = (KXT + W - 1) / W;           // input unit tiles finalised per wave
    constexpr int NT = 64 * W;                       // threads of the chain waves
    constexpr int DA_ROWS = 16 * W * MTW;            // includes dummy rows for tiles past HT
    constexpr int XH_PER_THREAD = (KT * 64 + NT - 1) / NT;
    constexpr int XH_ROWS = (16 * MB > 16 * XH_PER_THREAD) ? 16 * MB : 16 * XH_PER_THREAD;

    __shared__ float da_lds[2][DA_ROWS * kLdsPad];   // [mt][4*gate + unit][series]
    __shared__ float xh_lds[2][XH_ROWS * kLdsPad];   // [row of x ; h][series]; rows past 4*KT are scratch
    __shared__ float part_lds[2][W][MB * 4][64];     // partial d[x ; h] of every chain wave
    static_assert(2 * (DA_ROWS * kLdsPad + XH_ROWS * kLdsPad + W * MB * 4 * 64) * 4 <= 128 * 1024,
                  "LDS budget of the reverse kernel");

    const int lane = threadIdx.x & 63, bt = blockIdx.x;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave index, known to be uniform
    const bool chain = wv < W;
    const int s = wv & (W - 1);
    const int Pt = a.pmax[bt];      // the chains of this tile stop at its longest series
    const int g = lane >> 4, n = lane & 15;
    for (int i = threadIdx.x; i < 2 * XH_ROWS * kLdsPad; i += 2 * NT) (&xh_lds[0][0])[i] = 0.0f;
    for (int i = threadIdx.x; i < 2 * DA_ROWS * kLdsPad; i += 2 * NT) (&da_lds[0][0])[i] = 0.0f;
    const size_t part = (size_t)bt * gridDim.y + blockIdx.y;

    if (!chain) {
        // ---- dW waves: rows (W-1-s) + W*j of the weight gradient, in accumulators for the whole launch
        const bool last_row_valid = (W - 1 - s) + W * (MTW - 1) < HT;
        f32x4 dw[MTW][MB];
#pragma unroll
        for (int j = 0; j < MTW; ++j)
#pragma unroll
            for (int nbk = 0; nbk < MB; ++nbk) dw[j][nbk] = f32x4{0.f, 0.f, 0.f, 0.f};
        auto accumulate = [&](int buf) {
            lds_barrier();          // da and [x ; h] of the position are complete in copy `buf`
            float xb[MB][4], ar[MTW][4];
#pragma unroll
            for (int nbk = 0; nbk < MB; ++nbk)
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) xb[nbk][ks] = xh_lds[buf][(nbk * 16 + n) * kLdsPad + 4 * ks + g];
#pragma unroll
            for (int j = 0; j < MTW; ++j)
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
                    ar[j][ks] = da_lds[buf][(((W - 1 - s) + W * j) * 16 + n) * kLdsPad + 4 * ks + g];
#pragma unroll
            for (int j = 0; j < MTW; ++j)
                if (j < MTW - 1 || last_row_valid) {
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                        for (int nbk = 0; nbk < MB; ++nbk) dw[j][nbk] = mfma16(ar[j][ks], xb[nbk][ks], dw[j][nbk]);
                }
        };
        for (int r0 = blockIdx.y; r0 < a.d && r0 < Pt; r0 += gridDim.y) {
            const int p_last = r0 + ((Pt - 1 - r0) / a.d) * a.d;
            __syncthreads();
            int buf = 0;
            for (int p = p_last; p >= a.d; p -= a.d) {
                accumulate(buf);
                buf ^= 1;
            }
            accumulate(buf);
        }
#pragma unroll
        for (int j = 0; j < MTW; ++j) {
            const int row = (W - 1 - s) + W * j;
            if (row < HT) {
#pragma unroll
                for (int nbk = 0; nbk < MB; ++nbk) {
                    float *dst = a.dw_partial + (part * (HT * MB) + row * MB + nbk) * 256 + lane;
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) dst[rr * 64] = dw[j][nbk][rr];
                }
            }
        }
        return;
    }

    // ---- chain waves: steps A and B
    const bool last_own_valid = s + W * (MTW - 1) < HT;           // unit tile s + 4(MTW-1)
    const bool last_qx_valid = s + W * (QXW - 1) < KXT;
    float *sink_line = a.sink + ((bt + blockIdx.y * 61) % kSinkLines) * 64;
    // W^T operands of the k-steps this wave owns: k-step 4*mt + gate, mt = s + 4j
    float wreg[MB][4 * MTW];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int j = 0; j < MTW; ++j) {
            const int mt = s + W * j;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float w = a.wpack[((size_t)mb * 4 * HT + 4 * min(mt, HT - 1) + r) * 64 + lane];
                wreg[mb][4 * j + r] = mt < HT ? w : 0.0f;
            }
        }
    f32x4 dbacc[MTW];
#pragma unroll
    for (int j = 0; j < MTW; ++j) dbacc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    const size_t xtile = (size_t)KXT * 64, htile = (size_t)HT * 64;

    // operands of one position, requested one position ahead (branch-free, see the kernel above)
    float4 pf_gt[MTW];
    float pf_c[MTW], pf_cp[MTW], pf_g[MTW], pf_g2[MTW], pf_xh[XH_PER_THREAD];
    // The requests of a position go out piece by piece, each as soon as the registers it fills are free:
    // [x ; h] after it has gone to LDS, the operands of unit tile j after the elementwise step of tile j.
    auto fetch_xh = [&](int p) {
        const size_t pb = (size_t)p * a.NB + bt;
        const size_t pbd = (size_t)(p >= a.d ? p - a.d : p) * a.NB + bt;
#pragma unroll
        for (int i = 0; i < XH_PER_THREAD; ++i) {
            // unit tile s + W*i of [x ; h]; tiles past the end alias the last one
            const int q = min(s + W * i, KT - 1);
            const float *src = q < KXT ? a.xsrc + pb * xtile + q * 64 : a.hid + pbd * htile + (q - KXT) * 64;
            pf_xh[i] = src[lane];
        }
    };
    auto fetch_tile = [&](int j, int p, bool first) {
        const size_t pb = (size_t)p * a.NB + bt;
        const size_t pbd = (size_t)(p >= a.d ? p - a.d : p) * a.NB + bt;
        // wave-uniform tile bases plus the lane index: scalar address arithmetic
        const int mt = min(s + W * j, HT - 1);
        const size_t tile = (pb * HT + mt) * 64;
        pf_gt[j] = (reinterpret_cast<const float4 *>(a.gates) + tile)[lane];
        pf_c[j] = first ? (a.c + tile)[lane] : pf_cp[j];
        pf_cp[j] = (a.c + (pbd * HT + mt) * 64)[lane];
        pf_g[j] = (a.gsrc[0] + tile)[lane];
        pf_g2[j] = (a.gsrc[1] + tile)[lane];    // gsrc[1] repeats gsrc[0] when there is one source (ignored then)
    };
    auto fetch = [&](int p, bool first) {
        fetch_xh(p);
#pragma unroll
        for (int j = 0; j < MTW; ++j) fetch_tile(j, p, first);
    };
    const float g2_scale = a.n_gsrc >= 2 ? 1.0f : 0.0f;
    int n_valid = 0;
    float pen = 0.0f;
    if constexpr (CP) {
        const int col = bt * kTileN + n;
        const int len = col < a.B ? min(max(a.lengths[col], 0), a.T) : 0;
        n_valid = len - a.I - a.H + 1;
        pen = a.two_lambda_cs * a.sc->inv_n_cs;
    }
    float dcreg[MTW], dhreg[MTW];
    float da[MTW][4];
    auto step_a_tile = [&](int j, bool has_prev, int p_cur, int buf) {
        const float4 gt = pf_gt[j];
        const float dh = pf_g[j] + g2_scale * pf_g2[j] + dhreg[j];
        const float tc = tanh_f(pf_c[j]);
        // (products shared between the terms are formed once: the vector ALU's cycles are the matrix pipe's)
        const float dh_o = dh * gt.w;
        float dc = dcreg[j] + dh_o * (1.0f - tc * tc);
        if constexpr (CP) dc += p_cur < n_valid ? pen * pf_c[j] : 0.0f;
        const float cp = has_prev ? pf_cp[j] : 0.0f;
        const float dc_i = dc * gt.x, dc_f = dc * gt.y;
        da[j][0] = dc_i * gt.z * (1.0f - gt.x);
        da[j][1] = dc_f * cp * (1.0f - gt.y);
        da[j][2] = dc_i * (1.0f - gt.z * gt.z);
        da[j][3] = dh_o * tc * (1.0f - gt.w);
        dcreg[j] = dc_f;
        float *dst = da_lds[buf] + ((s + W * j) * 16 + g) * kLdsPad + n;   // dummy rows for tiles past HT
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            dst[r * 4 * kLdsPad] = da[j][r];
            dbacc[j][r] += da[j][r];
        }
    };
    auto store_xh = [&](bool has_prev, int buf) {
#pragma unroll
        for (int i = 0; i < XH_PER_THREAD; ++i) {
            const int e = threadIdx.x + i * NT;
            xh_lds[buf][(e >> 4) * kLdsPad + (e & 15)] = (e < KXT * 64 || has_prev) ? pf_xh[i] : 0.0f;
        }
    };
    auto step_b = [&](int buf) {
        f32x4 acc[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) acc[mb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < MTW - 1; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) acc[mb] = mfma16(wreg[mb][4 * j + r], da[j][r], acc[mb]);
        if (last_own_valid) {
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
                    acc[mb] = mfma16(wreg[mb][4 * (MTW - 1) + r], da[MTW - 1][r], acc[mb]);
        }
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int r = 0; r < 4; ++r) part_lds[buf][s][mb * 4 + r][lane] = acc[mb][r];
    };
    float dxv[QXW];
    auto finish = [&](int buf) {
        lds_barrier();              // partials, da, [x ; h] of the position complete
        const float (*pt)[MB * 4][64] = part_lds[buf];
#pragma unroll
        for (int j = 0; j < MTW; ++j) {
            const int q = min(KXT + s + W * j, KT - 1);   // row of part_lds = unit tile of [x ; h]
            dhreg[j] = (pt[0][q][lane] + pt[1][q][lane]) + (pt[2][q][lane] + pt[3][q][lane]);
        }
#pragma unroll
        for (int j = 0; j < QXW; ++j) {
            const int q = min(s + W * j, KXT - 1);
            dxv[j] = (pt[0][q][lane] + pt[1][q][lane]) + (pt[2][q][lane] + pt[3][q][lane]);
        }
    };
    auto store_dx = [&](int p) {     // every wave issues the same number of stores (see the kernel above)
        const size_t pb = (size_t)p * a.NB + bt;
#pragma unroll
        for (int j = 0; j < QXW; ++j) {
            float *dst = (j < QXW - 1 || last_qx_valid) ? a.gdst + pb * xtile + (s + W * j) * 64 : sink_line;
            dst[lane] = dxv[j];
        }
    };

    for (int r0 = blockIdx.y; r0 < a.d && r0 < Pt; r0 += gridDim.y) {
        const int p_last = r0 + ((Pt - 1 - r0) / a.d) * a.d;
#pragma unroll
        for (int j = 0; j < MTW; ++j) { dcreg[j] = 0.0f; dhreg[j] = 0.0f; }
        __syncthreads();            // LDS free (previous chain / initial clearing)
        int buf = 0;
        fetch(p_last, true);
        store_xh(p_last >= a.d, buf);
#pragma unroll
        for (int j = 0; j < MTW; ++j) step_a_tile(j, p_last >= a.d, p_last, buf);
        fetch(max(p_last - a.d, r0), false);
        step_b(buf);
        for (int p = p_last; p >= a.d; p -= a.d) {
            finish(buf);
            buf ^= 1;               // position p - d goes to the other copy
            store_dx(p);
            const bool has_prev = p >= 2 * a.d;
            const int p_next = max(p - 2 * a.d, r0);
            store_xh(has_prev, buf);
            fetch_xh(p_next);
#pragma unroll
            for (int j = 0; j < MTW; ++j) {
                step_a_tile(j, has_prev, p - a.d, buf);
                fetch_tile(j, p_next, false);
            }
            step_b(buf);
        }
        finish(buf);
        store_dx(r0);
    }
#pragma unroll
    for (int j = 0; j < MTW; ++j) {
        const int mt = s + W * j;
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            const float tot = group16_sum(dbacc[j][rr]);
            if (n == 0 && mt < HT) a.db_partial[(part * HT + mt) * 16 + g * 4 + rr] = tot;
        }
    }
}

// out = a + b (+ c): gradient sources of a layer behind three or more residual blocks
__global__ void __launch_bounds__(256) sum_sources_kernel(const float4 *__restrict__ a, const float4 *__restrict__ b,
                                                           const float4 *__restrict__ c, float4 *__restrict__ out, size_t n)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    float4 v = a[i];
    const float4 w = b[i];
    v.x += w.x; v.y += w.y; v.z += w.z; v.w += w.w;
    if (c) {
        const float4 u = c[i];
        v.x += u.x; v.y += u.y; v.z += u.z; v.w += u.w;
    }
    out[i] = v;
}

template <int HT, int KXT>
hipError_t run_fwd(const LstmFwdArgs &a, int chains, hipStream_t st)
{
    if (a.cs_partial) lstm_forward_kernel<HT, KXT, true><<<dim3(a.NB, chains), 64 * kLstmWaves, 0, st>>>(a);
    else lstm_forward_kernel<HT, KXT, false><<<dim3(a.NB, chains), 64 * kLstmWaves, 0, st>>>(a);
    return hipGetLastError();
}

template <int HT, int KXT>
hipError_t run_bwd(const LstmBwdArgs &a, int chains, bool split, hipStream_t st)
{
    if (split || HT >= kSplitBwdFromHT) {
        if (a.sc) lstm_backward_split_kernel<HT, KXT, true><<<dim3(a.NB, chains), 128 * kLstmWaves, 0, st>>>(a);
        else lstm_backward_split_kernel<HT, KXT, false><<<dim3(a.NB, chains), 128 * kLstmWaves, 0, st>>>(a);
    } else if constexpr (HT < kSplitBwdFromHT) {   // (the four-wave kernel is not built for the larger hidden sizes)
        if (a.sc) lstm_backward_kernel<HT, KXT, true><<<dim3(a.NB, chains), 64 * kLstmWaves, 0, st>>>(a);
        else lstm_backward_kernel<HT, KXT, false><<<dim3(a.NB, chains), 64 * kLstmWaves, 0, st>>>(a);
    }
    return hipGetLastError();
}

#define ESRNN_LSTM_SHAPES(X) \
    X(2, 1) X(2, 2) X(8, 2) X(8, 3) X(8, 8) X(10, 1) X(10, 3) X(10, 6) X(10, 8) X(10, 10) X(13, 3) X(13, 5) X(13, 13) X(16, 16)

}  // namespace

hipError_t launch_lstm_forward(const Plan &pl, int layer, const int32_t *lengths, const float *weights, float *ws,
                               hipStream_t st)
{
    const LayerPlan &lp = pl.layer[layer];
    if (lp.narrow) return launch_lstm_forward_narrow(pl, layer, lengths, weights, ws, st);
    const bool cp = lp.first_in_block && pl.cfg.lambda_cs != 0.0f;
    LstmFwdArgs a{ws + lp.wpack_fwd, ws + lp.bias_pack, ws + lp.xsrc, ws + lp.gates, ws + lp.c, ws + lp.hid,
                  lp.out ? ws + lp.resid : nullptr, lp.out ? ws + lp.out : nullptr, pl.P, pl.NB, lp.dil,
                  reinterpret_cast<const int32_t *>(ws + pl.pmax),
                  lengths, cp ? ws + lp.cs_partial : nullptr, pl.B, pl.T, pl.I, pl.H};
#define X(HT_, KXT_) if (pl.HT == HT_ && lp.KXT == KXT_) return run_fwd<HT_, KXT_>(a, lp.chains, st);
    ESRNN_LSTM_SHAPES(X)
#undef X
    return hipErrorInvalidValue;
}

hipError_t launch_lstm_backward(const Plan &pl, int layer, const int32_t *lengths, float *ws, hipStream_t st)
{
    const LayerPlan &lp = pl.layer[layer];
    LstmBwdArgs a{};
    const bool cp = lp.first_in_block && pl.cfg.lambda_cs != 0.0f;
    a.lengths = lengths;
    a.sc = cp ? reinterpret_cast<const Scalars *>(ws + pl.scalars) : nullptr;
    a.two_lambda_cs = 2.0f * pl.cfg.lambda_cs;
    a.B = pl.B; a.T = pl.T; a.I = pl.I; a.H = pl.H;
    a.wpack = ws + lp.wpack_bwd; a.xsrc = ws + lp.xsrc; a.gates = ws + lp.gates; a.c = ws + lp.c; a.hid = ws + lp.hid;
    a.n_gsrc = lp.n_gsrc < 2 ? lp.n_gsrc : 2;
    a.gsrc[0] = ws + lp.gsrc[0];
    a.gsrc[1] = ws + lp.gsrc[lp.n_gsrc >= 2 ? 1 : 0];
    if (lp.n_gsrc > 2) {
        // three or more residual blocks: the sources past the first are summed into a buffer of their
        // own first (they stay intact for the layers that consume them separately)
        const size_t n4 = (size_t)pl.P * pl.NB * pl.HT * 16;   // float4 elements of a TL(HP) array
        const float *s3 = lp.n_gsrc > 3 ? ws + lp.gsrc[3] : nullptr;
        sum_sources_kernel<<<(unsigned)((n4 + 255) / 256), 256, 0, st>>>(
            reinterpret_cast<const float4 *>(ws + lp.gsrc[1]), reinterpret_cast<const float4 *>(ws + lp.gsrc[2]),
            reinterpret_cast<const float4 *>(s3), reinterpret_cast<float4 *>(ws + pl.gsum), n4);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        a.gsrc[1] = ws + pl.gsum;
    }
    if (lp.narrow) return launch_lstm_backward_narrow(pl, layer, lengths, ws, st);
    a.gdst = ws + lp.gdst; a.dw_partial = ws + lp.dw_partial; a.db_partial = ws + lp.db_partial;
    a.sink = ws + pl.sink;
    a.P = pl.P; a.NB = pl.NB; a.d = lp.dil;
    a.pmax = reinterpret_cast<const int32_t *>(ws + pl.pmax);
#define X(HT_, KXT_) if (pl.HT == HT_ && lp.KXT == KXT_) return run_bwd<HT_, KXT_>(a, lp.chains_bwd, lp.split_bwd != 0, st);
    ESRNN_LSTM_SHAPES(X)
#undef X
    return hipErrorInvalidValue;
}

}  // namespace esrnn
