// Output stage of the network (Section 3.4: tanh layer, then linear layer), the
// pinball loss over unmasked outputs (Section 3.5) and the reverse pass of both
// in ONE kernel (the forecasts of Eq. (5) follow in a small kernel of their own,
// for callers that want them): the gradient of the loss
// with respect to an output depends only on that output, its target and the
// number of unmasked outputs (known from the lengths), so the reverse pass of
// this stage can run while the activations are still in registers.  Every
// (window position, 16-series) tile is independent: one wave processes one
// tile at a time with the four weight operands (both matrices, both
// orientations) register-resident for the 16x16x4 fp32 MFMA.
//
// Row order.  "Unit-tile order" of a 16-row output tile m: row 4g+r is logical
// row 4(4m+r)+g, so that component r of lane (g, n) belongs to unit tile 4m+r
// in the one-float-per-lane layout and can be fed back, as it stands, as the B
// operand of k-step 4m+r.  Both forward products use it: the tanh layer's
// output feeds the linear layer, and the linear layer's output (hence the loss
// gradient) feeds the transposed products.
#include "device_utils.h"
#include "esrnn_internal.h"

namespace esrnn {

namespace {

struct HeadArgs {
    const float *WaF, *baF, *WoF, *boF;   // forward A operands and biases
    const float *WoT, *WaT;               // transposed A operands
    const float *R;         // TL(HP) top block output
    const float *Z;         // TL(OP) targets
    const int32_t *lengths;
    const int32_t *pmax;    // [NB] window positions the longest series of a tile has
    const Scalars *sc;
    float *O;               // TL(OP) outputs
    float *loss_partial;    // [gridDim.x]
    float *gO;              // TL(OP): dL/d(output); the target's gradient is its negative
    float *gTop;            // TL(HP): dL/d(top block output)
    float *partial;         // [4 * gridDim.x][stride] weight-gradient partials of every wave
    int P, NB, B, T, I, H, stride;
    int orows;              // rows of the Z, O and gO tiles: 4 * ceil(H / 4)
    float tau;
    int reverse;            // 0: forward only (outputs and loss); the reverse pass and its stores are skipped
};

template <int HT, int MO>
__global__ void __launch_bounds__(256) head_kernel(HeadArgs a)
{
    constexpr int MA = (HT + 3) / 4;
    constexpr int OP = 16 * MO;
    constexpr int OTMAX = 4 * MO;                 // k-steps that cover OP rows
    constexpr int HP16 = 16 * MA;                 // hidden rows padded to whole 16-row tiles
    // per-wave staging for the transposed operand reads of the weight-gradient tiles
    __shared__ float s_go[4][OP * kLdsPad];
    __shared__ float s_a[4][HP16 * kLdsPad];
    __shared__ float s_dp[4][HP16 * kLdsPad];
    __shared__ float s_r[4][HP16 * kLdsPad];
    __shared__ float s_part[4];
    // The transposed weight operands stay in registers where all four operand sets fit; for the larger
    // shapes they are read from LDS, one copy per workgroup (the register file holds the forward operands,
    // the weight-gradient accumulators and two tiles of inputs).
    constexpr bool kTLds = (HT >= 13 && MO >= 2) || MO >= 3;
    // ... and the forward operands too for the largest shapes, as long as the workgroup stays within
    // 128 KB of LDS (this build keeps every kernel below that)
    constexpr int kStagingFloats = 4 * (OP + 3 * HP16) * kLdsPad + 4;
    constexpr int kTFloats = MA * (OTMAX + HT) * 64, kFFloats = (MA + MO) * HT * 64;
    constexpr bool kFLds = HT >= 13 && MO >= 3 && (kStagingFloats + kTFloats + kFFloats) * 4 <= 128 * 1024;
    static_assert((kStagingFloats + (kTLds ? kTFloats : 0)) * 4 <= 128 * 1024, "LDS budget of the output-stage kernel");
    __shared__ float s_wT[kTLds ? MA * (OTMAX + HT) * 64 : 1];
    __shared__ float s_wF[kFLds ? (MA + MO) * HT * 64 : 1];

    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave index, known to be uniform
    const int g = lane >> 4, n = lane & 15;
    const int OT = (a.H + 3) / 4;
    float *go_l = s_go[wv], *a_l = s_a[wv], *dp_l = s_dp[wv], *r_l = s_r[wv];
    for (int i = lane; i < OP * kLdsPad; i += 64) go_l[i] = 0.0f;
    for (int i = lane; i < HP16 * kLdsPad; i += 64) { a_l[i] = 0.0f; dp_l[i] = 0.0f; r_l[i] = 0.0f; }

    float wa[kFLds ? 1 : MA][kFLds ? 1 : HT], wo[kFLds ? 1 : MO][kFLds ? 1 : HT];
    float woT[kTLds ? 1 : MA][kTLds ? 1 : OTMAX], waT[kTLds ? 1 : MA][kTLds ? 1 : HT];
    f32x4 ba[MA], bo[MO];
#pragma unroll
    for (int ma = 0; ma < MA; ++ma) {
#pragma unroll
        for (int q = 0; q < HT; ++q) {
            if (!kFLds) wa[ma][q] = a.WaF[(ma * HT + q) * 64 + lane];
            if (!kTLds) waT[ma][q] = a.WaT[(ma * HT + q) * 64 + lane];
        }
        if (!kTLds) {
#pragma unroll
            for (int ks = 0; ks < OTMAX; ++ks) woT[ma][ks] = ks < OT ? a.WoT[(ma * OT + ks) * 64 + lane] : 0.0f;
        }
        const float4 v = *reinterpret_cast<const float4 *>(a.baF + (ma * 4 + g) * 4);
        ba[ma] = f32x4{v.x, v.y, v.z, v.w};
    }
    if (kTLds) {
        // [ma][OTMAX][64] then [ma][HT][64]
        for (int i = threadIdx.x; i < MA * OTMAX * 64; i += 256) {
            const int l = i & 63, ks = (i >> 6) % OTMAX, ma = (i >> 6) / OTMAX;
            s_wT[i] = ks < OT ? a.WoT[(ma * OT + ks) * 64 + l] : 0.0f;
        }
        for (int i = threadIdx.x; i < MA * HT * 64; i += 256) s_wT[MA * OTMAX * 64 + i] = a.WaT[i];
        if (kFLds) {
            for (int i = threadIdx.x; i < MA * HT * 64; i += 256) s_wF[i] = a.WaF[i];
            for (int i = threadIdx.x; i < MO * HT * 64; i += 256) s_wF[MA * HT * 64 + i] = a.WoF[i];
        }
        __syncthreads();
    }
    auto wa_op = [&](int ma, int q) { return kFLds ? s_wF[(ma * HT + q) * 64 + lane] : wa[kFLds ? 0 : ma][kFLds ? 0 : q]; };
    auto wo_op = [&](int mo, int q) {
        return kFLds ? s_wF[((MA + mo) * HT + q) * 64 + lane] : wo[kFLds ? 0 : mo][kFLds ? 0 : q];
    };
    auto woT_op = [&](int ma, int ks) { return kTLds ? s_wT[(ma * OTMAX + ks) * 64 + lane] : woT[kTLds ? 0 : ma][kTLds ? 0 : ks]; };
    auto waT_op = [&](int ma, int q) {
        return kTLds ? s_wT[(MA * OTMAX + ma * HT + q) * 64 + lane] : waT[kTLds ? 0 : ma][kTLds ? 0 : q];
    };
#pragma unroll
    for (int mo = 0; mo < MO; ++mo) {
#pragma unroll
        for (int q = 0; q < HT; ++q)
            if (!kFLds) wo[mo][q] = a.WoF[(mo * HT + q) * 64 + lane];
        const float4 v = *reinterpret_cast<const float4 *>(a.boF + (mo * 4 + g) * 4);
        bo[mo] = f32x4{v.x, v.y, v.z, v.w};
    }
    f32x4 dWo[MO * MA], dWa[MA * MA];
#pragma unroll
    for (int i = 0; i < MO * MA; ++i) dWo[i] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < MA * MA; ++i) dWa[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    float dbo[OTMAX], dba[4 * MA];
#pragma unroll
    for (int i = 0; i < OTMAX; ++i) dbo[i] = 0.0f;
#pragma unroll
    for (int i = 0; i < 4 * MA; ++i) dba[i] = 0.0f;

    const float inv_n = a.sc->inv_n_pin;
    float loss = 0.0f;
    // Tiles are numbered p * NB + (series tile); a wave takes every stride-th one and keeps (p, series
    // tile) by increments.  All of it is wave-uniform, so tile bases live on the scalar unit and the
    // lanes only add their own index.
    const int n_tiles = a.P * a.NB;
    const int stride = gridDim.x * 4;
    const int step_p = stride / a.NB, step_bt = stride % a.NB;

    // operands of one tile; those of the next tile are requested before this one is computed
    struct Ops {
        float br[HT];
        float z[OTMAX];                // row 4*ks + g
        int len;
        int pmax;                      // window positions of the tile's longest series
    };
    auto load_ops = [&](int tile, int p, int bt, Ops &o) {
        if (tile >= n_tiles) { tile = n_tiles - 1; p = a.P - 1; bt = a.NB - 1; }
        const int b = bt * 16 + n;
        const float *rt = a.R + (size_t)tile * HT * 64;
#pragma unroll
        for (int q = 0; q < HT; ++q) o.br[q] = (rt + q * 64)[lane];
        o.len = a.lengths[b < a.B ? b : a.B - 1];
        o.pmax = a.pmax[bt];
        const float *zt = a.Z + (size_t)tile * a.orows * 16;
#pragma unroll
        for (int ks = 0; ks < OTMAX; ++ks) {
            const int j = 4 * ks + g;
            o.z[ks] = zt[(j < a.orows ? j : a.orows - 1) * 16 + n];
        }
    };
    auto advance = [&](int &tile, int &p, int &bt) {
        tile += stride; p += step_p; bt += step_bt;
        if (bt >= a.NB) { bt -= a.NB; ++p; }
    };

    Ops cur, nxt;
    int tile = blockIdx.x * 4 + wv;
    int p = tile / a.NB, bt = tile % a.NB;
    if (tile < n_tiles) load_ops(tile, p, bt, cur);
    for (; tile < n_tiles; advance(tile, p, bt)) {
        {
            int tn = tile, pn = p, btn = bt;
            advance(tn, pn, btn);
            load_ops(tn, pn, btn, nxt);
        }
        const int b = bt * 16 + n;
        // Ragged batches: a tile past the longest series of its 16 holds no window.  Nothing was computed
        // for it upstream and nothing downstream reads it.
        // (the bound travels with the tile's operands: read here, it would stall the wave on every tile until the
        // operand loads just issued for the next tile had all returned)
        if (p >= cur.pmax) {
            cur = nxt;
            continue;
        }
        int len = cur.len < 0 ? 0 : (cur.len > a.T ? a.T : cur.len);
        if (b >= a.B) len = 0;
        const bool valid = p < len - a.I - a.H + 1;

        // ---- forward: tanh layer, linear layer
        f32x4 acc[MA];
#pragma unroll
        for (int ma = 0; ma < MA; ++ma) acc[ma] = ba[ma];
#pragma unroll
        for (int q = 0; q < HT; ++q)
#pragma unroll
            for (int ma = 0; ma < MA; ++ma) acc[ma] = mfma16(wa_op(ma, q), cur.br[q], acc[ma]);
        float av[4 * MA];
#pragma unroll
        for (int ma = 0; ma < MA; ++ma)
#pragma unroll
            for (int r = 0; r < 4; ++r) av[4 * ma + r] = (4 * ma + r < HT) ? tanh_f(acc[ma][r]) : 0.0f;
        f32x4 oc[MO];
#pragma unroll
        for (int mo = 0; mo < MO; ++mo) oc[mo] = bo[mo];
#pragma unroll
        for (int q = 0; q < HT; ++q)
#pragma unroll
            for (int mo = 0; mo < MO; ++mo) oc[mo] = mfma16(wo_op(mo, q), av[q], oc[mo]);

        // ---- outputs, loss and the gradient of the pinball loss; k-step ks holds rows 4ks..4ks+3
        float go[OTMAX];
        float *ot = a.O + (size_t)tile * a.orows * 16, *got = a.gO + (size_t)tile * a.orows * 16;
#pragma unroll
        for (int ks = 0; ks < OTMAX; ++ks) {
            const int j = 4 * ks + g;               // 0-based step of the horizon
            const float o = oc[ks >> 2][ks & 3];
            const float d = cur.z[ks] - o;
            const bool counted = valid && j < a.H;
            if (counted) loss += d >= 0.0f ? a.tau * d : (a.tau - 1.0f) * d;
            const float val = counted ? (d >= 0.0f ? -a.tau : 1.0f - a.tau) * inv_n : 0.0f;
            go[ks] = val;
            if (j < a.orows) {
                ot[j * 16 + n] = o;
                got[j * 16 + n] = val;
            }
            go_l[j * kLdsPad + n] = val;
            dbo[ks] += val;
        }
        if (!a.reverse) {       // forward-only callers: nothing below is needed
            cur = nxt;
            continue;
        }
        // ---- reverse: dA = Wo^T gO (unit-tile order), through the tanh
#pragma unroll
        for (int ma = 0; ma < MA; ++ma) acc[ma] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < OTMAX; ++ks)
#pragma unroll
            for (int ma = 0; ma < MA; ++ma) acc[ma] = mfma16(woT_op(ma, ks), go[ks], acc[ma]);
        float dp[4 * MA];
#pragma unroll
        for (int ma = 0; ma < MA; ++ma)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int q = 4 * ma + r;
                const float rv = q < HT ? cur.br[q < HT ? q : HT - 1] : 0.0f;   // unit tiles past HT are padding (the index stays in range)
                dp[q] = acc[ma][r] * (1.0f - av[q] * av[q]);
                dba[q] += dp[q];
                const int row = 4 * q + g;
                a_l[row * kLdsPad + n] = av[q];
                dp_l[row * kLdsPad + n] = dp[q];
                r_l[row * kLdsPad + n] = rv;
            }
        // dR = Wa^T dpre
#pragma unroll
        for (int ma = 0; ma < MA; ++ma) acc[ma] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int q = 0; q < HT; ++q)
#pragma unroll
            for (int ma = 0; ma < MA; ++ma) acc[ma] = mfma16(waT_op(ma, q), dp[q], acc[ma]);
#pragma unroll
        for (int ma = 0; ma < MA; ++ma)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int q = 4 * ma + r;
                if (q < HT) (a.gTop + (size_t)tile * HT * 64 + q * 64)[lane] = acc[ma][r];
            }
        // weight gradients: contraction over the 16 series of the tile
#pragma unroll
        for (int mo = 0; mo < MO; ++mo)
#pragma unroll
            for (int na = 0; na < MA; ++na)
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
                    dWo[mo * MA + na] = mfma16(go_l[(16 * mo + n) * kLdsPad + 4 * ks + g],
                                               a_l[(16 * na + n) * kLdsPad + 4 * ks + g], dWo[mo * MA + na]);
#pragma unroll
        for (int ma = 0; ma < MA; ++ma)
#pragma unroll
            for (int na = 0; na < MA; ++na)
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
                    dWa[ma * MA + na] = mfma16(dp_l[(16 * ma + n) * kLdsPad + 4 * ks + g],
                                               r_l[(16 * na + n) * kLdsPad + 4 * ks + g], dWa[ma * MA + na]);
        cur = nxt;
    }

    // per-wave partial block: dWo tiles, dWa tiles, dbo, dba
    float *dst = a.partial + (size_t)(blockIdx.x * 4 + wv) * a.stride;
#pragma unroll
    for (int i = 0; i < MO * MA; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) dst[(i * 4 + r) * 64 + lane] = dWo[i][r];
    dst += MO * MA * 256;
#pragma unroll
    for (int i = 0; i < MA * MA; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) dst[(i * 4 + r) * 64 + lane] = dWa[i][r];
    dst += MA * MA * 256;
#pragma unroll
    for (int ks = 0; ks < OTMAX; ++ks) {
        const float tot = group16_sum(dbo[ks]);
        if (n == 0 && ks < OT) dst[4 * ks + g] = tot;
    }
    dst += 4 * OT;
#pragma unroll
    for (int q = 0; q < 4 * MA; ++q) {
        const float tot = group16_sum(dba[q]);
        if (n == 0 && q < HT) dst[4 * q + g] = tot;
    }

    const float tot = wave_sum(loss);
    if (lane == 0) s_part[wv] = tot;
    __syncthreads();
    if (threadIdx.x == 0) a.loss_partial[blockIdx.x] = (s_part[0] + s_part[1]) + (s_part[2] + s_part[3]);
}

// ---------------------------------------------------------------------------
// Forecasts of Eq. (5) at every window position: exp(output) * level * seasonal factors of the target
// time, zero where the window does not fit into the series.  One wave per (position, 16-series) tile.
// Lane (g, n) computes the steps j = g, g+4, ... of series n: the tile of outputs and the rows of the
// seasonal factors are read in their storage order.  The tile's 16 * H forecasts are contiguous in the
// [P][B][H] array but ordered [series][step]: they are turned through the wave's corner of LDS and written
// out in storage order as well.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) forecast_kernel(const float *__restrict__ O, const float *__restrict__ u,
                                                        const float *__restrict__ S1, const float *__restrict__ S2,
                                                        const int32_t *__restrict__ lengths, const int32_t *__restrict__ pmax,
                                                        float *__restrict__ forecasts, int P, int NB, int B, int Bp, int T,
                                                        int I, int H, int orows, int n_seas)
{
    __shared__ float s_f[4][16 * ESRNN_MAX_WINDOW];
    const int lane = threadIdx.x & 63, g = lane >> 4, n = lane & 15;
    float *fl = s_f[threadIdx.x >> 6];
    const long long tile = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (tile >= (long long)P * NB) return;              // (no workgroup barrier below)
    const int p = (int)(tile / NB), bt = (int)(tile % NB);
    const int t = p + I - 1;
    const int b = bt * 16 + n;
    const int cols = min(16, B - bt * 16);              // series of this tile that exist
    const int len = b < B ? min(max(lengths[b], 0), T) : 0;
    const bool valid = p < pmax[bt] && p < len - I - H + 1;     // past pmax the tile of outputs holds nothing
    const float ut = valid ? u[(size_t)t * Bp + b] : 0.0f;
    const float *ot = O + (size_t)tile * orows * 16;
    for (int j = g; j < H; j += 4) {
        float f = 0.0f;
        if (valid) {
            float seas = 1.0f;
            if (n_seas >= 1) seas = S1[(size_t)(t + 1 + j) * Bp + b];
            if (n_seas >= 2) seas *= S2[(size_t)(t + 1 + j) * Bp + b];
            f = __expf(ot[j * 16 + n] + ut) * seas;
        }
        fl[n * H + j] = f;
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");     // same wave: LDS serves its instructions in order
    float *ft = forecasts + ((size_t)p * B + bt * 16) * H;
    for (int e = lane; e < cols * H; e += 64) ft[e] = fl[e];
}

#define ESRNN_HEAD_SHAPES(X) \
    X(2, 1) X(2, 2) X(2, 3) X(2, 4) X(8, 1) X(8, 2) X(8, 3) X(8, 4) X(10, 1) X(10, 2) X(10, 3) X(10, 4) \
    X(13, 1) X(13, 2) X(13, 3) X(13, 4) X(16, 1) X(16, 2) X(16, 3) X(16, 4)

}  // namespace

hipError_t launch_forecasts(const Plan &pl, const int32_t *lengths, float *ws, float *forecasts, hipStream_t st)
{
    const long long tiles = (long long)pl.P * pl.NB;
    forecast_kernel<<<(unsigned)((tiles + 3) / 4), 256, 0, st>>>(
        ws + pl.O, ws + pl.u, ws + pl.S1, ws + pl.S2, lengths, reinterpret_cast<const int32_t *>(ws + pl.pmax), forecasts,
        pl.P, pl.NB, pl.B, pl.Bt, pl.T, pl.I, pl.H, pl.OP, pl.cfg.n_seas);
    return hipGetLastError();
}

hipError_t launch_head(const Plan &pl, const int32_t *lengths, float *ws, bool reverse, hipStream_t st)
{
    const HeadPack hp = head_pack_layout(pl);
    const float *f = ws + pl.head_fwd_pack, *bk = ws + pl.head_bwd_pack;
    const int blocks = pl.n_head_waves / 4;
    HeadArgs a{f + hp.WaF, f + hp.baF, f + hp.WoF, f + hp.boF, bk + hp.WoT, bk + hp.WaT,
               ws + pl.blk_out[pl.cfg.n_blocks - 1], ws + pl.Z, lengths,
               reinterpret_cast<const int32_t *>(ws + pl.pmax), reinterpret_cast<const Scalars *>(ws + pl.scalars), ws + pl.O, ws + pl.loss_partial,
               ws + pl.gO, ws + pl.gTop, ws + pl.head_dw_partial,
               pl.P, pl.NB, pl.B, pl.T, pl.I, pl.H, pl.head_dw_stride, pl.OP, pl.cfg.tau,
               reverse ? 1 : 0};
#define X(HT_, MO_)                                              \
    if (pl.HT == HT_ && pl.MO == MO_) {                          \
        head_kernel<HT_, MO_><<<blocks, 256, 0, st>>>(a);        \
        return hipGetLastError();                                \
    }
    ESRNN_HEAD_SHAPES(X)
#undef X
    return hipErrorInvalidValue;
}

}  // namespace esrnn
