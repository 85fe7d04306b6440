// Streaming kernels of the training step: loss normalisers, operand packing,
// exponential-smoothing recursions (forward and adjoint), window extraction
// (forward and adjoint), loss reduction and weight-gradient reduction.
#include <algorithm>
#include <mutex>
#include <type_traits>

#include "device_utils.h"
#include "esrnn_internal.h"

namespace esrnn {

namespace {

__device__ __forceinline__ int clamp_len(int len, int T) { return len < 0 ? 0 : (len > T ? T : len); }

// ---------------------------------------------------------------------------
// Loss normalisers (Section 3.5: padded outputs are masked out of the loss).
// ---------------------------------------------------------------------------
struct PrepArgs {
    const int32_t *lengths;
    Scalars *sc;
    int32_t *pmax;       // [NB] window positions needed by the longest series of every 16-series tile
    int NB;
    int B, T, I, H;
    int cs_per_window;   // cell-state values per valid window in the cell-state penalty: hidden * blocks
};

__device__ void prep_body(const PrepArgs &pa)
{
    const int32_t *__restrict__ lengths = pa.lengths;
    Scalars *__restrict__ sc = pa.sc;
    const int B = pa.B, T = pa.T, I = pa.I, H = pa.H;
    __shared__ double s_pin[256], s_lv[256];
    double np_ = 0.0, nl = 0.0;
    // eight independent loads in flight per thread: one workgroup has to read all lengths
    for (int b0 = threadIdx.x; b0 < B; b0 += 8 * 256) {
        int len[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int b = b0 + k * 256;
            len[k] = b < B ? lengths[b] : 0;
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int l = clamp_len(len[k], T);
            const int Pb = l - I - H + 1;
            if (Pb > 0) np_ += (double)Pb * H;
            if (l > 2) nl += (double)(l - 2);
        }
    }
    s_pin[threadIdx.x] = np_;
    s_lv[threadIdx.x] = nl;
    __syncthreads();
    for (int off = 128; off >= 1; off >>= 1) {
        if ((int)threadIdx.x < off) {
            s_pin[threadIdx.x] += s_pin[threadIdx.x + off];
            s_lv[threadIdx.x] += s_lv[threadIdx.x + off];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        sc->inv_n_pin = s_pin[0] > 0.0 ? (float)(1.0 / s_pin[0]) : 0.0f;
        sc->inv_n_lv = s_lv[0] > 0.0 ? (float)(1.0 / s_lv[0]) : 0.0f;
        const double n_cs = s_pin[0] / (double)H * (double)pa.cs_per_window;   // valid windows x hidden x blocks
        sc->inv_n_cs = n_cs > 0.0 ? (float)(1.0 / n_cs) : 0.0f;
    }
}

// Ragged batches (Section 8.1: padding multiplies the iterations of the recursions): every later kernel
// stops a 16-series tile at the number of window positions its longest series has.  One thread per tile.
__device__ void pmax_body(const PrepArgs &pa, int first_block, int n_blocks)
{
    for (int bt = (blockIdx.x - first_block) * 256 + threadIdx.x; bt < pa.NB; bt += n_blocks * 256) {
        int best = 0;
        for (int k = 0; k < kTileN; ++k) {
            const int b = bt * kTileN + k;
            if (b < pa.B) best = max(best, clamp_len(pa.lengths[b], pa.T) - pa.I - pa.H + 1);
        }
        pa.pmax[bt] = best;
    }
}

// ---------------------------------------------------------------------------
// Operand packing: weights rearranged into the per-lane operand order of the
// 16x16x4 MFMA (lane l supplies A[l%16][l/16]) so that every wave loads its
// register-resident slice with coalesced reads.
// ---------------------------------------------------------------------------
struct PackLstmArgs {
    const float *W, *b;
    float *fwd, *bias, *bwd;
    int h, in_dim, HT, KXT;
    int narrow;          // operand order of the 4-series kernels (4x4x1 MFMA) instead
};

// Operands of the 4-series kernels.  v_mfma_f32_4x4x1: lane l supplies A[l%4] of block l/4.
//   forward  [wave][column k of x ; h][lane]: gate l%4 of unit wave*HT + min(l/4, HT-1) (the blocks past HT
//            repeat the last unit, so that all lanes do the same work on the same addresses)
//   reverse  [wave][group g][k-step 4*u + gate][lane]: W[gate, unit wave*HT + u][column 64*g + l]
__device__ void pack_lstm_narrow_body(const PackLstmArgs &a)
{
    const int KX = 4 * a.KXT, KT4 = KX + 4 * a.HT, NG = (KT4 + 63) / 64, ld = a.in_dim + a.h;
    const int n_fwd = 4 * KT4 * 64, n_bwd = 4 * NG * 4 * a.HT * 64;
    auto user_col = [&](int k) {
        if (k < KX) return k < a.in_dim ? k : -1;
        if (k < KT4) return k - KX < a.h ? a.in_dim + k - KX : -1;
        return -1;
    };
    for (int idx = blockIdx.x * 256 + threadIdx.x; idx < n_fwd + n_bwd; idx += gridDim.x * 256) {
        if (idx < n_fwd) {
            const int lane = idx & 63, k = (idx >> 6) % KT4, w = (idx >> 6) / KT4;
            const int blk = min(lane >> 2, a.HT - 1), gate = lane & 3, unit = w * a.HT + blk, col = user_col(k);
            a.fwd[idx] = (unit < a.h && col >= 0) ? a.W[(size_t)(gate * a.h + unit) * ld + col] : 0.0f;
        } else {
            const int j = idx - n_fwd;
            const int lane = j & 63, ks = (j >> 6) % (4 * a.HT), g = ((j >> 6) / (4 * a.HT)) % NG, w = (j >> 6) / (4 * a.HT * NG);
            const int unit = w * a.HT + (ks >> 2), gate = ks & 3, col = user_col(64 * g + lane);
            a.bwd[j] = (unit < a.h && col >= 0) ? a.W[(size_t)(gate * a.h + unit) * ld + col] : 0.0f;
        }
    }
}

__device__ void pack_lstm_body(const PackLstmArgs &a)
{
    if (a.narrow) {
        pack_lstm_narrow_body(a);
        return;
    }
    const int KT = a.KXT + a.HT, MB = (KT + 3) / 4, ld = a.in_dim + a.h;
    const int n_fwd = a.HT * KT * 64, n_bias = a.HT * 16, n_bwd = MB * 4 * a.HT * 64;
    for (int idx = blockIdx.x * 256 + threadIdx.x; idx < n_fwd + n_bias + n_bwd; idx += gridDim.x * 256) {
        if (idx < n_fwd) {
            // gate contraction: row 4g+r of unit tile mt is gate r of unit 4mt+g
            const int lane = idx & 63, ks = (idx >> 6) % KT, mt = (idx >> 6) / KT;
            const int i = lane & 15, kk = lane >> 4;
            const int unit = 4 * mt + (i >> 2), gate = i & 3;
            int col = -1;
            if (ks < a.KXT) { const int xc = 4 * ks + kk; if (xc < a.in_dim) col = xc; }
            else { const int hu = 4 * (ks - a.KXT) + kk; if (hu < a.h) col = a.in_dim + hu; }
            a.fwd[idx] = (unit < a.h && col >= 0) ? a.W[(size_t)(gate * a.h + unit) * ld + col] : 0.0f;
        } else if (idx < n_fwd + n_bias) {
            const int j = idx - n_fwd;
            const int gate = j & 3, unit = j >> 2;   // (mt*4+g)*4 + r  ->  unit = 4mt+g
            a.bias[j] = unit < a.h ? a.b[gate * a.h + unit] : 0.0f;
        } else {
            // transposed contraction: k-step 4mt+gate, lane group = unit within tile;
            // output row 4g+r of tile mb is row g of input unit tile 4mb+r
            const int j = idx - n_fwd - n_bias;
            const int lane = j & 63, ks = (j >> 6) % (4 * a.HT), mb = (j >> 6) / (4 * a.HT);
            const int i = lane & 15, gk = lane >> 4;
            const int mt = ks >> 2, gate = ks & 3;
            const int unit = 4 * mt + gk;
            const int q = 4 * mb + (i & 3), gi = i >> 2;
            int col = -1;
            if (q < a.KXT) { const int xc = 4 * q + gi; if (xc < a.in_dim) col = xc; }
            else if (q < KT) { const int hu = 4 * (q - a.KXT) + gi; if (hu < a.h) col = a.in_dim + hu; }
            a.bwd[j] = (unit < a.h && col >= 0) ? a.W[(size_t)(gate * a.h + unit) * ld + col] : 0.0f;
        }
    }
}

struct PackHeadArgs {
    const float *Wa, *ba, *Wo, *bo;
    float *WaF, *baF, *WoF, *boF, *WoT, *WaT;
    int h, H, HT, MA, MO, OT;
};

__device__ void pack_head_body(const PackHeadArgs &a)
{
    const int nWaF = a.MA * a.HT * 64, nbaF = a.MA * 16, nWoF = a.MO * a.HT * 64, nboF = a.MO * 16;
    const int nWoT = a.MA * a.OT * 64, nWaT = a.MA * a.HT * 64;
    const int total = nWaF + nbaF + nWoF + nboF + nWoT + nWaT;
    for (int idx = blockIdx.x * 256 + threadIdx.x; idx < total; idx += gridDim.x * 256) {
        int j = idx;
        if (j < nWaF) {
            const int lane = j & 63, q = (j >> 6) % a.HT, ma = (j >> 6) / a.HT;
            const int i = lane & 15, kk = lane >> 4;
            const int out = 4 * (4 * ma + (i & 3)) + (i >> 2), in = 4 * q + kk;
            a.WaF[j] = (out < a.h && in < a.h) ? a.Wa[out * a.h + in] : 0.0f;
            continue;
        }
        j -= nWaF;
        if (j < nbaF) {
            const int r = j & 3, g = (j >> 2) & 3, ma = j >> 4;
            const int unit = 4 * (4 * ma + r) + g;
            a.baF[j] = unit < a.h ? a.ba[unit] : 0.0f;
            continue;
        }
        j -= nbaF;
        if (j < nWoF) {
            const int lane = j & 63, q = (j >> 6) % a.HT, mo = (j >> 6) / a.HT;
            const int i = lane & 15;
            const int row = 4 * (4 * mo + (i & 3)) + (i >> 2), in = 4 * q + (lane >> 4);
            a.WoF[j] = (row < a.H && in < a.h) ? a.Wo[row * a.h + in] : 0.0f;
            continue;
        }
        j -= nWoF;
        if (j < nboF) {
            const int r = j & 3, g = (j >> 2) & 3, mo = j >> 4;
            const int row = 4 * (4 * mo + r) + g;
            a.boF[j] = row < a.H ? a.bo[row] : 0.0f;
            continue;
        }
        j -= nboF;
        if (j < nWoT) {
            const int lane = j & 63, ks = (j >> 6) % a.OT, ma = (j >> 6) / a.OT;
            const int i = lane & 15, kk = lane >> 4;
            const int unit = 4 * (4 * ma + (i & 3)) + (i >> 2), row = 4 * ks + kk;
            a.WoT[j] = (unit < a.h && row < a.H) ? a.Wo[row * a.h + unit] : 0.0f;
            continue;
        }
        j -= nWoT;
        {
            const int lane = j & 63, q = (j >> 6) % a.HT, ma = (j >> 6) / a.HT;
            const int i = lane & 15, kk = lane >> 4;
            const int unit = 4 * (4 * ma + (i & 3)) + (i >> 2), row = 4 * q + kk;
            a.WaT[j] = (unit < a.h && row < a.h) ? a.Wa[row * a.h + unit] : 0.0f;
        }
    }
}

// One launch for everything that only depends on the weights and the lengths:
// blockIdx.z selects an LSTM layer, the output stage, or the loss normalisers.
struct SetupArgs {
    PackLstmArgs lstm[kMaxLayers];
    PackHeadArgs head;
    PrepArgs prep;
    int L, pack;     // pack = 0: only the loss normalisers
};

__global__ void __launch_bounds__(256) setup_kernel(SetupArgs a)
{
    const int z = blockIdx.z;
    if (a.pack && z < a.L) pack_lstm_body(a.lstm[z]);
    else if (a.pack && z == a.L) pack_head_body(a.head);
    else if (blockIdx.x == 0) prep_body(a.prep);
    else pmax_body(a.prep, 1, gridDim.x - 1);
}

// ---------------------------------------------------------------------------
// Exponential-smoothing recursions, Section 3.1 Eq. (1) and (3) without trend;
// Section 8.2 variants (two seasonalities, none).  One lane per series, time
// sequential; every load and store is one contiguous row segment of a
// time-major array.  The seasonal factors that will apply m steps ahead live
// in a per-lane ring in LDS (slot t mod m holds the factor for time t until
// step t has used it, then the factor for time t + m).
// ---------------------------------------------------------------------------
struct EsArgs {
    const float *y;           // [T][B]
    const int32_t *lengths;
    const float *es;          // [K][B]
    float *lvl, *S1, *S2, *u, *v;   // [T][Bp], one column per lane of every wave
    float *lv_partial;        // [gridDim.x]
    int B, Bp, T, n_seas, m1, m2, logit;   // Bp: row stride of the time-major arrays (batch padded to 64)
    int row_gamma1, row_gamma2, row_s1, row_s2;
};

// CS: how many consecutive time steps take their seasonal factors out of the ring together (and put the
// new ones back together): a divisor of 8 not larger than the shorter period, so that no factor a group
// reads is produced inside the group.  Within a group the steps are then plain register arithmetic whose
// only chain is the level (one multiply-add per step); divisions and seasonal updates of the other steps
// overlap with it.
//
// Division of labour.  A workgroup serves 64 series with three or four waves.  Wave 0 runs the recursion and
// nothing else: it reads observations (several chunks ahead), keeps the rings, and leaves level,
// de-seasonalised value and factors of every step in an LDS staging buffer; it issues no global store and
// computes no logarithm.  Of the previous chunk, wave 1 turns the staged level into lvl, u = ln(level) and
// the level penalty, wave 2 the staged value into v, and wave 3 (seasonal shapes) stores the factors.  A lone
// wave issues one instruction every few cycles whatever the instruction is; with the chain, five stores and two
// logarithms per step on the same wave a step took about three times as long as the chain alone.
constexpr int kEsChunk = 8;                 // steps per staging buffer
constexpr int kEsAhead = 4;                 // chunks between the request of a row and its use
// staged per step: level, de-seasonalised value, and one factor per seasonality
constexpr int es_stage_floats(int n_seas) { return 2 * kEsChunk * (2 + n_seas) * 64; }

template <int NS, int CS>
__global__ void __launch_bounds__(NS == 0 ? 192 : 256) es_forward_kernel(EsArgs a)
{
    extern __shared__ float ring[];   // [m1 + m2][64] rings, then [2][kEsChunk][2 + NS][64] staging
    constexpr int CH = kEsChunk, NF = 2 + NS;
    static_assert(CH % CS == 0, "groups tile a chunk");
    const int role = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int b = blockIdx.x * 64 + lane;
    const bool in_batch = b < a.B;
    const int len = in_batch ? clamp_len(a.lengths[b], a.T) : 0;
    float *ring1 = ring, *ring2 = ring + (size_t)a.m1 * 64;
    float *stage = ring + (size_t)(a.m1 + a.m2) * 64;       // [buffer][step][lt, q, s1, s2][lane]
    // Ragged batches (Section 8.1): the sweep ends at the longest series of the wave.  Rows between a
    // series' own length and that bound get the defined padding values; rows beyond it are neither written
    // here nor read by any later kernel (their bounds are those of 16-series tiles, never larger).
    // (every wave of the workgroup holds the same 64 series, so the bound is the same in all of them)
    const int t_end = wave_max_int(len);
    const int n_chunks = (t_end + CH - 1) / CH;
    // Every lane owns a column of the time-major arrays (their rows are padded to whole waves), so no store
    // is ever skipped and a row address is a wave-uniform base plus the lane: scalar address arithmetic.
    const unsigned ub = b;

    // Initial seasonal factors into the rings (ring 2 follows ring 1): all waves of the workgroup share the
    // rows, eight requests in flight each - read one after the other by a single wave, the m1 + m2 rows of a
    // long-period shape took longer than the whole recursion.
    {
        constexpr int NWV = NS == 0 ? 3 : 4;
        const int rows = a.m1 + a.m2;
        for (int k0 = role * 8; k0 < rows; k0 += NWV * 8) {
            float sv[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int k = min(k0 + j, rows - 1);
                const int row = k < a.m1 ? a.row_s1 + k : a.row_s2 + (k - a.m1);
                sv[j] = in_batch ? a.es[(size_t)row * a.B + b] : 1.0f;
            }
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (k0 + j < rows) ring[(k0 + j) * 64 + lane] = (a.logit && in_batch) ? expf(sv[j]) : sv[j];
        }
        __syncthreads();
    }
    if (role == 0) {
        float alpha = 0.5f, g1 = 0.0f, g2 = 0.0f;
        if (in_batch) {
            alpha = a.es[b];
            if (NS >= 1) g1 = a.es[(size_t)a.row_gamma1 * a.B + b];
            if (NS >= 2) g2 = a.es[(size_t)a.row_gamma2 * a.B + b];
            if (a.logit) {
                alpha = 1.0f / (1.0f + expf(-alpha));
                g1 = 1.0f / (1.0f + expf(-g1));
                g2 = 1.0f / (1.0f + expf(-g2));
            }
        }
        float l_prev = 1.0f;
        int i1 = 0, i2 = 0;           // ring slot of the current time: t mod m
        const float one_m_alpha = 1.0f - alpha;

        // CS consecutive steps t0 .. t0+CS-1, staged at `out`.  WRAP: whether a ring index may pass the end of
        // its ring inside the group; if not, the group's slots are consecutive and every LDS address is one
        // per-lane base plus a constant.
        auto steps = [&](auto wrap, int t0, const float *yv, float *out) {
            constexpr bool WRAP = decltype(wrap)::value;
            float s1v[CS], s2v[CS], w1v[CS], w2v[CS];
            float *r1 = ring1 + i1 * 64 + lane, *r2 = ring2 + i2 * 64 + lane;
            auto slot1 = [&](int k) { return WRAP ? ring1 + (i1 + k < a.m1 ? i1 + k : i1 + k - a.m1) * 64 + lane : r1 + k * 64; };
            auto slot2 = [&](int k) { return WRAP ? ring2 + (i2 + k < a.m2 ? i2 + k : i2 + k - a.m2) * 64 + lane : r2 + k * 64; };
#pragma unroll
            for (int k = 0; k < CS; ++k) {
                s1v[k] = NS >= 1 ? *slot1(k) : 1.0f;             // CS <= m: at most one wrap
                s2v[k] = NS >= 2 ? *slot2(k) : 1.0f;
            }
#pragma unroll
            for (int k = 0; k < CS; ++k) {
                const int t = t0 + k;
                // Past the end of a series the observation is replaced by 1: levels and factors stay finite,
                // the storing waves replace what they write there by the padding values.
                const float yt = t < len ? yv[k] : 1.0f;
                const float s1 = s1v[k], s2 = s2v[k];
                const float r12 = fast_rcp(s1 * s2);         // one reciprocal serves 1/(s1 s2), 1/s1 and 1/s2
                const float q = yt * r12;
                // reading for the state before the first observation: l_{-1} = y_0 / S[0]
                const float lt = (t == 0) ? q : alpha * q + one_m_alpha * l_prev;
                // Eq. (3): divide by the previous level (and the other factor); at t = 0 the produced factor
                // equals the initial one
                const float ry = yt * fast_rcp(l_prev);
                w1v[k] = (NS >= 1 && t >= 1) ? g1 * ry * (NS >= 2 ? r12 * s1 : 1.0f) + (1.0f - g1) * s1 : s1;
                w2v[k] = (NS >= 2 && t >= 1) ? g2 * ry * (r12 * s2) + (1.0f - g2) * s2 : s2;
                float *o = out + k * NF * 64 + lane;
                o[0] = lt;
                o[64] = q;
                if (NS >= 1) o[128] = s1;
                if (NS >= 2) o[192] = s2;
                l_prev = t < len ? lt : l_prev;
            }
#pragma unroll
            for (int k = 0; k < CS; ++k) {
                if (NS >= 1) *slot1(k) = w1v[k];     // the factor for time t + m
                if (NS >= 2) *slot2(k) = w2v[k];
            }
            if (NS >= 1) { i1 += CS; if (i1 >= a.m1) i1 -= a.m1; }
            if (NS >= 2) { i2 += CS; if (i2 >= a.m2) i2 -= a.m2; }
        };
        // Observations are requested kEsAhead chunks ahead: a request takes about as long as a chunk of steps,
        // and one chunk of lead made every chunk wait for memory.  The register sets rotate through a loop
        // unrolled kEsAhead times, so that their indices are constants.  Row offsets in 32 bits (B * T is at
        // most 2^30): one scalar multiply per request instead of a 64-bit product.
        float ybuf[kEsAhead][CH];
        const unsigned ycol = in_batch ? ub : 0u;
        auto load_chunk = [&](int c, float *dst) {
#pragma unroll
            for (int k = 0; k < CH; ++k) {
                // raw value of a wave-uniform row (the last row again past the end); the step replaces what
                // lies past the series' length
                const unsigned t = (unsigned)min(c * CH + k, a.T - 1);
                dst[k] = a.y[t * (unsigned)a.B + ycol];
            }
        };
        static_for<0, kEsAhead>([&](auto d) { load_chunk(decltype(d)::value, ybuf[decltype(d)::value]); });
        for (int c0 = 0; c0 < n_chunks; c0 += kEsAhead) {
            static_for<0, kEsAhead>([&](auto dd) {
                constexpr int d = decltype(dd)::value;
                const int c = c0 + d;
                if (c < n_chunks) {                         // (wave-uniform)
                    float *out = stage + (c & 1) * (CH * NF * 64);
#pragma unroll
                    for (int k = 0; k < CH; k += CS) {
                        const bool wraps = (NS >= 1 && i1 + CS > a.m1) || (NS >= 2 && i2 + CS > a.m2);   // (wave-uniform)
                        if (wraps) steps(std::true_type{}, c * CH + k, ybuf[d] + k, out + k * NF * 64);
                        else steps(std::false_type{}, c * CH + k, ybuf[d] + k, out + k * NF * 64);
                    }
                    load_chunk(c + kEsAhead, ybuf[d]);
                    // chunk c is staged; the other waves have finished with chunk c - 1, whose buffer chunk
                    // c + 1 reuses
                    lds_barrier();
                }
            });
        }
        return;
    }

    // ---- the storing waves: chunk c after the barrier that publishes it.  One loop per role, the staged
    // values of a whole chunk read together, no branch inside a full chunk.
    const int full_chunks = t_end / CH;            // chunks that lie entirely below the bound
    if (role == 1) {
        float u1 = 0.0f, u2 = 0.0f, lv_sum = 0.0f;
        auto chunk = [&](int c, int n_steps) {
            const float *in = stage + (c & 1) * (CH * NF * 64) + lane;
            float lt[CH];
#pragma unroll
            for (int k = 0; k < CH; ++k) lt[k] = in[k * NF * 64];
#pragma unroll
            for (int k = 0; k < CH; ++k) {
                if (k >= n_steps) break;
                const int t = c * CH + k;
                const bool live = t < len;
                const float l = live ? lt[k] : 1.0f;
                const float ut = live ? fast_log(l) : 0.0f;
                const unsigned at = (unsigned)t * (unsigned)a.Bp + ub;     // (B * T is at most 2^30)
                a.lvl[at] = l;
                a.u[at] = ut;
                // Section 8.4: squared second difference of the log level
                const float e = ut - 2.0f * u1 + u2;
                lv_sum += (live && t >= 2) ? e * e : 0.0f;
                u2 = u1; u1 = ut;
            }
        };
        for (int c = 0; c < n_chunks; ++c) {
            lds_barrier();
            if (c < full_chunks) chunk(c, CH);
            else chunk(c, t_end - c * CH);
        }
        const float tot = wave_sum(lv_sum);
        if (lane == 0) a.lv_partial[blockIdx.x] = tot;
    } else if (role == 2) {
        auto chunk = [&](int c, int n_steps) {
            const float *in = stage + (c & 1) * (CH * NF * 64) + 64 + lane;
            float q[CH];
#pragma unroll
            for (int k = 0; k < CH; ++k) q[k] = in[k * NF * 64];
#pragma unroll
            for (int k = 0; k < CH; ++k) {
                if (k >= n_steps) break;
                const int t = c * CH + k;
                a.v[(unsigned)t * (unsigned)a.Bp + ub] = t < len ? fast_log(q[k]) : 0.0f;      // ln y - ln(S1 S2)
            }
        };
        for (int c = 0; c < n_chunks; ++c) {
            lds_barrier();
            if (c < full_chunks) chunk(c, CH);
            else chunk(c, t_end - c * CH);
        }
    } else {
        auto chunk = [&](int c, int n_steps) {
            const float *in = stage + (c & 1) * (CH * NF * 64) + 128 + lane;
            float s1[CH], s2[CH];
#pragma unroll
            for (int k = 0; k < CH; ++k) {
                s1[k] = NS >= 1 ? in[k * NF * 64] : 1.0f;
                s2[k] = NS >= 2 ? in[k * NF * 64 + 64] : 1.0f;
            }
#pragma unroll
            for (int k = 0; k < CH; ++k) {
                if (k >= n_steps) break;
                const int t = c * CH + k;
                const unsigned at = (unsigned)t * (unsigned)a.Bp + ub;
                if (NS >= 1) a.S1[at] = t < len ? s1[k] : 1.0f;
                if (NS >= 2) a.S2[at] = t < len ? s2[k] : 1.0f;
            }
        };
        for (int c = 0; c < n_chunks; ++c) {
            lds_barrier();
            if (c < full_chunks) chunk(c, CH);
            else chunk(c, t_end - c * CH);
        }
    }
}

// ---------------------------------------------------------------------------
// Windows, Section 5.3 and Eq. (6): with u = ln(level), v = ln y - ln(seasonal
// factors), input x[p][i] = v[p+i] - u[t], target z[p][j] = v[t+j] - u[t],
// t = p + I - 1.  One wave writes one (p, 16-series) tile; every store
// instruction covers 4 rows x 16 series = 256 contiguous bytes.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) window_forward_kernel(const float *__restrict__ u, const float *__restrict__ v,
                                                              float *__restrict__ X, float *__restrict__ Z,
                                                              int P, int NB, int Bp, int I, int H, int xrows, int zrows,
                                                              int p_per_wave, const int32_t *__restrict__ categories,
                                                              int n_cat, int B, const int32_t *__restrict__ pmax)
{
    const int lane = threadIdx.x & 63;
    const int g = lane >> 4, n = lane & 15;
    // the four waves of a workgroup take four adjacent series tiles at the same positions, so that the
    // workgroup writes 1 KB (X, I = 4) and 2 KB (Z, H = 8) contiguous per position
    const int bt = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (bt >= NB) return;
    const int p0 = blockIdx.y * p_per_wave;
    const int col = bt * 16 + n;
    // Section 5.3: the one-hot block of the series' category follows the window (rows I .. I+n_cat-1)
    const int hot = (n_cat > 0 && col < B) ? I + categories[col] : -1;
    const int Pt = min(P, pmax[bt]);     // windows past the tile's longest series are not needed by any later kernel
    for (int p = p0; p < p0 + p_per_wave && p < Pt; ++p) {
        const size_t tile = (size_t)p * NB + bt;
        const int t = p + I - 1;
        const float ut = u[(size_t)t * Bp + col];
        float *xo = X + tile * xrows * 16 + lane;
        // streaming stores: the tiles are consumed by later kernels, not by this one
        for (int r = g; r < xrows; r += 4)
            __builtin_nontemporal_store((r < I) ? v[(size_t)(p + r) * Bp + col] - ut : (r == hot ? 1.0f : 0.0f),
                                        xo + (r - g) * 16);
        float *zo = Z + tile * zrows * 16 + lane;
        for (int r = g; r < zrows; r += 4)
            __builtin_nontemporal_store((r < H) ? v[(size_t)(t + 1 + r) * Bp + col] - ut : 0.0f, zo + (r - g) * 16);
    }
}

// ---------------------------------------------------------------------------
// Loss: sum of the per-workgroup partial sums in double, then
// loss = pinball_sum / n_pin + lambda * level_sum / n_lv.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) loss_finalize_kernel(const float *__restrict__ partial, int n_pin_parts, int n_lv_parts,
                                                             const float *__restrict__ cs_partial, int n_cs_parts,
                                                             const Scalars *__restrict__ sc, float lambda, float lambda_cs,
                                                             float *__restrict__ loss)
{
    __shared__ double s_a[256], s_b[256], s_c[256];
    double a = 0.0, b = 0.0, c = 0.0;
    for (int i = threadIdx.x; i < n_pin_parts; i += 256) a += (double)partial[i];
    for (int i = threadIdx.x; i < n_lv_parts; i += 256) b += (double)partial[n_pin_parts + i];
    for (int i = threadIdx.x; i < n_cs_parts; i += 256) c += (double)cs_partial[i];
    s_a[threadIdx.x] = a;
    s_b[threadIdx.x] = b;
    s_c[threadIdx.x] = c;
    __syncthreads();
    for (int off = 128; off >= 1; off >>= 1) {
        if ((int)threadIdx.x < off) {
            s_a[threadIdx.x] += s_a[threadIdx.x + off];
            s_b[threadIdx.x] += s_b[threadIdx.x + off];
            s_c[threadIdx.x] += s_c[threadIdx.x + off];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0)
        *loss = (float)(s_a[0] * (double)sc->inv_n_pin + (double)lambda * s_b[0] * (double)sc->inv_n_lv +
                        (double)lambda_cs * s_c[0] * (double)sc->inv_n_cs);
}

// Gradient of the level penalty (Section 8.4) with respect to u[t] of one series, times `scale`:
// e[k] = u[k] - 2u[k-1] + u[k-2] for 2 <= k < len; d/du[t] of sum e^2 = 2(e[t] - 2e[t+1] + e[t+2]).
__device__ __forceinline__ float level_penalty_grad(const float *__restrict__ u, int Bp, int col, int t, int len, float scale)
{
    float acc = 0.0f;
#pragma unroll
    for (int dk = 0; dk <= 2; ++dk) {
        const int k = t + dk;
        if (k >= 2 && k < len) {
            const float e = u[(size_t)k * Bp + col] - 2.0f * u[(size_t)(k - 1) * Bp + col] + u[(size_t)(k - 2) * Bp + col];
            acc += (dk == 1 ? -2.0f : 1.0f) * e;
        }
    }
    return scale * acc;
}

// ---------------------------------------------------------------------------
// Window adjoint in gather form (no atomics): every x and z is v[.] - u[t], so
//   gv[k] = sum_i gX[k-i][i] + sum_j gZ[k-(I-1)-j][j],  gu[t] = -(sum of row p = t-I+1),
// with gZ = -gO, plus the gradient of the level penalty (Section 8.4).
// One thread per (t, series); a workgroup takes 64 series at four consecutive t.
//
// Every 128-byte line of gX / gO holds two rows of a tile and is read for two neighbouring t and once
// more for the row sum, by different workgroups.  The workgroups that touch the tiles of one group of 64
// series therefore all run on the same XCD (workgroups go to the XCDs in turn), one after the other in
// time order: the line is then fetched from memory once and found in that XCD's L2 afterwards.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) window_backward_kernel(const float *__restrict__ gX, const float *__restrict__ gO,
                                                               const float *__restrict__ u, const int32_t *__restrict__ lengths,
                                                               const Scalars *__restrict__ sc, float lambda,
                                                               float *__restrict__ gu, float *__restrict__ gv,
                                                               int P_all, int NB, int B, int Bp, int T, int I, int H, int xrows, int zrows,
                                                               const int32_t *__restrict__ pmax, int t_chunks)
{
    // Bp: row stride of the time-major arrays (the batch padded to 64); columns past the 16 * NB series of
    // the tiles have no windows
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int cg = (slot / t_chunks) * 8 + xcd;                 // group of 64 series
    const int t = (slot % t_chunks) * 4 + (threadIdx.x >> 6);
    if (cg * 64 >= Bp || t >= T) return;
    const int col = cg * 64 + (threadIdx.x & 63);
    const size_t idx = (size_t)t * Bp + col;
    if (col >= 16 * NB) {
        gu[idx] = 0.0f;
        gv[idx] = 0.0f;
        return;
    }
    const int bt = col >> 4, n = col & 15;
    const int P = min(P_all, pmax[bt]);      // window gradients past the tile's longest series do not exist
    float sv = 0.0f, su = 0.0f;
    for (int i = 0; i < I; ++i) {
        const int p = t - i;
        if (p >= 0 && p < P) sv += gX[((size_t)(p * NB + bt) * xrows + i) * 16 + n];
    }
    for (int j = 1; j <= H; ++j) {
        const int p = t - (I - 1) - j;
        if (p >= 0 && p < P) sv -= gO[((size_t)(p * NB + bt) * zrows + (j - 1)) * 16 + n];
    }
    {
        const int p = t - I + 1;
        if (p >= 0 && p < P) {
            for (int i = 0; i < I; ++i) su -= gX[((size_t)(p * NB + bt) * xrows + i) * 16 + n];
            for (int j = 0; j < H; ++j) su += gO[((size_t)(p * NB + bt) * zrows + j) * 16 + n];
        }
    }
    if (lambda != 0.0f)
        su += level_penalty_grad(u, Bp, col, t, col < B ? clamp_len(lengths[col], T) : 0, lambda * 2.0f * sc->inv_n_lv);
    gu[idx] = su;
    gv[idx] = sv;
}

// ---------------------------------------------------------------------------
// Window adjoint in streaming form, for batches with many series tiles.  One wave owns a series tile and
// walks over the positions in time order.  Every row group of gX and gO (four rows of 16 series, 256
// contiguous bytes) is loaded exactly once, by one full-width instruction; lane (g, n) adds its element of
// row c of position p to slot (p + c) mod R of a ring of R >= I + H + 4 anti-diagonal sums in LDS (plain read, add,
// write: the lanes of one instruction hit different slots, and the LDS unit serves a wave's instructions in
// order, so no atomic is needed and the sums are formed in a fixed order).  After a block of four positions the four oldest slots are complete:
// lane group g writes gv[s + g] and clears its slot, and writes gu[s + g + I - 1] from the row sum of its
// position.  The gather kernel above reads every element twice in 64-byte pieces; this one is the faster
// of the two once there are enough tiles for the waves to hide each other's memory latency.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) window_backward_stream_kernel(const float *__restrict__ gX, const float *__restrict__ gO,
                                                                      const float *__restrict__ u, const int32_t *__restrict__ lengths,
                                                                      const Scalars *__restrict__ sc, float lambda,
                                                                      float *__restrict__ gu, float *__restrict__ gv,
                                                                      int P_all, int NB, int B, int Bp, int T, int I, int H, int xrows,
                                                                      int zrows, const int32_t *__restrict__ pmax, int R)
{
    extern __shared__ float ring_all[];                     // [wave][R][16]
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int g = lane >> 4, n = lane & 15;
    const int bt = blockIdx.x * 4 + wave;
    if (bt >= NB) return;                                   // (no workgroup barrier below)
    float *ring = ring_all + wave * R * 16;
    for (int e = lane; e < R * 16; e += 64) ring[e] = 0.0f;
    const int mask = R - 1;
    const int Pt = min(P_all, pmax[bt]);
    const int col = bt * 16 + n;
    const int len = col < B ? clamp_len(lengths[col], T) : 0;
    const float pen = lambda * 2.0f * sc->inv_n_lv;
    const int QX = (I + 3) >> 2, Q = QX + ((H + 3) >> 2);   // row groups that hold window elements
    // columns between the last tile and the padded batch: the wave of the last tile clears them
    const int pad_col = 16 * NB + lane;
    const bool pads = bt == NB - 1 && 16 * NB < Bp;         // (wave-uniform)

    for (int s0 = -((I + 2) & ~3); s0 < T; s0 += 4) {      // output block: gv[s0 .. s0+3], gu[s0+I-1 .. s0+I+2]
        float su[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        // the penalty term of this lane's gu row, requested ahead of the gradient tiles: its five loads then
        // travel together with theirs instead of being a second round trip at the end of the block
        const int t_pen = s0 + g + I - 1;
        const float pen_grad = (lambda != 0.0f && t_pen >= 0 && t_pen < T) ? level_penalty_grad(u, Bp, col, t_pen, len, pen) : 0.0f;
        if (s0 + 3 >= 0 && s0 < Pt) {
            for (int e0 = 0; e0 < Q; e0 += 4) {
                float w[4][4];
                // sixteen independent loads in flight, then sixteen LDS additions
#pragma unroll
                for (int sp = 0; sp < 4; ++sp) {
                    const int p = min(max(s0 + sp, 0), Pt - 1);
                    const size_t tile = (size_t)p * NB + bt;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int e = min(e0 + j, Q - 1);
                        const float *src = e < QX ? gX + (tile * xrows + 4 * e) * 16 : gO + (tile * zrows + 4 * (e - QX)) * 16;
                        w[sp][j] = src[lane];
                    }
                }
#pragma unroll
                for (int sp = 0; sp < 4; ++sp) {
                    const int p = s0 + sp;
                    if (p < 0 || p >= Pt) continue;                     // (wave-uniform)
                    // The row groups of one position go to different slots in every lane (row c of the window
                    // part is below I, row c of the horizon part is I or more), so their four read-add-write
                    // sequences are independent: all reads, then all writes.  Two positions do share slots.
                    bool ok[4];
                    int at[4];
                    float val[4], old[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int e = e0 + j;
                        const bool is_x = e < QX;
                        const int r = 4 * (is_x ? e : e - QX) + g;
                        // gX rows past the window (categories, padding) and gO rows past the horizon do not count
                        ok[j] = e < Q && r < (is_x ? I : H);
                        at[j] = ((p + (is_x ? r : I + r)) & mask) * 16 + n;
                        val[j] = is_x ? w[sp][j] : -w[sp][j];           // dL/dz = -dL/do
                        if (ok[j]) old[j] = ring[at[j]];
                    }
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        if (ok[j]) {
                            ring[at[j]] = old[j] + val[j];
                            su[sp] -= val[j];
                        }
                    }
                }
            }
        }
        // row sums over the four lane groups; lane group g keeps the one of position s0 + g
        float mine = 0.0f;
#pragma unroll
        for (int sp = 0; sp < 4; ++sp) {
            float v = su[sp];
            v += __shfl_xor(v, 16, 64);
            v += __shfl_xor(v, 32, 64);
            mine = g == sp ? v : mine;
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        const int s = s0 + g;
        if (s >= 0 && s < T) {
            float *slot = &ring[(s & mask) * 16 + n];
            gv[(size_t)s * Bp + col] = *slot;
            *slot = 0.0f;
        }
        const int t = s + I - 1;
        if (t >= 0 && t < T) {
            gu[(size_t)t * Bp + col] = mine + pen_grad;
        }
        if (pads && pad_col < Bp) {
            for (int k = 0; k < 4; ++k) {
                if (s0 + k >= 0 && s0 + k < T) gv[(size_t)(s0 + k) * Bp + pad_col] = 0.0f;
                if (s0 + k + I - 1 >= 0 && s0 + k + I - 1 < T) gu[(size_t)(s0 + k + I - 1) * Bp + pad_col] = 0.0f;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    }
}

// ---------------------------------------------------------------------------
// Adjoint of the smoothing recursions: reverse sweep over time, one lane per
// series.  Lb is the adjoint of the level; the adjoints of the seasonal factors
// sit in a per-lane LDS ring (slot t mod m holds the adjoint of the factor for
// time t + m when step t starts, and that of time t when it ends).
// ---------------------------------------------------------------------------
struct EsBwdArgs {
    const float *y;
    const int32_t *lengths;
    const float *es;
    const float *lvl, *S1, *S2, *gu, *gv;   // [T][Bp]
    float *grad_es;                          // [K][B]
    int B, Bp, T, n_seas, m1, m2, logit;
    int row_gamma1, row_gamma2, row_s1, row_s2;
};

// Division of labour, as in the forward recursion.  The reverse recursion is linear in the adjoints: at step t
//   Lb   = gu[t] / l[t] + (carry),            x = Lb * alpha * q,   z1 = A1 * g1 * r1,   z2 = A2 * g2 * r2,
//   S1b  = -gv[t] / s1 + A1 (1 - g1) - (z2 + x) / s1,        S2b likewise with the indices exchanged,
//   Lb'  = Lb (1 - alpha) - (z1 + z2) / l[t-1]               (carried to step t-1),
// with q = y / (s1 s2), r1 = y / (l[t-1] s2), r2 = y / (l[t-1] s1): every coefficient depends on the forward
// pass only.  Three helper waves read the rows of a chunk of steps (a chunk ahead), form the twelve
// coefficients of every step - all the divisions - and stage them in LDS; wave 0 carries the adjoints through
// them: a dozen multiply-adds, the ring accesses and nothing else.
constexpr int kEsBwdChunk = 6;                // steps per staging buffer
constexpr int kEsBwdHelpers = 3;              // waves that form coefficients, each every third step
// coefficients per step: four, and four more per seasonality
constexpr int es_bwd_coefs(int n_seas) { return 4 + 4 * n_seas; }
constexpr int es_bwd_stage_floats(int n_seas) { return 2 * kEsBwdChunk * es_bwd_coefs(n_seas) * 64; }

template <int NS>
__global__ void __launch_bounds__(64 * (1 + kEsBwdHelpers)) es_backward_kernel(EsBwdArgs a)
{
    extern __shared__ float ring[];           // [m1 + m2][64] rings, then [2][kEsBwdChunk][4 + 4 NS][64] staging
    constexpr int CH = kEsBwdChunk, NC = es_bwd_coefs(NS);
    const int role = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int b = blockIdx.x * 64 + lane;     // column of the time-major arrays (their rows are padded to whole waves)
    const bool in_batch = b < a.B;
    const int bc = in_batch ? b : a.B - 1;    // column of the arrays with B columns
    const int len = in_batch ? clamp_len(a.lengths[b], a.T) : 0;
    // the sweep starts at the last observation of the wave's longest series (rows beyond were not produced);
    // both waves hold the same 64 series, so the bound is the same in both
    const int t_top = max(wave_max_int(len), 1) - 1;
    float *ring1 = ring, *ring2 = ring + (size_t)a.m1 * 64;
    float *stage = ring + (size_t)(a.m1 + a.m2) * 64;
    float alpha = a.es[bc], g1 = 0.0f, g2 = 0.0f;
    if (NS >= 1) g1 = a.es[(size_t)a.row_gamma1 * a.B + bc];
    if (NS >= 2) g2 = a.es[(size_t)a.row_gamma2 * a.B + bc];
    if (a.logit) {
        alpha = 1.0f / (1.0f + expf(-alpha));
        g1 = 1.0f / (1.0f + expf(-g1));
        g2 = 1.0f / (1.0f + expf(-g2));
    }
    for (int e = threadIdx.x; e < (a.m1 + a.m2) * 64; e += 64 * (1 + kEsBwdHelpers)) ring[e] = 0.0f;
    __syncthreads();
    // The sweep runs over the same times t_top ... 1 in every lane; a lane takes part from its own last
    // observation on (its state updates are switched off before that).  Time, ring slots and row addresses
    // are then wave-uniform.  Rows past a series' length hold defined values (level 1, factors 1, zero
    // adjoints).  Chunk c holds the steps t = t_top - c CH - k, k = 0 .. CH-1, as far as t >= 1.
    const int n_chunks = (t_top + CH - 1) / CH;
    float ab = 0.0f, g1b = 0.0f, g2b = 0.0f;
    float Lb_carry = 0.0f;      // contributions to the adjoint of l[t] from later steps

    // All waves run the same loop and meet at its one barrier: in interval j the helper waves stage chunk j
    // (helper h the steps k = h, h + 3, ...) while wave 0 consumes chunk j - 1 from the other buffer.
    if (role >= 1) {
        constexpr int NK = CH / kEsBwdHelpers;      // steps of a chunk per helper
        static_assert(CH % kEsBwdHelpers == 0, "helpers share a chunk evenly");
        struct Raw { float gu, gv, y, lt, lp, s1, s2; };
        Raw raw[kEsAhead][NK];
        const unsigned ub = b, ubc = bc;
        auto load_chunk = [&](int c, Raw *r) {
#pragma unroll
            for (int i = 0; i < NK; ++i) {
                const int k = (role - 1) + i * kEsBwdHelpers;
                const unsigned tc = (unsigned)max(t_top - c * CH - k, 1);      // steps below 1 are not executed
                // element offsets in 32 bits (B * T is at most 2^30): one scalar multiply per row
                const unsigned at = tc * (unsigned)a.Bp + ub;
                r[i].gu = a.gu[at];
                r[i].gv = a.gv[at];
                r[i].y = a.y[tc * (unsigned)a.B + ubc];
                r[i].lt = a.lvl[at];
                r[i].lp = a.lvl[at - (unsigned)a.Bp];
                r[i].s1 = NS >= 1 ? a.S1[at] : 1.0f;
                r[i].s2 = NS >= 2 ? a.S2[at] : 1.0f;
            }
        };
        // rows are requested kEsAhead chunks ahead (register sets rotating through an unrolled loop, as in the
        // forward recursion)
        static_for<0, kEsAhead>([&](auto d) { load_chunk(decltype(d)::value, raw[decltype(d)::value]); });
        for (int j0 = 0; j0 <= n_chunks; j0 += kEsAhead) {
            static_for<0, kEsAhead>([&](auto dd) {
                constexpr int d = decltype(dd)::value;
                const int j = j0 + d;
                if (j > n_chunks) return;                   // (wave-uniform)
                if (j < n_chunks) {
                    float *out = stage + (j & 1) * (CH * NC * 64) + lane;
#pragma unroll
                    for (int i = 0; i < NK; ++i) {
                        const int k = (role - 1) + i * kEsBwdHelpers;
                        const Raw &r = raw[d][i];
                        const float ilp = fast_rcp(r.lp);
                        const float is1 = NS >= 1 ? fast_rcp(r.s1) : 1.0f, is2 = NS >= 2 ? fast_rcp(r.s2) : 1.0f;
                        const float ry = r.y * ilp;
                        const float r1 = ry * is2, r2 = ry * is1;
                        const float q = r.y * (is1 * is2);
                        float *o = out + k * NC * 64;
                        o[0 * 64] = r.gu * fast_rcp(r.lt);
                        o[1 * 64] = ilp;
                        o[2 * 64] = alpha * q;
                        o[3 * 64] = q - r.lp;
                        if (NS >= 1) {
                            o[4 * 64] = -r.gv * is1;
                            o[5 * 64] = is1;
                            o[6 * 64] = g1 * r1;
                            o[7 * 64] = r1 - r.s1;
                        }
                        if (NS >= 2) {
                            o[8 * 64] = -r.gv * is2;
                            o[9 * 64] = is2;
                            o[10 * 64] = g2 * r2;
                            o[11 * 64] = r2 - r.s2;
                        }
                    }
                    load_chunk(j + kEsAhead, raw[d]);
                }
                lds_barrier();
            });
        }
        return;
    }

    int i1 = NS >= 1 ? t_top % a.m1 : 0, i2 = NS >= 2 ? t_top % a.m2 : 0;   // ring slot of time t: t mod m
    // adjoint of the factor for time t + m, requested one step ahead of its use
    float A1 = 0.0f, A2 = 0.0f;
    const float one_m_alpha = 1.0f - alpha, one_m_g1 = 1.0f - g1, one_m_g2 = 1.0f - g2;
    auto step = [&](int t, const float (&cf)[NC]) {
        const bool active = t <= len - 1;
        // slot of the next step (time t-1): last written m-1 steps ago unless m = 1
        const int j1 = i1 == 0 ? a.m1 - 1 : i1 - 1, j2 = i2 == 0 ? a.m2 - 1 : i2 - 1;
        float A1n = 0.0f, A2n = 0.0f;
        if (NS >= 1) A1n = ring1[j1 * 64 + lane];
        if (NS >= 2) A2n = ring2[j2 * 64 + lane];
        const float Lb = cf[0] + Lb_carry;
        const float ilp = cf[1];
        const float x = Lb * cf[2];
        ab += active ? Lb * cf[3] : 0.0f;
        const float z1 = NS >= 1 ? A1 * cf[NS >= 1 ? 6 : 0] : 0.0f;
        const float z2 = NS >= 2 ? A2 * cf[NS >= 2 ? 10 : 0] : 0.0f;
        if (NS >= 1) {
            const float S1b = cf[NS >= 1 ? 4 : 0] + A1 * one_m_g1 - (z2 + x) * cf[NS >= 1 ? 5 : 0];
            g1b += active ? A1 * cf[NS >= 1 ? 7 : 0] : 0.0f;
            // an inactive lane leaves the slot as it is (zero)
            ring1[i1 * 64 + lane] = active ? S1b : A1;
            A1 = (a.m1 == 1 && active) ? S1b : A1n;
            i1 = j1;
        }
        if (NS >= 2) {
            const float S2b = cf[NS >= 2 ? 8 : 0] + A2 * one_m_g2 - (z1 + x) * cf[NS >= 2 ? 9 : 0];
            g2b += active ? A2 * cf[NS >= 2 ? 11 : 0] : 0.0f;
            ring2[i2 * 64 + lane] = active ? S2b : A2;
            A2 = (a.m2 == 1 && active) ? S2b : A2n;
            i2 = j2;
        }
        const float Lb_prev = Lb * one_m_alpha - (z1 + z2) * ilp;
        Lb_carry = active ? Lb_prev : 0.0f;
    };
    if (NS >= 1) A1 = ring1[i1 * 64 + lane];
    if (NS >= 2) A2 = ring2[i2 * 64 + lane];
    for (int j = 0; j <= n_chunks; ++j) {
        if (j >= 1) {
            const int c = j - 1;
            const float *in = stage + (c & 1) * (CH * NC * 64) + lane;
            const int t_hi = t_top - c * CH;
            // the coefficients of the whole chunk, read together: one LDS round trip per chunk
            float cf[CH][NC];
#pragma unroll
            for (int k = 0; k < CH; ++k)
#pragma unroll
                for (int i = 0; i < NC; ++i) cf[k][i] = in[(k * NC + i) * 64];
            if (t_hi - CH >= 0) {                   // a whole chunk: no branch inside
#pragma unroll
                for (int k = 0; k < CH; ++k) step(t_hi - k, cf[k]);
            } else {
#pragma unroll
                for (int k = 0; k < CH; ++k)
                    if (t_hi - k >= 1) step(t_hi - k, cf[k]);
            }
        }
        lds_barrier();
    }
    if (!in_batch) return;      // (no barrier below)
    if (len >= 1) {
        // t = 0: l[0] = y0 / (S1[0] S2[0]); the first produced factors equal the initial ones
        const size_t o = b;
        const float l0 = a.lvl[o];
        const float Lb = a.gu[o] / l0 + Lb_carry;
        const float gv0 = a.gv[o];
        if (NS >= 1) {
            const float s1 = a.S1[o];
            const float A = (a.m1 <= len - 1) ? ring1[lane] : 0.0f;
            ring1[lane] = -gv0 / s1 + A - Lb * l0 / s1;
        }
        if (NS >= 2) {
            const float s2 = a.S2[o];
            const float A = (a.m2 <= len - 1) ? ring2[lane] : 0.0f;
            ring2[lane] = -gv0 / s2 + A - Lb * l0 / s2;
        }
    }
    a.grad_es[b] = a.logit ? ab * alpha * (1.0f - alpha) : ab;
    if (NS >= 1) {
        a.grad_es[(size_t)a.row_gamma1 * a.B + b] = a.logit ? g1b * g1 * (1.0f - g1) : g1b;
        for (int k = 0; k < a.m1; ++k) {
            float gs = (k < len) ? ring1[k * 64 + lane] : 0.0f;
            if (a.logit) gs *= (k < len) ? a.S1[(size_t)k * a.Bp + b] : 0.0f;
            a.grad_es[(size_t)(a.row_s1 + k) * a.B + b] = gs;
        }
    }
    if (NS >= 2) {
        a.grad_es[(size_t)a.row_gamma2 * a.B + b] = a.logit ? g2b * g2 * (1.0f - g2) : g2b;
        for (int k = 0; k < a.m2; ++k) {
            float gs = (k < len) ? ring2[k * 64 + lane] : 0.0f;
            if (a.logit) gs *= (k < len) ? a.S2[(size_t)k * a.Bp + b] : 0.0f;
            a.grad_es[(size_t)(a.row_s2 + k) * a.B + b] = gs;
        }
    }
}

// ---------------------------------------------------------------------------
// Weight-gradient reduction: sums the per-workgroup (LSTM) and per-wave (head)
// partial tiles in a fixed order and writes the caller's packing.
// ---------------------------------------------------------------------------
// Stage 1: every job (one block of partial results per producer workgroup or
// wave) is cut into `splits` interleaved subsets of the producers; a thread sums
// one element over one subset.  Stage 2 (the kernels below) sums the subsets and
// writes the caller's packing.  Both orders are fixed.
struct ReduceJob {
    const float *src;
    float *dst;          // [splits][n_elems]
    unsigned stride;     // floats between consecutive partial blocks
    int n_part, n_elems, splits;
};
constexpr int kMaxReduceJobs = 2 * kMaxLayers + 1;
struct ReduceJobs {
    ReduceJob job[kMaxReduceJobs];
};

__global__ void __launch_bounds__(256) reduce_stage1_kernel(ReduceJobs jobs)
{
    const ReduceJob &j = jobs.job[blockIdx.z];
    const int e = blockIdx.x * 256 + threadIdx.x, sp = blockIdx.y;
    if (sp >= j.splits || e >= j.n_elems) return;
    const float *src = j.src + e;
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
    int w = sp;
    for (; w + 3 * j.splits < j.n_part; w += 4 * j.splits) {
        a0 += src[(size_t)w * j.stride];
        a1 += src[(size_t)(w + j.splits) * j.stride];
        a2 += src[(size_t)(w + 2 * j.splits) * j.stride];
        a3 += src[(size_t)(w + 3 * j.splits) * j.stride];
    }
    for (; w < j.n_part; w += j.splits) a0 += src[(size_t)w * j.stride];
    j.dst[(size_t)sp * j.n_elems + e] = (a0 + a1) + (a2 + a3);
}

struct ReduceLstmArgs {
    const float *dw_partial, *db_partial;
    float *gW, *gb;
    int NB, h, in_dim, HT, KXT;
};

// Sums `n_part` partial blocks for 64 consecutive elements per workgroup: the
// four waves take interleaved quarters of the partials (each load instruction
// reads 256 contiguous bytes of one partial), then combine in a fixed order.
__device__ __forceinline__ float reduce_partials(const float *__restrict__ base, size_t stride, int n_part, int elem,
                                                 bool active, float (*s_red)[64])
{
    const int e = threadIdx.x & 63, sl = threadIdx.x >> 6;
    float acc = 0.0f;
    if (active) {
        const float *src = base + elem;
        int w = sl;
        for (; w + 12 < n_part; w += 16) {
            const float a0 = src[(size_t)w * stride], a1 = src[(size_t)(w + 4) * stride];
            const float a2 = src[(size_t)(w + 8) * stride], a3 = src[(size_t)(w + 12) * stride];
            acc += (a0 + a1) + (a2 + a3);
        }
        for (; w < n_part; w += 4) acc += src[(size_t)w * stride];
    }
    s_red[sl][e] = acc;
    __syncthreads();
    return (s_red[0][e] + s_red[1][e]) + (s_red[2][e] + s_red[3][e]);
}

__device__ void reduce_lstm_body(const ReduceLstmArgs &a, float (*s_red)[64])
{
    const int KT = a.KXT + a.HT, MB = (KT + 3) / 4, ld = a.in_dim + a.h;
    const int n_dw = a.HT * MB * 256, n_db = a.HT * 16;
    const int n_dw_blocks = (n_dw + 63) / 64;
    const int e = threadIdx.x & 63;
    if ((int)blockIdx.x < n_dw_blocks) {
        const int idx = blockIdx.x * 64 + e;                  // element of the tile block: [tile][component][lane]
        const float tot = reduce_partials(a.dw_partial, (size_t)n_dw, a.NB, idx, idx < n_dw, s_red);
        if (threadIdx.x < 64 && idx < n_dw) {
            const int lane = idx & 63, comp = (idx >> 6) & 3, tix = idx >> 8;
            const int mt = tix / MB, nbk = tix % MB;
            // tile row 4*gate + unit-in-tile sits in lane group `gate`, component `unit-in-tile`
            const int gate = lane >> 4, unit = 4 * mt + comp;
            const int xr = 16 * nbk + (lane & 15);
            int col = -1;
            if (xr < 4 * a.KXT) { if (xr < a.in_dim) col = xr; }
            else if (xr - 4 * a.KXT < a.h) col = a.in_dim + xr - 4 * a.KXT;
            if (unit < a.h && col >= 0) a.gW[(size_t)(gate * a.h + unit) * ld + col] = tot;
        }
    } else {
        const int idx = (blockIdx.x - n_dw_blocks) * 64 + e;   // [unit tile][unit][gate]
        const float tot = reduce_partials(a.db_partial, (size_t)n_db, a.NB, idx, idx < n_db, s_red);
        if (threadIdx.x < 64 && idx < n_db) {
            const int gate = idx & 3, unit = idx >> 2;
            if (unit < a.h) a.gb[gate * a.h + unit] = tot;
        }
    }
}

struct ReduceHeadArgs {
    const float *partial;
    float *gWa, *gba, *gWo, *gbo;
    int n_part, stride, h, H, HT, MA, MO, OT;
};

__device__ void reduce_head_body(const ReduceHeadArgs &a, float (*s_red)[64])
{
    // partial block: dWo tiles [MO*MA][4][64], dWa tiles [MA*MA][4][64], dbo [4*OT], dba [4*HT]
    const int offWa = a.MO * a.MA * 256, offbo = offWa + a.MA * a.MA * 256, offba = offbo + 4 * a.OT;
    const int n = offba + 4 * a.HT;
    const int idx = blockIdx.x * 64 + (threadIdx.x & 63);
    const float tot = reduce_partials(a.partial, (size_t)a.stride, a.n_part, idx, idx < n, s_red);
    if (threadIdx.x >= 64 || idx >= n) return;
    if (idx < offbo) {
        const bool isWa = idx >= offWa;
        const int j = isWa ? idx - offWa : idx;
        const int lane = j & 63, comp = (j >> 6) & 3, tix = j >> 8;
        const int mt = tix / a.MA, nt = tix % a.MA;
        const int row = 16 * mt + 4 * (lane >> 4) + comp, col = 16 * nt + (lane & 15);
        if (col < a.h) {
            if (isWa) { if (row < a.h) a.gWa[row * a.h + col] = tot; }
            else if (row < a.H) a.gWo[row * a.h + col] = tot;
        }
    } else if (idx < offba) {
        const int j = idx - offbo;
        if (j < a.H) a.gbo[j] = tot;
    } else {
        const int j = idx - offba;
        if (j < a.h) a.gba[j] = tot;
    }
}

struct ReduceStage2Args {
    ReduceLstmArgs lstm[kMaxLayers];
    ReduceHeadArgs head;
    int L;
};

__global__ void __launch_bounds__(256) reduce_stage2_kernel(ReduceStage2Args a)
{
    __shared__ float s_red[4][64];
    const int z = blockIdx.z;
    if (z < a.L) reduce_lstm_body(a.lstm[z], s_red);
    else reduce_head_body(a.head, s_red);
}

}  // namespace

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
namespace {
// Dynamic LDS above 64 KB has to be allowed per kernel.  Done once per kernel and device for the whole
// 160 KB, on the first launch that needs it (not on every launch: the call is not a stream operation).
hipError_t allow_large_lds(const void *kernel, size_t lds)
{
    if (lds <= 64 * 1024) return hipSuccess;
    constexpr int kMaxKernels = 32, kMaxDevices = 64;
    static std::mutex mu;
    static const void *known[kMaxKernels];
    static bool done[kMaxKernels][kMaxDevices];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mu);
    int slot = -1;
    for (int i = 0; i < kMaxKernels && slot < 0; ++i)
        if (known[i] == kernel || known[i] == nullptr) { known[i] = kernel; slot = i; }
    if (slot >= 0 && dev >= 0 && dev < kMaxDevices && done[slot][dev]) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e == hipSuccess && slot >= 0 && dev >= 0 && dev < kMaxDevices) done[slot][dev] = true;
    return e;
}
}  // namespace

hipError_t launch_setup(const Plan &pl, const int32_t *lengths, const float *weights, float *ws, hipStream_t st)
{
    SetupArgs a{};
    a.L = pl.L;
    a.pack = weights != nullptr;
    a.prep = PrepArgs{lengths, reinterpret_cast<Scalars *>(ws + pl.scalars), reinterpret_cast<int32_t *>(ws + pl.pmax), pl.NB,
                      pl.B, pl.T, pl.I, pl.H, pl.h * pl.cfg.n_blocks};
    if (!a.pack) {
        // block 0 counts the loss normalisers, the others find the position bound of every tile
        setup_kernel<<<dim3(1 + std::min((pl.NB + 255) / 256, 63), 1, 1), 256, 0, st>>>(a);
        return hipGetLastError();
    }
    int max_total = 256;
    for (int l = 0; l < pl.L; ++l) {
        const LayerPlan &lp = pl.layer[l];
        a.lstm[l] = PackLstmArgs{weights + lp.w_off, weights + lp.b_off, ws + lp.wpack_fwd, ws + lp.bias_pack,
                                 ws + lp.wpack_bwd, pl.h, lp.in_dim, pl.HT, lp.KXT, lp.narrow};
        const int KT = lp.KXT + pl.HT, MB = (KT + 3) / 4;
        max_total = std::max(max_total, lp.narrow ? 4 * 4 * KT * 64 + 4 * ((4 * KT + 63) / 64) * 4 * pl.HT * 64
                                                  : pl.HT * KT * 64 + pl.HT * 16 + MB * 4 * pl.HT * 64);
    }
    const HeadPack hp = head_pack_layout(pl);
    float *f = ws + pl.head_fwd_pack, *b = ws + pl.head_bwd_pack;
    a.head = PackHeadArgs{weights + pl.Wa_off, weights + pl.ba_off, weights + pl.Wo_off, weights + pl.bo_off,
                          f + hp.WaF, f + hp.baF, f + hp.WoF, f + hp.boF, b + hp.WoT, b + hp.WaT,
                          pl.h, pl.H, pl.HT, pl.MA, pl.MO, pl.OT};
    const int blocks = std::max(2, std::min((max_total + 255) / 256, 64));   // the bodies loop over their elements
    setup_kernel<<<dim3(blocks, 1, pl.L + 2), 256, 0, st>>>(a);
    return hipGetLastError();
}

hipError_t launch_es_forward(const Plan &pl, const float *y, const int32_t *lengths, const float *es, float *ws,
                             hipStream_t st)
{
    const esrnn_config &c = pl.cfg;
    EsArgs a{y, lengths, es, ws + pl.lvl, ws + pl.S1, ws + pl.S2, ws + pl.u, ws + pl.v,
             ws + pl.loss_partial + (pl.n_loss_partial - pl.es_blocks),
             pl.B, pl.Bt, pl.T, c.n_seas, c.n_seas >= 1 ? c.m1 : 0, c.n_seas >= 2 ? c.m2 : 0,
             c.param_space == ESRNN_PARAMS_LOGIT, pl.row_gamma1, pl.row_gamma2, pl.row_s1, pl.row_s2};
    const size_t lds = ((size_t)(a.m1 + a.m2) * 64 + es_stage_floats(c.n_seas)) * sizeof(float);
    auto run = [&](auto kernel) {
        hipError_t e = allow_large_lds(reinterpret_cast<const void *>(kernel), lds);
        if (e != hipSuccess) return e;
        kernel<<<pl.es_blocks, c.n_seas == 0 ? 192 : 256, lds, st>>>(a);
        return hipGetLastError();
    };
    // steps per group: the largest divisor of 8 that no period is shorter than
    int m_min = 8;
    if (c.n_seas >= 1) m_min = std::min(m_min, c.m1);
    if (c.n_seas >= 2) m_min = std::min(m_min, c.m2);
    const int cs = m_min >= 8 ? 8 : (m_min >= 4 ? 4 : (m_min >= 2 ? 2 : 1));
    if (c.n_seas == 0) return run(es_forward_kernel<0, 8>);
    if (c.n_seas == 1) {
        if (cs == 8) return run(es_forward_kernel<1, 8>);
        if (cs == 4) return run(es_forward_kernel<1, 4>);
        if (cs == 2) return run(es_forward_kernel<1, 2>);
        return run(es_forward_kernel<1, 1>);
    }
    if (cs == 8) return run(es_forward_kernel<2, 8>);
    if (cs == 4) return run(es_forward_kernel<2, 4>);
    if (cs == 2) return run(es_forward_kernel<2, 2>);
    return run(es_forward_kernel<2, 1>);
}

hipError_t launch_window_forward(const Plan &pl, const int32_t *categories, float *ws, hipStream_t st)
{
    // few positions per wave at small batches (enough waves), more at large ones (less per-wave overhead)
    const int p_per_wave = pl.NB >= 2048 ? 8 : (pl.NB >= 512 ? 4 : 1);
    window_forward_kernel<<<dim3((pl.NB + 3) / 4, (pl.P + p_per_wave - 1) / p_per_wave), 256, 0, st>>>(ws + pl.u, ws + pl.v, ws + pl.X, ws + pl.Z,
                                                                         pl.P, pl.NB, pl.Bt, pl.I, pl.H, 4 * pl.IT,
                                                                         pl.OP, p_per_wave, categories, pl.C, pl.B,
                                                                         reinterpret_cast<const int32_t *>(ws + pl.pmax));
    return hipGetLastError();
}

hipError_t launch_loss_finalize(const Plan &pl, float *ws, float *loss, hipStream_t st)
{
    loss_finalize_kernel<<<1, 256, 0, st>>>(ws + pl.loss_partial, pl.n_loss_partial - pl.es_blocks, pl.es_blocks,
                                            ws + pl.cs_partial, pl.n_cs_partial,
                                            reinterpret_cast<const Scalars *>(ws + pl.scalars), pl.cfg.lambda_lv,
                                            pl.cfg.lambda_cs, loss);
    return hipGetLastError();
}

hipError_t launch_window_backward(const Plan &pl, const int32_t *lengths, float *ws, hipStream_t st)
{
    const Scalars *sc = reinterpret_cast<const Scalars *>(ws + pl.scalars);
    const int32_t *pmax = reinterpret_cast<const int32_t *>(ws + pl.pmax);
    if (pl.window_stream) {
        int R = 16;
        while (R < pl.I + pl.H + 4) R *= 2;                 // ring of anti-diagonal sums, a power of two
        window_backward_stream_kernel<<<(unsigned)((pl.NB + 3) / 4), 256, (size_t)4 * R * 16 * sizeof(float), st>>>(
            ws + pl.gX, ws + pl.gO, ws + pl.u, lengths, sc, pl.cfg.lambda_lv, ws + pl.gu, ws + pl.gv, pl.P, pl.NB, pl.B,
            pl.Bt, pl.T, pl.I, pl.H, 4 * pl.IT, pl.OP, pmax, R);
        return hipGetLastError();
    }
    const int t_chunks = (pl.T + 3) / 4;                    // four time steps per workgroup
    const int col_slots = (pl.Bt / 64 + 7) / 8;             // groups of 64 series per XCD
    window_backward_kernel<<<(unsigned)(8 * col_slots * t_chunks), 256, 0, st>>>(
        ws + pl.gX, ws + pl.gO, ws + pl.u, lengths, sc, pl.cfg.lambda_lv, ws + pl.gu, ws + pl.gv, pl.P, pl.NB, pl.B, pl.Bt,
        pl.T, pl.I, pl.H, 4 * pl.IT, pl.OP, pmax, t_chunks);
    return hipGetLastError();
}

hipError_t launch_es_backward(const Plan &pl, const float *y, const int32_t *lengths, const float *es, float *ws,
                              float *grad_es, hipStream_t st)
{
    const esrnn_config &c = pl.cfg;
    EsBwdArgs a{y, lengths, es, ws + pl.lvl, ws + pl.S1, ws + pl.S2, ws + pl.gu, ws + pl.gv, grad_es,
                pl.B, pl.Bt, pl.T, c.n_seas, c.n_seas >= 1 ? c.m1 : 0, c.n_seas >= 2 ? c.m2 : 0,
                c.param_space == ESRNN_PARAMS_LOGIT, pl.row_gamma1, pl.row_gamma2, pl.row_s1, pl.row_s2};
    const size_t lds = ((size_t)(a.m1 + a.m2) * 64 + es_bwd_stage_floats(c.n_seas)) * sizeof(float);
    auto run = [&](auto kernel) {
        hipError_t e = allow_large_lds(reinterpret_cast<const void *>(kernel), lds);
        if (e != hipSuccess) return e;
        kernel<<<(pl.B + 63) / 64, 64 * (1 + kEsBwdHelpers), lds, st>>>(a);
        return hipGetLastError();
    };
    if (c.n_seas == 0) return run(es_backward_kernel<0>);
    if (c.n_seas == 1) return run(es_backward_kernel<1>);
    return run(es_backward_kernel<2>);
}

// ---------------------------------------------------------------------------
// Out-of-sample forecasts, Section 3.4 with Eq. (4) and (5).  The forward pass is
// run with every length extended by H: the window that ends at a series' last
// observation then counts as a complete window (its "targets" are rows past the
// series and never reach the forecast), and the network is causal in the window
// position, so its output there is the out-of-sample output.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) extend_lengths_kernel(const int32_t *__restrict__ lengths, int32_t *__restrict__ ext,
                                                              int B, int T, int I, int H)
{
    const int b = blockIdx.x * 256 + threadIdx.x;
    if (b >= B) return;
    const int len = lengths[b];
    ext[b] = (len >= I && len <= T - H) ? len + H : 0;   // 0: the series takes no part
}

// forecast[b][h-1] = exp(output_h + ln l_t) * S1[t + ((h-1) mod m1) + 1] * S2[...], t = len-1: the last m
// factors the recursion produced, repeated with their period (Eq. (4)).
__global__ void __launch_bounds__(256) forecast_tail_kernel(const float *__restrict__ O, const float *__restrict__ u,
                                                             const float *__restrict__ S1, const float *__restrict__ S2,
                                                             const int32_t *__restrict__ lengths, float *__restrict__ out,
                                                             int B, int Bp, int NB, int T, int I, int H, int orows,
                                                             int m1, int m2)
{
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= B * H) return;
    const int b = idx / H, j = idx % H;
    const int len = lengths[b];
    float f = 0.0f;
    if (len >= I && len <= T - H) {
        const int t = len - 1, p = len - I;
        const float o = O[(((size_t)p * NB + (b >> 4)) * orows + j) * 16 + (b & 15)];
        float sv = 1.0f;
        if (m1 > 0) sv = S1[(size_t)(t + (j % m1) + 1) * Bp + b];
        if (m2 > 0) sv *= S2[(size_t)(t + (j % m2) + 1) * Bp + b];
        f = __expf(o + u[(size_t)t * Bp + b]) * sv;
    }
    out[idx] = f;
}

// Accuracy of forecasts against actual values, per series (Section 3.5 names the two metrics of the
// M4 competition): sMAPE = mean_h 200 |a - f| / (|a| + |f|); MASE = mean_h |a - f| divided by the
// in-sample mean of |y_t - y_{t-m}|, t = m .. len-1 (seasonal naive forecast of period m).
__global__ void __launch_bounds__(256) forecast_metrics_kernel(const float *__restrict__ f, const float *__restrict__ a,
                                                                const float *__restrict__ y, const int32_t *__restrict__ lengths,
                                                                float *__restrict__ smape, float *__restrict__ mase,
                                                                int B, int T, int H, int m)
{
    const int b = blockIdx.x * 256 + threadIdx.x;
    if (b >= B) return;
    float s_sym = 0.0f, s_abs = 0.0f;
    for (int j = 0; j < H; ++j) {
        const float fv = f[(size_t)b * H + j], av = a[(size_t)b * H + j];
        const float d = fabsf(av - fv);
        s_sym += 200.0f * d / (fabsf(av) + fabsf(fv));
        s_abs += d;
    }
    const int len = clamp_len(lengths[b], T);
    float s_naive = 0.0f;
    for (int t = m; t < len; ++t) s_naive += fabsf(y[(size_t)t * B + b] - y[(size_t)(t - m) * B + b]);
    smape[b] = s_sym / (float)H;
    mase[b] = (s_abs / (float)H) / (s_naive / (float)(len - m));
}

hipError_t launch_extend_lengths(const Plan &pl, const int32_t *lengths, float *ws, hipStream_t st)
{
    extend_lengths_kernel<<<(pl.B + 255) / 256, 256, 0, st>>>(lengths, reinterpret_cast<int32_t *>(ws + pl.len_ext),
                                                               pl.B, pl.T, pl.I, pl.H);
    return hipGetLastError();
}

hipError_t launch_forecast_tail(const Plan &pl, const int32_t *lengths, float *ws, float *out, hipStream_t st)
{
    const esrnn_config &c = pl.cfg;
    const int n = pl.B * pl.H;
    forecast_tail_kernel<<<(n + 255) / 256, 256, 0, st>>>(ws + pl.O, ws + pl.u, ws + pl.S1, ws + pl.S2, lengths, out,
                                                          pl.B, pl.Bt, pl.NB, pl.T, pl.I, pl.H, pl.OP,
                                                          c.n_seas >= 1 ? c.m1 : 0, c.n_seas >= 2 ? c.m2 : 0);
    return hipGetLastError();
}

hipError_t launch_forecast_metrics(const Plan &pl, const float *forecasts, const float *actuals, const float *y,
                                   const int32_t *lengths, int m, float *smape, float *mase, hipStream_t st)
{
    forecast_metrics_kernel<<<(pl.B + 255) / 256, 256, 0, st>>>(forecasts, actuals, y, lengths, smape, mase,
                                                                 pl.B, pl.T, pl.H, m);
    return hipGetLastError();
}

hipError_t launch_reduce_weight_grads(const Plan &pl, float *ws, float *grad_weights, hipStream_t st)
{
    ReduceJobs jobs{};
    int nj = 0, max_elems = 0, max_splits = 1;
    auto add = [&](size_t src, size_t dst, size_t stride, int n_part, int n_elems) {
        const int splits = n_part < kReduceSplits ? n_part : kReduceSplits;
        jobs.job[nj++] = ReduceJob{ws + src, ws + dst, (unsigned)stride, n_part, n_elems, splits};
        if (n_elems > max_elems) max_elems = n_elems;
        if (splits > max_splits) max_splits = splits;
        return splits;
    };
    int lstm_splits[kMaxLayers];
    for (int l = 0; l < pl.L; ++l) {
        const LayerPlan &lp = pl.layer[l];
        const int MB = (lp.KXT + pl.HT + 3) / 4;
        const int n_dw = pl.HT * MB * 256, n_db = pl.HT * 16;
        lstm_splits[l] = add(lp.dw_partial, lp.dw_reduced, n_dw, pl.partial_groups(lp), n_dw);
        add(lp.db_partial, lp.db_reduced, n_db, pl.partial_groups(lp), n_db);
    }
    const int n_head = (pl.MO * pl.MA + pl.MA * pl.MA) * 256 + 4 * pl.OT + 4 * pl.HT;
    const int head_splits = add(pl.head_dw_partial, pl.head_dw_reduced, pl.head_dw_stride, pl.n_head_waves, n_head);
    reduce_stage1_kernel<<<dim3((max_elems + 255) / 256, max_splits, nj), 256, 0, st>>>(jobs);

    ReduceStage2Args r{};
    r.L = pl.L;
    int max_blocks = (n_head + 63) / 64;
    for (int l = 0; l < pl.L; ++l) {
        const LayerPlan &lp = pl.layer[l];
        r.lstm[l] = ReduceLstmArgs{ws + lp.dw_reduced, ws + lp.db_reduced, grad_weights + lp.w_off,
                                   grad_weights + lp.b_off, lstm_splits[l], pl.h, lp.in_dim, pl.HT, lp.KXT};
        const int MB = (lp.KXT + pl.HT + 3) / 4;
        max_blocks = std::max(max_blocks, (pl.HT * MB * 256 + 63) / 64 + (pl.HT * 16 + 63) / 64);
    }
    r.head = ReduceHeadArgs{ws + pl.head_dw_reduced, grad_weights + pl.Wa_off, grad_weights + pl.ba_off,
                            grad_weights + pl.Wo_off, grad_weights + pl.bo_off,
                            head_splits, n_head, pl.h, pl.H, pl.HT, pl.MA, pl.MO, pl.OT};
    reduce_stage2_kernel<<<dim3(max_blocks, 1, pl.L + 1), 256, 0, st>>>(r);
    return hipGetLastError();
}

}  // namespace esrnn
