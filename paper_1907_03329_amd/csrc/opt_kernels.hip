// Parameter update after a training step: gradient clipping by the global L2 norm and the Adam rule
// (Kingma & Ba, 2015, Algorithm 1, with bias correction), for the shared network weights and the
// per-series smoothing parameters that are trained jointly (Section 3.3).  The paper does not name its
// optimiser; this is the published algorithm, stated in the header of the library.
//
// Two launches, both deterministic: per-workgroup sums of squares in a fixed order, then an elementwise
// update in which every workgroup adds up the same partial sums in the same order to get the clipping
// factor.
#include "device_utils.h"
#include "esrnn_internal.h"

namespace esrnn {

namespace {

constexpr int kNormBlocks = 128;   // at most 256: the update kernel adds them up with one thread each

__global__ void __launch_bounds__(256) grad_sumsq_kernel(const float *__restrict__ ga, size_t na,
                                                          const float *__restrict__ gb, size_t nb,
                                                          float *__restrict__ partial)
{
    __shared__ float s_w[4];
    float acc = 0.0f;
    const size_t n = na + nb;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        const float g = i < na ? ga[i] : gb[i - na];
        acc += g * g;
    }
    const float w = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) s_w[threadIdx.x >> 6] = w;
    __syncthreads();
    if (threadIdx.x == 0) partial[blockIdx.x] = (s_w[0] + s_w[1]) + (s_w[2] + s_w[3]);
}

struct AdamArgs {
    float *p;
    const float *g;
    float *m, *v;
    size_t n;
    float lr;
};

__global__ void __launch_bounds__(256) adam_kernel(AdamArgs wa, AdamArgs ea, const float *__restrict__ partial, int n_partial,
                                                    float clip_norm, float beta1, float beta2, float eps,
                                                    float corr1, float corr2)
{
    // clipping factor: min(1, clip / (norm + 1e-6)); every workgroup adds the partials up in the same
    // (tree) order, in double
    __shared__ double s_tot[256];
    __shared__ float s_scale;
    s_tot[threadIdx.x] = (clip_norm > 0.0f && (int)threadIdx.x < n_partial) ? (double)partial[threadIdx.x] : 0.0;
    __syncthreads();
    for (int off = 128; off >= 1; off >>= 1) {
        if ((int)threadIdx.x < off) s_tot[threadIdx.x] += s_tot[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) s_scale = clip_norm > 0.0f ? fminf(1.0f, clip_norm / ((float)sqrt(s_tot[0]) + 1e-6f)) : 1.0f;
    __syncthreads();
    const float scale = s_scale;
    const size_t n = wa.n + ea.n;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        const bool first = i < wa.n;
        const AdamArgs &a = first ? wa : ea;
        const size_t k = first ? i : i - wa.n;
        const float g = a.g[k] * scale;
        const float m = beta1 * a.m[k] + (1.0f - beta1) * g;
        const float v = beta2 * a.v[k] + (1.0f - beta2) * g * g;
        a.m[k] = m;
        a.v[k] = v;
        // bias-corrected moments: m / (1 - beta1^t), v / (1 - beta2^t)
        a.p[k] -= a.lr * (m * corr1) / (sqrtf(v * corr2) + eps);
    }
}

// ---------------------------------------------------------------------------
// Training over a store of N series, a batch of B at a time (Section 3.3: every series has its own
// smoothing parameters; Table 5: epochs of batches).  gather: the batch's series, lengths and parameters
// out of the store; indexed update: Adam on the shared weights, and on the store columns named by the
// batch index only, each series with its own update counter in the bias correction.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) gather_batch_kernel(const float *__restrict__ store_y, const int32_t *__restrict__ store_len,
                                                            const float *__restrict__ store_es, const int32_t *__restrict__ index,
                                                            float *__restrict__ y, int32_t *__restrict__ len, float *__restrict__ es,
                                                            int B, int N, int T, int K)
{
    const int b = blockIdx.x * 256 + threadIdx.x;
    if (b >= B) return;
    const int n = index[b];
    // rows of one kind per blockIdx.y: 0 .. T-1 series values, T .. T+K-1 parameters, T+K lengths
    for (int r = blockIdx.y; r < T + K + 1; r += gridDim.y) {
        if (r < T) y[(size_t)r * B + b] = store_y[(size_t)r * N + n];
        else if (r < T + K) es[(size_t)(r - T) * B + b] = store_es[(size_t)(r - T) * N + n];
        else len[b] = store_len[n];
    }
}

struct IndexedArgs {
    float *p;            // [K][N]
    const float *g;      // [K][B]
    float *m, *v;        // [K][N]
    const int32_t *index;   // [B]
    const int32_t *counts;  // [N] updates each series has had so far
    int B, N, K;
    float lr;
};

__global__ void __launch_bounds__(256) adam_indexed_kernel(AdamArgs wa, IndexedArgs ea, const float *__restrict__ partial,
                                                            int n_partial, float clip_norm, float beta1, float beta2,
                                                            float eps, float corr1, float corr2)
{
    __shared__ double s_tot[256];
    __shared__ float s_scale;
    s_tot[threadIdx.x] = (clip_norm > 0.0f && (int)threadIdx.x < n_partial) ? (double)partial[threadIdx.x] : 0.0;
    __syncthreads();
    for (int off = 128; off >= 1; off >>= 1) {
        if ((int)threadIdx.x < off) s_tot[threadIdx.x] += s_tot[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) s_scale = clip_norm > 0.0f ? fminf(1.0f, clip_norm / ((float)sqrt(s_tot[0]) + 1e-6f)) : 1.0f;
    __syncthreads();
    const float scale = s_scale;
    const size_t ne = (size_t)ea.K * ea.B, n = wa.n + ne;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        if (i < wa.n) {
            const float g = wa.g[i] * scale;
            const float m = beta1 * wa.m[i] + (1.0f - beta1) * g;
            const float v = beta2 * wa.v[i] + (1.0f - beta2) * g * g;
            wa.m[i] = m;
            wa.v[i] = v;
            wa.p[i] -= wa.lr * (m * corr1) / (sqrtf(v * corr2) + eps);
        } else {
            const size_t e = i - wa.n;
            const int k = (int)(e / ea.B), b = (int)(e % ea.B);
            const int col = ea.index[b];
            const size_t at = (size_t)k * ea.N + col;
            // bias correction with the series' own counter (in double: K*B elements only)
            const double t = (double)(ea.counts[col] + 1);
            const float c1 = (float)(1.0 / (1.0 - pow((double)beta1, t)));
            const float c2 = (float)(1.0 / (1.0 - pow((double)beta2, t)));
            const float g = ea.g[e] * scale;
            const float m = beta1 * ea.m[at] + (1.0f - beta1) * g;
            const float v = beta2 * ea.v[at] + (1.0f - beta2) * g * g;
            ea.m[at] = m;
            ea.v[at] = v;
            ea.p[at] -= ea.lr * (m * c1) / (sqrtf(v * c2) + eps);
        }
    }
}

__global__ void __launch_bounds__(256) bump_counts_kernel(const int32_t *__restrict__ index, int32_t *__restrict__ counts, int B)
{
    const int b = blockIdx.x * 256 + threadIdx.x;
    if (b < B) counts[index[b]] += 1;
}

}  // namespace

hipError_t launch_gather_batch(const Plan &pl, const float *store_y, const int32_t *store_len, const float *store_es,
                               const int32_t *index, int N, float *y, int32_t *len, float *es, hipStream_t st)
{
    const int rows = pl.T + pl.K + 1;
    gather_batch_kernel<<<dim3((pl.B + 255) / 256, std::min(rows, 64)), 256, 0, st>>>(store_y, store_len, store_es, index, y, len,
                                                                                      es, pl.B, N, pl.T, pl.K);
    return hipGetLastError();
}

hipError_t launch_adam_update_indexed(const Plan &pl, const esrnn_adam_config &opt, int step, float *weights,
                                      const float *grad_weights, float *m_w, float *v_w, float *es_store,
                                      const float *grad_es, float *m_es, float *v_es, int32_t *counts,
                                      const int32_t *index, int N, float *ws, hipStream_t st)
{
    const size_t nw = pl.n_weights, ne = (size_t)pl.K * pl.B;
    float *partial = ws + pl.opt_partial;
    if (opt.clip_norm > 0.0f) {
        grad_sumsq_kernel<<<kNormBlocks, 256, 0, st>>>(grad_weights, nw, grad_es, ne, partial);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    const double c1 = 1.0 / (1.0 - pow((double)opt.beta1, (double)step));
    const double c2 = 1.0 / (1.0 - pow((double)opt.beta2, (double)step));
    AdamArgs wa{weights, grad_weights, m_w, v_w, nw, opt.lr_weights};
    IndexedArgs ea{es_store, grad_es, m_es, v_es, index, counts, pl.B, N, pl.K, opt.lr_es};
    const unsigned blocks = (unsigned)std::min<size_t>((nw + ne + 255) / 256, 2048);
    adam_indexed_kernel<<<blocks, 256, 0, st>>>(wa, ea, partial, kNormBlocks, opt.clip_norm, opt.beta1, opt.beta2, opt.eps,
                                                 (float)c1, (float)c2);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    bump_counts_kernel<<<(pl.B + 255) / 256, 256, 0, st>>>(index, counts, pl.B);
    return hipGetLastError();
}

hipError_t launch_adam_update(const Plan &pl, const esrnn_adam_config &opt, int step, float *weights,
                              const float *grad_weights, float *m_w, float *v_w, float *es_params,
                              const float *grad_es, float *m_es, float *v_es, float *ws, hipStream_t st)
{
    const size_t nw = pl.n_weights, ne = (size_t)pl.K * pl.B;
    float *partial = ws + pl.opt_partial;
    if (opt.clip_norm > 0.0f) {
        grad_sumsq_kernel<<<kNormBlocks, 256, 0, st>>>(grad_weights, nw, grad_es, ne, partial);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    const double c1 = 1.0 / (1.0 - pow((double)opt.beta1, (double)step));
    const double c2 = 1.0 / (1.0 - pow((double)opt.beta2, (double)step));
    AdamArgs wa{weights, grad_weights, m_w, v_w, nw, opt.lr_weights};
    AdamArgs ea{es_params, grad_es, m_es, v_es, ne, opt.lr_es};
    const unsigned blocks = (unsigned)std::min<size_t>((nw + ne + 255) / 256, 2048);
    adam_kernel<<<blocks, 256, 0, st>>>(wa, ea, partial, kNormBlocks, opt.clip_norm, opt.beta1, opt.beta2, opt.eps,
                                         (float)c1, (float)c2);
    return hipGetLastError();
}

}  // namespace esrnn
