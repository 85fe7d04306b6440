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

}  // namespace

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
