// Diagnostic kernel: do fp32 MFMA instructions and ordinary vector instructions of one SIMD run at the
// same time?  The LSTM kernels are priced against the fp32 matrix peak; how much of a SIMD's time their
// elementwise work takes away from the matrix pipe depends on the answer, which this probe measures
// rather than assumes.  Synthetic registers only: no input, one float per thread written at the end so
// that the work is not removed.
#include "device_utils.h"
#include "esrnn_internal.h"

#include <mutex>

namespace esrnn {
namespace {

constexpr int kProbeLds = 80 * 1024;   // per workgroup: at most two workgroups share a compute unit

template <int NM, int NV>
__device__ __forceinline__ void probe_body(f32x4 (&acc)[4], float (&v)[8], float a, float b, int iterations)
{
    for (int it = 0; it < iterations; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            if (i < NM) acc[i & 3] = mfma16(a, b, acc[i & 3]);
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (i * 4 + k < NV) v[(i * 4 + k) & 7] = __builtin_fmaf(v[(i * 4 + k) & 7], a, b);
        }
    }
}

__global__ void __launch_bounds__(256) probe_issue_overlap_kernel(float *out, int mode, int iterations)
{
    extern __shared__ float probe_lds[];
    f32x4 acc[4] = {};
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = threadIdx.x * 0.001f + i;
    const float a = 1.0f + threadIdx.x * 1e-6f, b = 1e-7f;
    const int role = mode == 3 ? (int)(blockIdx.y & 1) : mode;
    if (role == 0) probe_body<16, 0>(acc, v, a, b, iterations);
    else if (role == 1) probe_body<0, 64>(acc, v, a, b, iterations);
    else probe_body<16, 64>(acc, v, a, b, iterations);
    float r = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i) r += (acc[i][0] + acc[i][1]) + (acc[i][2] + acc[i][3]);
#pragma unroll
    for (int i = 0; i < 8; ++i) r += v[i];
    probe_lds[threadIdx.x] = r;
    __syncthreads();
    out[(blockIdx.y * gridDim.x + blockIdx.x) * 256 + threadIdx.x] = probe_lds[(threadIdx.x + 64) & 255];
}

}  // namespace

hipError_t launch_probe_issue_overlap(int mode, int iterations, int per_cu, float *out, hipStream_t st)
{
    static std::once_flag once;
    static hipError_t attr = hipSuccess;
    std::call_once(once, [] {
        attr = hipFuncSetAttribute(reinterpret_cast<const void *>(probe_issue_overlap_kernel),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, kProbeLds);
    });
    if (attr != hipSuccess) return attr;
    probe_issue_overlap_kernel<<<dim3(256, per_cu), 256, kProbeLds, st>>>(out, mode, iterations);
    return hipGetLastError();
}

}  // namespace esrnn
