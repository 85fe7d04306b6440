// Device helpers shared by the kernels: the 16x16x4 fp32 MFMA tile, LDS-only
// barrier, activation functions, wave reductions.
#pragma once

#include <hip/hip_runtime.h>

#include <type_traits>

namespace esrnn {

typedef float f32x4 __attribute__((ext_vector_type(4)));

// compile-time loop: f(std::integral_constant<int, I>) for I = 0 .. N-1 (for indices that must be immediates:
// MFMA broadcast blocks, register sets that rotate through a loop)
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// D = A(16x4) * B(4x16) + C(16x16), fp32.  Lane l supplies A[l%16][l/16] and
// B[l/16][l%16]; it holds D[4*(l/16) + r][l%16] in component r.
__device__ __forceinline__ f32x4 mfma16(float a, float b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// Buffer addressing for the wave-uniform tiles of the LSTM kernels: the tile's base is a scalar resource (built
// with scalar instructions from a pointer that is the same in every lane), the tile's offset inside it a scalar
// byte offset, the lane's share a 32-bit byte offset that never changes.  No address arithmetic is left on the
// vector ALU, whose cycles the fp32 MFMAs need.  A resource spans 4 GiB from its base (raw buffer, no stride, no
// range limit): callers rebase it per window position and keep the offsets inside one position.
typedef __amdgpu_buffer_rsrc_t buf_rsrc;
__device__ __forceinline__ buf_rsrc make_rsrc(const void *base)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, -1, 0x00020000);
}
__device__ __forceinline__ float buf_load(buf_rsrc r, unsigned lane_bytes, unsigned tile_bytes)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, lane_bytes, tile_bytes, 0));
}
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ f32x4 buf_load4(buf_rsrc r, unsigned lane_bytes, unsigned tile_bytes)
{
    return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, lane_bytes, tile_bytes, 0));
}
// kStream: the value is not read again soon (streaming store)
template <bool kStream = false>
__device__ __forceinline__ void buf_store(buf_rsrc r, unsigned lane_bytes, unsigned tile_bytes, float v)
{
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), r, lane_bytes, tile_bytes, kStream ? 2 : 0);
}
template <bool kStream = false>
__device__ __forceinline__ void buf_store4(buf_rsrc r, unsigned lane_bytes, unsigned tile_bytes, f32x4 v)
{
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), r, lane_bytes, tile_bytes, kStream ? 2 : 0);
}

// Workgroup barrier that orders LDS traffic only: global loads and stores in
// flight are not waited for.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__device__ __forceinline__ float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }

// Natural logarithm of a normal positive number (series values, levels and seasonal factors are far from
// the denormal range): the hardware log2 without the rescaling path for denormals.
__device__ __forceinline__ float fast_log(float x) { return __builtin_amdgcn_logf(x) * 0.69314718055994531f; }

__device__ __forceinline__ float sigmoid_f(float x)
{
    return fast_rcp(1.0f + __expf(-x));
}

// tanh(x) = 1 - 2 / (1 + exp(2x)); saturates correctly at both ends.  exp(2x) = 2^(x * 2 log2(e)): one
// multiplication, with the same result as doubling x first (doubling is exact).
__device__ __forceinline__ float tanh_f(float x)
{
    return 1.0f - 2.0f * fast_rcp(1.0f + __builtin_amdgcn_exp2f(x * 2.8853900817779268f));
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// maximum over the ACTIVE lanes of the wave, the same value in every lane (wave-uniform)
__device__ __forceinline__ int wave_max_int(int v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = max(v, __shfl_xor(v, off, 64));
    return __builtin_amdgcn_readfirstlane(v);
}

// sum over the 16 lanes that share lane/16
__device__ __forceinline__ float group16_sum(float v)
{
#pragma unroll
    for (int off = 8; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

}  // namespace esrnn
