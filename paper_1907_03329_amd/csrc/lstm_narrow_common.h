// Dilated LSTM layer for small batches (Section 3.2, Table 1; Section 8.3 notes
// how little of a GPU such small cells use): forward and reverse kernels that
// give a workgroup FOUR series instead of sixteen.
//
// When series tiles x chains of a layer is far below the number of compute
// units, the 16-series kernels of lstm_kernels.hip leave most of the chip idle
// and the layer costs (positions of the longest chain) x (time of one position
// on one compute unit).  Both factors are attacked here: four times as many
// workgroups, and a position costs a quarter of the matrix work.
//
// Arithmetic.  v_mfma_f32_4x4x1_16B_f32: sixteen independent 4x4 outer products
// ("blocks") per instruction, one k-step.  Lane l belongs to block l/4; it
// supplies A[l%4] and B[l%4] of its block and holds D[0..3][l%4].  With its
// broadcast control (cbsz = 4, abid = b) all sixteen blocks take the A values
// of block b.  Here A carries the ACTIVATIONS of the four series for one input
// column, broadcast from the block whose four lanes hold them, and B carries
// the weights: block u, lane g of a wave holds gate g of hidden unit u.  One
// instruction advances 16 units x 4 gates x 4 series by one input column, and no
// operand has to be replicated over the blocks: a wave reads [x_p ; h_{p-d}] of
// the four series from LDS with one 4-byte load per 16 columns.  A workgroup has
// four waves; wave w owns the units w*HT .. w*HT+HT-1 (HT <= 16; the padded
// hidden size is 4*HT).  A lane ends up with one gate of one unit for the four
// series; a 4x4 transpose inside each quad of lanes (DPP) turns that into the
// four gates of one unit for ONE series, and the cell update is lane-local as
// in the 16-series kernels.
//
// The reverse kernel follows the 16-series one step by step (gate gradients,
// transposed contraction split over the waves along the contraction, weight
// gradient in accumulators for the whole launch) with these differences: the
// transposed contraction runs on the 4x4x1 instruction with the gate gradients
// broadcast straight from the registers of the lanes that computed them; the
// weight gradient contracts over the four series, which is exactly the k = 4 of
// ONE 16x16x4 instruction per 16x16 tile of dW; the LDS arrays a position writes
// are double-buffered by position parity, which leaves one barrier per
// position.  Every LDS array is laid out [row][4 series], so that each access
// of a wave covers consecutive addresses.
//
// Global operands.  A position takes a fraction of a microsecond here, less
// than the latency of HBM, so operands are requested a whole chunk of positions
// ahead into registers and staged in LDS: the requests for the next chunk go
// out at the start of a chunk, and at its end the registers are written to LDS.
// A whole chunk is ONE straight run of instructions (the position loop inside
// it is unrolled): memory operations complete in order, and only with request
// and use in the same run does the compiler's wait for a request count the
// stores issued since instead of waiting for all of them.  (With the request in
// one loop iteration and the use in another, every chunk waited for its newest
// stores; a ring of registers with one request per position was slower still.)
// Blocks past HT repeat the last unit of the wave, operands and addresses alike,
// and threads without an input row stage into a spare LDS column, so no memory
// operation sits behind a divergent branch.
//
// All tensors keep the layouts of the 16-series kernels (TL(R) tiles of 16
// series), so layers of both kinds mix freely and the weight-gradient
// reduction is unchanged; a workgroup touches 16-byte pieces of each row.
#pragma once

#include <type_traits>

#include "device_utils.h"
#include "esrnn_internal.h"

namespace esrnn {

namespace {

constexpr int kNW = 4;          // waves per workgroup
constexpr int kNT = 64 * kNW;   // threads per workgroup

// D_blk[i][j] += A_ABID[i] * B_blk[j] for all 16 blocks: the A values of block ABID serve every block.
template <int ABID>
__device__ __forceinline__ f32x4 mfma4_bcast(float a, float b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_4x4x1f32(a, b, c, 4, ABID, 0);
}

// value of the same register in another lane of the quad: quad_perm control [a, b, c, d]
template <int CTRL>
__device__ __forceinline__ float quad_perm(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}

// 4x4 transpose inside each quad of lanes: lane j, component c  <->  lane c, component j
__device__ __forceinline__ void quad_transpose(f32x4 &v, int j)
{
    const bool lo = j & 1, hi = j & 2;
    {   // lanes j ^ 1, component pairs (0,1) and (2,3)
        const float r01 = quad_perm<0xB1>(lo ? v[0] : v[1]);
        const float r23 = quad_perm<0xB1>(lo ? v[2] : v[3]);
        if (lo) { v[0] = r01; v[2] = r23; } else { v[1] = r01; v[3] = r23; }
    }
    {   // lanes j ^ 2, component pairs (0,2) and (1,3)
        const float r02 = quad_perm<0x4E>(hi ? v[0] : v[2]);
        const float r13 = quad_perm<0x4E>(hi ? v[1] : v[3]);
        if (hi) { v[0] = r02; v[1] = r13; } else { v[2] = r02; v[3] = r13; }
    }
}

// workgroups along x: groups of 32 = 8 tiles x 4 quarters
inline int narrow_grid_x(int NB) { return ((NB + 7) / 8) * 32; }

#define ESRNN_LSTM_SHAPES(X) \
    X(2, 1) X(2, 2) X(8, 2) X(8, 3) X(8, 8) X(10, 1) X(10, 3) X(10, 6) X(10, 8) X(10, 10) X(13, 3) X(13, 5) X(13, 13) X(16, 16)

}  // namespace

}  // namespace esrnn
