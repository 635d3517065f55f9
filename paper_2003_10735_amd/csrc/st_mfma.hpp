// Vector types of the gfx950 matrix-core builtins.
#pragma once
#include "st_common.hpp"

namespace st {
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// v_mfma_f32_32x32x16_bf16: D[32x32] += A[32x16] * B[16x32].  Lane l supplies A[l % 32][8*(l/32) .. +7]
// and B[8*(l/32) .. +7][l % 32]; it receives D[8*(r/4) + 4*(l/32) + r%4][l % 32] in register r.

// Channel-major operand copies ("XT") feed the weight-gradient kernels, whose MFMA fragments are
// 32 channels x 8 consecutive positions.  They are stored blocked so that such a fragment is one
// contiguous 512-byte run and a wavefront's fragment load is fully coalesced:
//     [channel / 32][column / 8][channel % 32][column % 8],   column = guard + padded position,
// with NG = PPT / 8 column groups per channel block.
__host__ __device__ __forceinline__ size_t xt_index(int c, int col, int NG)
{
    return (((size_t)(c >> 5) * NG + (col >> 3)) << 8) + ((c & 31) << 3) + (col & 7);
}

// Weights of the 3x3 matrix-core convolutions, [rows][9 taps][K], are kept in the order in which
// that kernel's wavefronts consume them: one A fragment (32 rows x 16 k of one tap, lane l holding
// row l % 32, k 8*(l/32) .. +7) is one contiguous 1 KB run,
//     [row / 32][tap][k / 16][(k / 8) % 2][row % 32][k % 8].
__host__ __device__ __forceinline__ size_t wfrag_index(int row, int tap, int k, int K)
{
    return ((((size_t)(row >> 5) * 9 + tap) * (K >> 4) + (k >> 4)) * 64 + ((k >> 3) & 1) * 32 + (row & 31)) * 8 + (k & 7);
}
}  // namespace st
