// Matrix-core helpers for the bf16 kernels (gfx950, 64-wide wavefronts).
//
// Both MFMA kernels compute their GEMM chains TRANSPOSED: D^T[out, row] = W^T[out, in] * X^T[in, row],
// i.e. the weight fragment is the first (A) operand and the activation fragment the second (B).
// With v_mfma_f32_32x32x16_bf16 the operands of lane l (i = l % 32, g = l / 32) are
//   A: 8 bf16 = A[i][kslot(g, 0..7)]        B: 8 bf16 = B[kslot(g, 0..7)][j = i]
//   D: 16 f32, register r = D[8*(r/4) + 4*g + r%4][j = i]
// so a lane owns ONE activation row (column j of D) and 16 of the 32 output features of a tile.
// That is exactly the B-operand shape of the next GEMM of the chain (one row per lane, 8
// contraction slots per K-step), so GEMM1's accumulators, after the activation, feed GEMM2
// from registers with no LDS round trip or cross-lane traffic: registers 8s..8s+7 of a 32-feature
// tile form K-step s (s = 0, 1), slot m of lane group g being feature
//   feat(s, g, m) = 16*s + 8*(m/4) + 4*g + m%4.
// The contraction order is free, so the weights of GEMM2 are simply packed in that slot order.
#pragma once
#include "common.h"
#include "gelu_poly.h"

namespace slicemoe {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f32x16 mfma_bf16(bf16x8 a, bf16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// feature index inside a 32-wide tile held by accumulator register r of lane group g
__host__ __device__ __forceinline__ int acc_feature(int r, int g) { return 8 * (r >> 2) + 4 * g + (r & 3); }
// feature index inside a 32-wide tile that sits in contraction slot m of K-step s for lane group g
__host__ __device__ __forceinline__ int chain_feature(int s, int g, int m) { return 16 * s + 8 * (m >> 2) + 4 * g + (m & 3); }

// A slice of DS bf16 values (DS a multiple of 8: whole 16-byte pieces) as matrix-core operand: K-steps of 16 for the
// GEMM that contracts over it, output tiles of 32 for the GEMM that produces it.  Widths that are not multiples of
// 16 / 32 (24, 48) are padded with zeros: in the packed weights, and here for the activation operand.
template <int DS> struct SliceTiles {
    static_assert(DS % 8 == 0, "slice rows are whole 16-byte pieces");
    static constexpr int KS = (DS + 15) / 16;
    static constexpr int OT = (DS + 31) / 32;
    static constexpr int P = DS / 8;   // 16-byte pieces per row
};

// Piece 2*ks + g of a slice row (the B operand of K-step ks for lane group g); zeros past the end of the row, and
// then the address read stays inside the row.
template <int DS>
__device__ __forceinline__ bf16x8 load_row_piece(const uint4 *__restrict__ row, int ks, int g)
{
    constexpr int P = SliceTiles<DS>::P;
    if (2 * ks + 1 < P) return __builtin_bit_cast(bf16x8, row[2 * ks + g]);
    const int piece = 2 * ks + g;
    uint4 v = row[piece < P ? piece : 0];
    if (piece >= P) v = make_uint4(0, 0, 0, 0);
    return __builtin_bit_cast(bf16x8, v);
}

}  // namespace slicemoe
