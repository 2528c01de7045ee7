// Measurement hook: the rate the matrix cores sustain on v_mfma_f32_32x32x16_bf16 when fed
// from registers only (no LDS, no memory traffic in the loop).  It is the ceiling any GEMM
// on this chip sits under for a given kind of operand data: the clock the chip holds depends
// on how many operand bits toggle, so all-zero operands and normally distributed operands
// give different rates.  Not on the stage's path.
#pragma once
#include "common.h"

namespace varuna {

// Every wave loads 4 + 4 operand fragments (8 bf16 per lane each) from `src` (n_vec 16-byte
// vectors, indices wrap) once, then issues iters x 8 independent products into 8 accumulator
// tiles and writes the sum of its accumulators so that the work cannot be dropped.
// PATTERN selects which fragments consecutive products read (the data is the same in all):
//   0: both operands change from one product to the next;
//   1: the first operand is held for 8 consecutive products, the second changes every time;
//   2: the first is held for 8, the second for 2 (the order a 4x2 register tile walked row by row gives);
//   3: both operands are the same fragments for every product;
//   4: as 0, but 4 consecutive products add to the same accumulator tile (a dependent chain, as
//      when the products of 4 k-steps of one output block are issued back to back);
//   5: as 4 with chains of 2;
//   6: as 0 with v_mfma_f32_16x16x32_bf16, two of them per product slot (the same operations per
//      slot; half the accumulator traffic and twice the operand traffic per operation);
//   7: as 2 with that instruction.
template <int PATTERN>
__global__ __launch_bounds__(256) void mfma_rate_kernel(const bf16x8* __restrict__ src, uint32_t n_vec,
                                                        float* __restrict__ sink, int iters) {
  bf16x8 a[4], b[4];
  const uint32_t gid = blockIdx.x * blockDim.x + threadIdx.x;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a[i] = src[(gid * 8u + i) % n_vec];
    b[i] = src[(gid * 8u + 4u + i) % n_vec];
  }
  if constexpr (PATTERN >= 6) {
    floatx4 acc4[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc4[i] = floatx4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; it += 4) {
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int ia = PATTERN == 6 ? (i & 3) : u;
          const int ib = PATTERN == 6 ? ((i + u) & 3) : ((i >> 1) & 3);
          acc4[2 * i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[ia], b[ib], acc4[2 * i], 0, 0, 0);
          acc4[2 * i + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[ia], b[(ib + 1) & 3], acc4[2 * i + 1], 0, 0, 0);
        }
    }
    float s4 = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s4 += acc4[i][0] + acc4[i][1] + acc4[i][2] + acc4[i][3];
    sink[gid] = s4;
    return;
  }
  floatx16 acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  for (int it = 0; it < iters; it += 4) {
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        if (PATTERN >= 4) {   // product number n = 8u + i of 32: accumulator changes every CH products
          constexpr int CH = PATTERN == 4 ? 4 : 2;
          const int n = 8 * u + i, t = (n / CH) & 7;
          acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[n & 3], b[(n + (n >> 2)) & 3], acc[t], 0, 0, 0);
        } else {
          const int ia = PATTERN == 0 ? (i & 3) : (PATTERN == 3 ? 0 : u);
          const int ib = PATTERN == 0 ? ((i + u) & 3) : (PATTERN == 1 ? (i & 3) : (PATTERN == 2 ? ((i >> 1) & 3) : 0));
          acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ia], b[ib], acc[i], 0, 0, 0);
        }
      }
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  sink[gid] = s;
}

}  // namespace varuna
