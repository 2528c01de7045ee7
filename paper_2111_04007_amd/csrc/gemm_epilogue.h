// Pieces shared by the bf16 MFMA GEMM kernels and their host-side dispatch: the fused
// epilogue applied to eight consecutive columns of one output row, the three products of a
// linear layer, and the tile descriptor.
#pragma once
#include "common.h"

namespace varuna {

//   forward  Y  = X W^T   : A = X  (k-major), B = W  (k-major)
//   dgrad    dX = dY W    : A = dY (k-major), B = W  (n-major)
//   wgrad    dW += dY^T X : A = dY (m-major), B = X  (n-major)
enum GemmOp : int { GEMM_FWD = 0, GEMM_DGRAD = 1, GEMM_WGRAD = 2 };

struct GemmTile { int bm, bn; };

// Eight consecutive columns of one output row.
template <int MODE>
__device__ __forceinline__ void gemm_epilogue8(const EpiArgs<bf16>& e, int64_t m, int64_t n, const float* acc) {
  const int64_t idx = m * e.ldc + n;
  float o[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) o[i] = acc[i];
  if (MODE == EPI_BIAS || MODE == EPI_BIAS_GELU || MODE == EPI_BIAS_RES) {
    const bf16x8 bv = *reinterpret_cast<const bf16x8*>(e.bias + n);
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] += (float)bv[i];
  }
  if (MODE == EPI_BIAS_GELU) {
    if (e.aux_out) {
      bf16x8 uv;
#pragma unroll
      for (int i = 0; i < 8; ++i) uv[i] = (bf16)o[i];
      *reinterpret_cast<bf16x8*>(e.aux_out + idx) = uv;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = gelu_logistic_f(o[i]);
  }
  if (MODE == EPI_BIAS_RES) {
    if (e.drop.thr != 0) {  // n is a multiple of 8: two patches of this row
      const uint32_t w0 = drop_row_word(e.drop, (uint32_t)m, (uint32_t)(n >> 2));
      const uint32_t w1 = drop_row_word(e.drop, (uint32_t)m, (uint32_t)(n >> 2) + 1);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        o[i] = drop_keep(e.drop, w0, i) ? o[i] * e.drop.scale : 0.f;
        o[4 + i] = drop_keep(e.drop, w1, i) ? o[4 + i] * e.drop.scale : 0.f;
      }
    }
    const bf16x8 rv = *reinterpret_cast<const bf16x8*>(e.aux_in + idx);
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] += (float)rv[i];
  }
  if (MODE == EPI_DGELU) {
    const bf16x8 uv = *reinterpret_cast<const bf16x8*>(e.aux_in + idx);
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] *= gelu_logistic_grad_f((float)uv[i]);
  }
  bf16x8 ov;
#pragma unroll
  for (int i = 0; i < 8; ++i) ov[i] = (bf16)o[i];
  *reinterpret_cast<bf16x8*>(e.out + idx) = ov;
}

}  // namespace varuna
