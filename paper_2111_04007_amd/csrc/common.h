// Shared device/host helpers for the gfx950 stage kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace varuna {

typedef __bf16 bf16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kWave = 64;

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16 v) { return (float)v; }

template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float v) { return (bf16)v; }  // RNE

// Butterfly reductions over the 64 lanes of a wavefront.
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}

// GeLU, tanh form, and its derivative, evaluated in fp32.
__device__ __forceinline__ float gelu_tanh_f(float u) {
  const float c = 0.7978845608028654f, a = 0.044715f;
  float t = tanhf(c * (u + a * u * u * u));
  return 0.5f * u * (1.0f + t);
}
__device__ __forceinline__ float gelu_tanh_grad_f(float u) {
  const float c = 0.7978845608028654f, a = 0.044715f;
  float t = tanhf(c * (u + a * u * u * u));
  float dinner = c * (1.0f + 3.0f * a * u * u);
  return 0.5f * (1.0f + t) + 0.5f * u * (1.0f - t * t) * dinner;
}
// The same two functions for the bf16 GEMM epilogues, written on the logistic form
// 0.5 (1 + tanh z) = 1 / (1 + e^{-2z}) with the hardware exp2 and reciprocal (relative error
// about 1e-6, far below the bf16 rounding of the result; no cancellation for large |u|: the
// exponential overflows to +inf or underflows to 0 and the reciprocal gives 0 or 1).
__device__ __forceinline__ float gelu_logistic_f(float u) {
  const float k1 = -2.3022081983f, k3 = -0.10294324f;   // -2 c log2(e) and that times a
  return u * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(u * (k1 + k3 * u * u)));
}
__device__ __forceinline__ float gelu_logistic_grad_f(float u) {
  const float k1 = -2.3022081983f, k3 = -0.10294324f, c = 0.7978845608028654f, a = 0.044715f;
  const float s = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(u * (k1 + k3 * u * u)));
  return s + u * s * (1.0f - s) * (2.0f * c * (1.0f + 3.0f * a * u * u));
}

// ---- dropout masks --------------------------------------------------------------------
// Masks are a pure function of (seed, micro-batch, layer, site, element), so the recompute
// pass regenerates exactly the masks of the forward pass it repeats (the paper's
// implementation saves and restores the generator state for that; Implementation, list of
// library functions).  Generator: Philox4x32-10 (Salmon et al., SC'11).
//   key = (seed low, seed high); counter = (row / 4, column / 4, site + 256 * layer, mb):
//   one call covers a 4 x 4 patch of a site's matrix; the element's byte is byte (column % 4),
//   little end first, of output word (row % 4); an element is kept iff byte >= thr
//   (thr = round(256 p)) and kept values are multiplied by scale = 256 / (256 - thr).
// Sites: 0 attention probabilities (row = (batch * heads + head) * s + query, column = key),
// 1 attention-output projection before the residual add, 2 MLP output before the residual
// add (row = token, column = hidden index).
struct DropArgs {
  uint32_t thr;         // 0: no dropout at this site
  float scale;
  uint32_t key0, key1;
  uint32_t tag;         // site + 256 * layer
  uint32_t mb;
};
enum : uint32_t { DROP_SITE_ATTN = 0, DROP_SITE_PROJ = 1, DROP_SITE_MLP = 2 };

__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                              uint32_t k1, uint32_t out[4]) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    c0 = hi1 ^ c1 ^ k0; c1 = lo1; c2 = hi0 ^ c3 ^ k1; c3 = lo0;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}
// The four words of the patch (row_patch, col_patch): word i holds the bytes of row 4*row_patch + i.
__device__ __forceinline__ void drop_patch(const DropArgs& d, uint32_t row_patch, uint32_t col_patch, uint32_t w[4]) {
  philox4x32_10(row_patch, col_patch, d.tag, d.mb, d.key0, d.key1, w);
}
// The word of one row: bytes of columns 4*col_patch .. +3.
__device__ __forceinline__ uint32_t drop_row_word(const DropArgs& d, uint32_t row, uint32_t col_patch) {
  uint32_t w[4];
  drop_patch(d, row >> 2, col_patch, w);
  const uint32_t i = row & 3;
  return i == 0 ? w[0] : (i == 1 ? w[1] : (i == 2 ? w[2] : w[3]));
}
__device__ __forceinline__ bool drop_keep(const DropArgs& d, uint32_t word, int byte) {
  return ((word >> (8 * byte)) & 0xffu) >= d.thr;
}

// Epilogue selectors shared by every GEMM kernel.
enum EpiMode : int {
  EPI_BIAS = 0,       // out = acc + bias[n]
  EPI_BIAS_GELU = 1,  // u = acc + bias[n]; aux_out = u (optional); out = GeLU(u)
  EPI_BIAS_RES = 2,   // out = acc + bias[n] + aux_in[m,n]
  EPI_DGELU = 3,      // out = acc * GeLU'(aux_in[m,n])
  EPI_PLAIN = 4,      // out = acc
  EPI_ACCUM_F32 = 5,  // out_f32[m,n] += acc
  EPI_STORE_F32 = 6   // out_f32[split][m,n] = acc over this split's share of the reduction (split-K partial sums)
};

template <typename T>
struct EpiArgs {
  const T* bias;     // [N] or null
  const T* aux_in;   // [M,N] residual or pre-GeLU u
  T* out;            // [M,N]
  T* aux_out;        // [M,N] pre-GeLU u, may be null
  float* out_f32;    // [M,N] accumulator for EPI_ACCUM_F32
  int64_t ldc;       // row pitch of out / aux_in / aux_out / out_f32 in elements
  DropArgs drop;     // EPI_BIAS_RES only: out = aux_in + dropout(acc + bias)
  int64_t split_stride;  // EPI_STORE_F32: elements between the partial results of consecutive splits
};

// One output element.
template <typename T, int MODE>
__device__ __forceinline__ void epilogue_store(const EpiArgs<T>& e, int64_t m, int64_t n, float acc) {
  const int64_t idx = m * e.ldc + n;
  if (MODE == EPI_BIAS) {
    e.out[idx] = from_f32<T>(acc + to_f32(e.bias[n]));
  } else if (MODE == EPI_BIAS_GELU) {
    float u = acc + to_f32(e.bias[n]);
    if (e.aux_out) e.aux_out[idx] = from_f32<T>(u);
    e.out[idx] = from_f32<T>(gelu_tanh_f(u));
  } else if (MODE == EPI_BIAS_RES) {
    float v = acc + to_f32(e.bias[n]);
    if (e.drop.thr != 0)
      v = drop_keep(e.drop, drop_row_word(e.drop, (uint32_t)m, (uint32_t)(n >> 2)), (int)(n & 3)) ? v * e.drop.scale : 0.f;
    e.out[idx] = from_f32<T>(v + to_f32(e.aux_in[idx]));
  } else if (MODE == EPI_DGELU) {
    e.out[idx] = from_f32<T>(acc * gelu_tanh_grad_f(to_f32(e.aux_in[idx])));
  } else if (MODE == EPI_PLAIN) {
    e.out[idx] = from_f32<T>(acc);
  } else {
    e.out_f32[idx] += acc;
  }
}

}  // namespace varuna
