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

// Epilogue selectors shared by every GEMM kernel.
enum EpiMode : int {
  EPI_BIAS = 0,       // out = acc + bias[n]
  EPI_BIAS_GELU = 1,  // u = acc + bias[n]; aux_out = u (optional); out = GeLU(u)
  EPI_BIAS_RES = 2,   // out = acc + bias[n] + aux_in[m,n]
  EPI_DGELU = 3,      // out = acc * GeLU'(aux_in[m,n])
  EPI_PLAIN = 4,      // out = acc
  EPI_ACCUM_F32 = 5   // out_f32[m,n] += acc
};

template <typename T>
struct EpiArgs {
  const T* bias;     // [N] or null
  const T* aux_in;   // [M,N] residual or pre-GeLU u
  T* out;            // [M,N]
  T* aux_out;        // [M,N] pre-GeLU u, may be null
  float* out_f32;    // [M,N] accumulator for EPI_ACCUM_F32
  int64_t ldc;       // row pitch of out / aux_in / aux_out / out_f32 in elements
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
    e.out[idx] = from_f32<T>(acc + to_f32(e.bias[n]) + to_f32(e.aux_in[idx]));
  } else if (MODE == EPI_DGELU) {
    e.out[idx] = from_f32<T>(acc * gelu_tanh_grad_f(to_f32(e.aux_in[idx])));
  } else if (MODE == EPI_PLAIN) {
    e.out[idx] = from_f32<T>(acc);
  } else {
    e.out_f32[idx] += acc;
  }
}

}  // namespace varuna
