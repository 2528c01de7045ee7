// Mini-batch tail of one stage: statistics of the accumulated fp32 gradients (sum of
// squares and number of non-finite entries: this GPU's share of the global gradient norm and
// of the overflow flag that the stages of a pipeline synchronise) and a mixed-precision Adam
// step (fp32 master weight, momentum and variance; parameter re-rounded to the stage's
// storage type).  Both are single passes over flat buffers, bound by HBM.
#pragma once
#include "common.h"

namespace varuna {

constexpr int kStatBlocks = 1024;  // partial results of the two-stage reduction (2 doubles each)

// partial[2*b] = sum of squares of the finite entries block b saw, partial[2*b+1] = its
// number of non-finite entries.  Fixed work split and fixed summation order: deterministic.
__global__ __launch_bounds__(256) void grad_stats_partial_kernel(const float* __restrict__ g, size_t n, double* __restrict__ partial) {
  const size_t n4 = n / 4;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
  unsigned bad = 0;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
    const floatx4 v = reinterpret_cast<const floatx4*>(g)[i];
    const bool f0 = isfinite(v[0]), f1 = isfinite(v[1]), f2 = isfinite(v[2]), f3 = isfinite(v[3]);
    s0 += f0 ? v[0] * v[0] : 0.f; s1 += f1 ? v[1] * v[1] : 0.f;
    s2 += f2 ? v[2] * v[2] : 0.f; s3 += f3 ? v[3] * v[3] : 0.f;
    bad += (unsigned)!f0 + (unsigned)!f1 + (unsigned)!f2 + (unsigned)!f3;
  }
  double s = (double)s0 + (double)s1 + (double)s2 + (double)s3;
  if (blockIdx.x == 0 && threadIdx.x == 0)
    for (size_t i = n4 * 4; i < n; ++i) {
      const float v = g[i];
      if (isfinite(v)) s += (double)v * (double)v; else ++bad;
    }
  __shared__ double ss[256];
  __shared__ unsigned sb[256];
  ss[threadIdx.x] = s;
  sb[threadIdx.x] = bad;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) { ss[threadIdx.x] += ss[threadIdx.x + w]; sb[threadIdx.x] += sb[threadIdx.x + w]; }
    __syncthreads();
  }
  if (threadIdx.x == 0) { partial[2 * blockIdx.x] = ss[0]; partial[2 * blockIdx.x + 1] = (double)sb[0]; }
}

__global__ __launch_bounds__(256) void grad_stats_final_kernel(const double* __restrict__ partial, int nblk, float* __restrict__ out2) {
  __shared__ double ss[256], sb[256];
  double s = 0.0, b = 0.0;
  for (int i = threadIdx.x; i < nblk; i += 256) { s += partial[2 * i]; b += partial[2 * i + 1]; }
  ss[threadIdx.x] = s; sb[threadIdx.x] = b;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) { ss[threadIdx.x] += ss[threadIdx.x + w]; sb[threadIdx.x] += sb[threadIdx.x + w]; }
    __syncthreads();
  }
  if (threadIdx.x == 0) { out2[0] = (float)ss[0]; out2[1] = (float)sb[0]; }
}

inline hipError_t launch_grad_stats(const float* g, size_t n, double* partial, float* out2, hipStream_t st) {
  size_t want = (n / 4 + 255) / 256;
  const int nblk = (int)(want < 1 ? 1 : (want > (size_t)kStatBlocks ? (size_t)kStatBlocks : want));
  hipLaunchKernelGGL(grad_stats_partial_kernel, dim3(nblk), dim3(256), 0, st, g, n, partial);
  hipLaunchKernelGGL(grad_stats_final_kernel, dim3(1), dim3(256), 0, st, partial, nblk, out2);
  return hipGetLastError();
}

struct AdamArgs {
  float lr, beta1, beta2, eps, weight_decay, grad_scale;
  float inv_bias1, inv_bias2;  // 1 / (1 - beta^step)
};

// Adam as published (Kingma & Ba, Algorithm 1) with decoupled weight decay, on the scaled
// gradient; the whole update is skipped when *skip is non-zero (an overflow anywhere in the
// pipeline cancels the step on every stage).  T: storage type of the stage's parameters.
template <typename T>
__device__ __forceinline__ void adam_one(float gi, float& wi, float& mi, float& vi, T& pi, const AdamArgs& a) {
  const float gs = a.grad_scale * gi;
  mi = a.beta1 * mi + (1.f - a.beta1) * gs;
  vi = a.beta2 * vi + (1.f - a.beta2) * gs * gs;
  const float upd = (mi * a.inv_bias1) / (sqrtf(vi * a.inv_bias2) + a.eps) + a.weight_decay * wi;
  wi = wi - a.lr * upd;
  pi = from_f32<T>(wi);
}

template <typename T>
__global__ __launch_bounds__(256) void adam_kernel(const float* __restrict__ g, float* __restrict__ w, float* __restrict__ m,
                                                   float* __restrict__ v, T* __restrict__ p, size_t n, AdamArgs a,
                                                   const float* __restrict__ skip) {
  if (skip != nullptr && *skip != 0.f) return;
  typedef T Tx4 __attribute__((ext_vector_type(4)));
  const size_t n4 = n / 4;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
    const floatx4 g4 = reinterpret_cast<const floatx4*>(g)[i];
    floatx4 w4 = reinterpret_cast<floatx4*>(w)[i], m4 = reinterpret_cast<floatx4*>(m)[i], v4 = reinterpret_cast<floatx4*>(v)[i];
    Tx4 p4;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float wi = w4[e], mi = m4[e], vi = v4[e];
      T pi;
      adam_one<T>(g4[e], wi, mi, vi, pi, a);
      w4[e] = wi; m4[e] = mi; v4[e] = vi; p4[e] = pi;
    }
    reinterpret_cast<floatx4*>(w)[i] = w4;
    reinterpret_cast<floatx4*>(m)[i] = m4;
    reinterpret_cast<floatx4*>(v)[i] = v4;
    reinterpret_cast<Tx4*>(p)[i] = p4;
  }
  if (blockIdx.x == 0 && threadIdx.x < n - n4 * 4) {
    const size_t i = n4 * 4 + threadIdx.x;
    adam_one<T>(g[i], w[i], m[i], v[i], p[i], a);
  }
}

template <typename T>
inline hipError_t launch_adam(const float* g, float* w, float* m, float* v, T* p, size_t n, const AdamArgs& a,
                              const float* skip, hipStream_t st) {
  size_t want = (n / 4 + 255) / 256;
  const unsigned nblk = (unsigned)(want > 8192 ? 8192 : (want < 1 ? 1 : want));
  hipLaunchKernelGGL((adam_kernel<T>), dim3(nblk), dim3(256), 0, st, g, w, m, v, p, n, a, skip);
  return hipGetLastError();
}

}  // namespace varuna
