// Softmax attention forward/backward in plain fp32 arithmetic, one wavefront
// per query row (forward, dQ) or per key row (dK, dV).  Exact two-pass softmax,
// no atomics, any head dim / sequence length up to ATS_MAX_S.  This is the fp32
// path and the fall-back for bf16 shapes the MFMA attention does not cover.
//
// qkv is [b*s, 3h]: Q at column j*d, K at h + j*d, V at 2h + j*d for head j.
#pragma once
#include "common.h"

namespace varuna {

constexpr int ATS_MAX_S = 4096;
constexpr int ATS_MAX_D = 256;

// ctx_i = sum_k P_ik V_k with P = softmax over k of scale * q_i.k_k (k <= i if causal).
// lse[b, j, i] = max + log(sum) (natural log), written when lse != null.
template <typename T>
__global__ void attention_fwd_simple_kernel(const T* __restrict__ qkv, T* __restrict__ ctx,
                                            float* __restrict__ lse, int s, int heads, int d,
                                            int causal, float scale, DropArgs drop) {
  extern __shared__ float smem[];
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const int nw = blockDim.x / kWave;
  const int i = blockIdx.x * nw + wave;
  const int j = blockIdx.y, bi = blockIdx.z;
  if (i >= s) return;
  const int h = heads * d;
  const int64_t ld = 3 * (int64_t)h;
  float* q = smem + (size_t)wave * (d + s);
  float* p = q + d;
  const T* base = qkv + (int64_t)bi * s * ld;
  const T* qrow = base + (int64_t)i * ld + j * d;
  for (int e = lane; e < d; e += kWave) q[e] = to_f32(qrow[e]);
  __builtin_amdgcn_wave_barrier();
  const int nk = causal ? i + 1 : s;
  float mx = -INFINITY;
  for (int k = lane; k < nk; k += kWave) {
    const T* krow = base + (int64_t)k * ld + h + j * d;
    float dot = 0.f;
    for (int e = 0; e < d; ++e) dot = fmaf(q[e], to_f32(krow[e]), dot);
    dot *= scale;
    p[k] = dot;
    mx = fmaxf(mx, dot);
  }
  mx = wave_max(mx);
  float sum = 0.f;
  const uint32_t drow = (uint32_t)(((int64_t)bi * heads + j) * s + i);  // row of the dropout mask
  for (int k = lane; k < nk; k += kWave) {
    float e = expf(p[k] - mx);
    sum += e;   // the softmax is normalised before the dropout
    if (drop.thr != 0 && !drop_keep(drop, drop_row_word(drop, drow, (uint32_t)k >> 2), k & 3)) e = 0.f;
    p[k] = e;
  }
  sum = wave_sum(sum);
  const float inv = (drop.thr != 0 ? drop.scale : 1.0f) / sum;
  if (lse && lane == 0) lse[((int64_t)bi * heads + j) * s + i] = mx + logf(sum);
  __builtin_amdgcn_wave_barrier();
  T* crow = ctx + ((int64_t)bi * s + i) * h + j * d;
  for (int e = lane; e < d; e += kWave) {
    float acc = 0.f;
    const T* vcol = base + 2 * h + j * d + e;
    for (int k = 0; k < nk; ++k) acc = fmaf(p[k], to_f32(vcol[(int64_t)k * ld]), acc);
    crow[e] = from_f32<T>(acc * inv);
  }
}

// Per query row i: delta_i = sum_e dctx_ie ctx_ie; dS_ik = P_ik (dctx_i.V_k - delta_i);
// dQ_i = scale * sum_k dS_ik K_k.  Writes delta for the key-side kernel.
template <typename T>
__global__ void attention_bwd_dq_simple_kernel(const T* __restrict__ qkv, const T* __restrict__ ctx,
                                               const float* __restrict__ lse,
                                               const T* __restrict__ dctx, T* __restrict__ dqkv,
                                               float* __restrict__ delta, int s, int heads, int d,
                                               int causal, float scale, DropArgs drop) {
  extern __shared__ float smem[];
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const int nw = blockDim.x / kWave;
  const int i = blockIdx.x * nw + wave;
  const int j = blockIdx.y, bi = blockIdx.z;
  if (i >= s) return;
  const int h = heads * d;
  const int64_t ld = 3 * (int64_t)h;
  float* q = smem + (size_t)wave * (2 * d + s);
  float* go = q + d;
  float* ds = go + d;
  const T* base = qkv + (int64_t)bi * s * ld;
  const int64_t orow = ((int64_t)bi * s + i) * h + j * d;
  float dl = 0.f;
  for (int e = lane; e < d; e += kWave) {
    q[e] = to_f32(base[(int64_t)i * ld + j * d + e]);
    float g = to_f32(dctx[orow + e]);
    go[e] = g;
    dl += g * to_f32(ctx[orow + e]);
  }
  dl = wave_sum(dl);
  const int64_t sidx = ((int64_t)bi * heads + j) * s + i;
  if (lane == 0) delta[sidx] = dl;
  const float l = lse[sidx];
  __builtin_amdgcn_wave_barrier();
  const int nk = causal ? i + 1 : s;
  for (int k = lane; k < nk; k += kWave) {
    const T* krow = base + (int64_t)k * ld + h + j * d;
    const T* vrow = krow + h;
    float dot = 0.f, dp = 0.f;
    for (int e = 0; e < d; ++e) {
      dot = fmaf(q[e], to_f32(krow[e]), dot);
      dp = fmaf(go[e], to_f32(vrow[e]), dp);
    }
    float pr = expf(dot * scale - l);
    if (drop.thr != 0)
      dp = drop_keep(drop, drop_row_word(drop, (uint32_t)sidx, (uint32_t)k >> 2), k & 3) ? dp * drop.scale : 0.f;
    ds[k] = pr * (dp - dl);
  }
  __builtin_amdgcn_wave_barrier();
  T* dq = dqkv + ((int64_t)bi * s + i) * ld + j * d;
  for (int e = lane; e < d; e += kWave) {
    float acc = 0.f;
    const T* kcol = base + h + j * d + e;
    for (int k = 0; k < nk; ++k) acc = fmaf(ds[k], to_f32(kcol[(int64_t)k * ld]), acc);
    dq[e] = from_f32<T>(acc * scale);
  }
}

// Per key row k: dV_k = sum_i P_ik dctx_i; dK_k = scale * sum_i dS_ik Q_i (i >= k if causal).
template <typename T>
__global__ void attention_bwd_dkv_simple_kernel(const T* __restrict__ qkv,
                                                const float* __restrict__ lse,
                                                const T* __restrict__ dctx,
                                                const float* __restrict__ delta,
                                                T* __restrict__ dqkv, int s, int heads, int d,
                                                int causal, float scale, DropArgs drop) {
  extern __shared__ float smem[];
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const int nw = blockDim.x / kWave;
  const int k = blockIdx.x * nw + wave;
  const int j = blockIdx.y, bi = blockIdx.z;
  if (k >= s) return;
  const int h = heads * d;
  const int64_t ld = 3 * (int64_t)h;
  float* kk = smem + (size_t)wave * (2 * d + 2 * s);
  float* vv = kk + d;
  float* pp = vv + d;
  float* ds = pp + s;
  const T* base = qkv + (int64_t)bi * s * ld;
  for (int e = lane; e < d; e += kWave) {
    kk[e] = to_f32(base[(int64_t)k * ld + h + j * d + e]);
    vv[e] = to_f32(base[(int64_t)k * ld + 2 * h + j * d + e]);
  }
  __builtin_amdgcn_wave_barrier();
  const int i0 = causal ? k : 0;
  const int64_t sbase = ((int64_t)bi * heads + j) * s;
  for (int i = i0 + lane; i < s; i += kWave) {
    const T* qrow = base + (int64_t)i * ld + j * d;
    const T* grow = dctx + ((int64_t)bi * s + i) * h + j * d;
    float dot = 0.f, dp = 0.f;
    for (int e = 0; e < d; ++e) {
      dot = fmaf(to_f32(qrow[e]), kk[e], dot);
      dp = fmaf(to_f32(grow[e]), vv[e], dp);
    }
    float pr = expf(dot * scale - lse[sbase + i]);
    float f = 1.0f;
    if (drop.thr != 0)
      f = drop_keep(drop, drop_row_word(drop, (uint32_t)(sbase + i), (uint32_t)k >> 2), k & 3) ? drop.scale : 0.f;
    pp[i] = pr * f;
    ds[i] = pr * (dp * f - delta[sbase + i]);
  }
  __builtin_amdgcn_wave_barrier();
  T* dk = dqkv + ((int64_t)bi * s + k) * ld + h + j * d;
  T* dv = dk + h;
  for (int e = lane; e < d; e += kWave) {
    float ak = 0.f, av = 0.f;
    const T* qcol = base + j * d + e;
    const T* gcol = dctx + (int64_t)bi * s * h + j * d + e;
    for (int i = i0; i < s; ++i) {
      ak = fmaf(ds[i], to_f32(qcol[(int64_t)i * ld]), ak);
      av = fmaf(pp[i], to_f32(gcol[(int64_t)i * h]), av);
    }
    dk[e] = from_f32<T>(ak * scale);
    dv[e] = from_f32<T>(av);
  }
}

// Waves per block such that the per-wave LDS rows fit the default 64 KB limit.
inline int ats_waves(size_t bytes_per_wave) {
  int nw = 4;
  while (nw > 0 && nw * bytes_per_wave > 60 * 1024) nw /= 2;
  return nw;
}

template <typename T>
inline hipError_t launch_attention_fwd_simple(const T* qkv, T* ctx, float* lse, int b, int s,
                                              int heads, int d, int causal, const DropArgs& drop, hipStream_t st) {
  const int nw = ats_waves((size_t)(d + s) * sizeof(float));
  if (nw == 0) return hipErrorInvalidValue;
  const size_t sm = (size_t)nw * (d + s) * sizeof(float);
  dim3 grid((unsigned)((s + nw - 1) / nw), (unsigned)heads, (unsigned)b);
  hipLaunchKernelGGL((attention_fwd_simple_kernel<T>), grid, dim3(nw * kWave), sm, st, qkv, ctx, lse,
                     s, heads, d, causal, 1.0f / sqrtf((float)d), drop);
  return hipGetLastError();
}

template <typename T>
inline hipError_t launch_attention_bwd_simple(const T* qkv, const T* ctx, const float* lse,
                                              const T* dctx, T* dqkv, float* delta, int b, int s,
                                              int heads, int d, int causal, const DropArgs& drop, hipStream_t st) {
  const float scale = 1.0f / sqrtf((float)d);
  {
    const int nw = ats_waves((size_t)(2 * d + s) * sizeof(float));
    if (nw == 0) return hipErrorInvalidValue;
    const size_t sm = (size_t)nw * (2 * d + s) * sizeof(float);
    dim3 grid((unsigned)((s + nw - 1) / nw), (unsigned)heads, (unsigned)b);
    hipLaunchKernelGGL((attention_bwd_dq_simple_kernel<T>), grid, dim3(nw * kWave), sm, st, qkv, ctx,
                       lse, dctx, dqkv, delta, s, heads, d, causal, scale, drop);
  }
  {
    const int nw = ats_waves((size_t)(2 * d + 2 * s) * sizeof(float));
    if (nw == 0) return hipErrorInvalidValue;
    const size_t sm = (size_t)nw * (2 * d + 2 * s) * sizeof(float);
    dim3 grid((unsigned)((s + nw - 1) / nw), (unsigned)heads, (unsigned)b);
    hipLaunchKernelGGL((attention_bwd_dkv_simple_kernel<T>), grid, dim3(nw * kWave), sm, st, qkv, lse,
                       dctx, delta, dqkv, s, heads, d, causal, scale, drop);
  }
  return hipGetLastError();
}

}  // namespace varuna
