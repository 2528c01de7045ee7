// LayerNorm forward/backward (one wavefront per row, shuffle reductions) and
// deterministic two-stage column reductions for bias / gamma / beta gradients.
// All of these are HBM-bound: the arithmetic is fp32, the traffic is what counts.
#pragma once
#include <initializer_list>

#include "common.h"

namespace varuna {

constexpr int LN_ROWS_PER_BLOCK = 4;  // 4 waves, one row each
constexpr int CR_COLS = 64;           // columns per block in the column reductions
constexpr int CR_ROWLANES = 4;
constexpr int CR_CHUNK = 256;         // rows per partial

template <typename T, int VEC> struct VecLoad;
template <typename T> struct VecLoad<T, 1> {
  static __device__ __forceinline__ void load(const T* p, float* v) { v[0] = to_f32(p[0]); }
  static __device__ __forceinline__ void store(T* p, const float* v) { p[0] = from_f32<T>(v[0]); }
};
template <> struct VecLoad<float, 4> {
  static __device__ __forceinline__ void load(const float* p, float* v) {
    floatx4 t = *reinterpret_cast<const floatx4*>(p);
    v[0] = t[0]; v[1] = t[1]; v[2] = t[2]; v[3] = t[3];
  }
  static __device__ __forceinline__ void store(float* p, const float* v) {
    floatx4 t = {v[0], v[1], v[2], v[3]};
    *reinterpret_cast<floatx4*>(p) = t;
  }
};
template <> struct VecLoad<bf16, 8> {
  static __device__ __forceinline__ void load(const bf16* p, float* v) {
    bf16x8 t = *reinterpret_cast<const bf16x8*>(p);
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = (float)t[i];
  }
  static __device__ __forceinline__ void store(bf16* p, const float* v) {
    bf16x8 t;
#pragma unroll
    for (int i = 0; i < 8; ++i) t[i] = (bf16)v[i];
    *reinterpret_cast<bf16x8*>(p) = t;
  }
};

// y = gamma * (x - mean) * rstd + beta per row; biased variance, two passes
// (mean first, then centred second moment) so fp32 holds 1e-5 parity.
template <typename T, int VEC>
__global__ __launch_bounds__(LN_ROWS_PER_BLOCK* kWave) void layernorm_fwd_kernel(
    const T* __restrict__ x, const T* __restrict__ gamma, const T* __restrict__ beta,
    T* __restrict__ y, float* __restrict__ stats, int64_t rows, int h, float eps) {
  const int lane = threadIdx.x % kWave;
  const int64_t row = (int64_t)blockIdx.x * LN_ROWS_PER_BLOCK + threadIdx.x / kWave;
  if (row >= rows) return;
  const T* xr = x + row * h;
  float v[VEC], s = 0.f;
  for (int j = lane * VEC; j < h; j += kWave * VEC) {
    VecLoad<T, VEC>::load(xr + j, v);
#pragma unroll
    for (int i = 0; i < VEC; ++i) s += v[i];
  }
  const float mean = wave_sum(s) / (float)h;
  s = 0.f;
  for (int j = lane * VEC; j < h; j += kWave * VEC) {
    VecLoad<T, VEC>::load(xr + j, v);
#pragma unroll
    for (int i = 0; i < VEC; ++i) { float c = v[i] - mean; s += c * c; }
  }
  const float rstd = 1.0f / sqrtf(wave_sum(s) / (float)h + eps);
  if (stats && lane == 0) { stats[row] = mean; stats[rows + row] = rstd; }
  T* yr = y + row * h;
  float g[VEC], b[VEC];
  for (int j = lane * VEC; j < h; j += kWave * VEC) {
    VecLoad<T, VEC>::load(xr + j, v);
    VecLoad<T, VEC>::load(gamma + j, g);
    VecLoad<T, VEC>::load(beta + j, b);
#pragma unroll
    for (int i = 0; i < VEC; ++i) v[i] = g[i] * ((v[i] - mean) * rstd) + b[i];
    VecLoad<T, VEC>::store(yr + j, v);
  }
}

// dx = res + rstd * (dxhat - mean_j dxhat - xhat * mean_j(dxhat * xhat)),
// dxhat = dy * gamma, xhat = (x - mean) * rstd from the stored statistics.
template <typename T, int VEC>
__global__ __launch_bounds__(LN_ROWS_PER_BLOCK* kWave) void layernorm_bwd_dx_kernel(
    const T* __restrict__ dy, const T* __restrict__ x, const float* __restrict__ stats,
    const T* __restrict__ gamma, const T* __restrict__ res, T* __restrict__ dx, int64_t rows,
    int h) {
  const int lane = threadIdx.x % kWave;
  const int64_t row = (int64_t)blockIdx.x * LN_ROWS_PER_BLOCK + threadIdx.x / kWave;
  if (row >= rows) return;
  const float mean = stats[row], rstd = stats[rows + row];
  const T* xr = x + row * h;
  const T* dyr = dy + row * h;
  float vx[VEC], vd[VEC], g[VEC], s1 = 0.f, s2 = 0.f;
  for (int j = lane * VEC; j < h; j += kWave * VEC) {
    VecLoad<T, VEC>::load(xr + j, vx);
    VecLoad<T, VEC>::load(dyr + j, vd);
    VecLoad<T, VEC>::load(gamma + j, g);
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
      float dxh = vd[i] * g[i];
      s1 += dxh;
      s2 += dxh * ((vx[i] - mean) * rstd);
    }
  }
  const float m1 = wave_sum(s1) / (float)h, m2 = wave_sum(s2) / (float)h;
  const T* rr = res + row * h;
  T* dxr = dx + row * h;
  float vr[VEC];
  for (int j = lane * VEC; j < h; j += kWave * VEC) {
    VecLoad<T, VEC>::load(xr + j, vx);
    VecLoad<T, VEC>::load(dyr + j, vd);
    VecLoad<T, VEC>::load(gamma + j, g);
    VecLoad<T, VEC>::load(rr + j, vr);
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
      float xh = (vx[i] - mean) * rstd;
      vr[i] = vr[i] + rstd * (vd[i] * g[i] - m1 - xh * m2);
    }
    VecLoad<T, VEC>::store(dxr + j, vr);
  }
}

// Raw 16-byte vectors of a row held in registers (NC per lane), so that every tensor is read
// from memory once: rows of up to NC * 64 * VEC elements.
template <typename T, int VEC> struct RawVec { typedef T type __attribute__((ext_vector_type(VEC))); };

template <typename T, int VEC, int NC>
__global__ __launch_bounds__(LN_ROWS_PER_BLOCK* kWave) void layernorm_fwd_cached_kernel(
    const T* __restrict__ x, const T* __restrict__ gamma, const T* __restrict__ beta,
    T* __restrict__ y, float* __restrict__ stats, int64_t rows, int h, float eps) {
  typedef typename RawVec<T, VEC>::type Raw;
  const int lane = threadIdx.x % kWave;
  const int64_t row = (int64_t)blockIdx.x * LN_ROWS_PER_BLOCK + threadIdx.x / kWave;
  if (row >= rows) return;
  const T* xr = x + row * h;
  Raw xc[NC];
  float s = 0.f;
#pragma unroll
  for (int it = 0; it < NC; ++it) {
    const int j = (it * kWave + lane) * VEC;
    if (j < h) {
      xc[it] = *reinterpret_cast<const Raw*>(xr + j);
#pragma unroll
      for (int i = 0; i < VEC; ++i) s += to_f32(xc[it][i]);
    }
  }
  const float mean = wave_sum(s) / (float)h;
  s = 0.f;
#pragma unroll
  for (int it = 0; it < NC; ++it) {
    const int j = (it * kWave + lane) * VEC;
    if (j < h) {
#pragma unroll
      for (int i = 0; i < VEC; ++i) { const float c = to_f32(xc[it][i]) - mean; s += c * c; }
    }
  }
  const float rstd = 1.0f / sqrtf(wave_sum(s) / (float)h + eps);
  if (stats && lane == 0) { stats[row] = mean; stats[rows + row] = rstd; }
  T* yr = y + row * h;
#pragma unroll
  for (int it = 0; it < NC; ++it) {
    const int j = (it * kWave + lane) * VEC;
    if (j < h) {
      const Raw g = *reinterpret_cast<const Raw*>(gamma + j), b = *reinterpret_cast<const Raw*>(beta + j);
      Raw o;
#pragma unroll
      for (int i = 0; i < VEC; ++i) o[i] = from_f32<T>(to_f32(g[i]) * ((to_f32(xc[it][i]) - mean) * rstd) + to_f32(b[i]));
      *reinterpret_cast<Raw*>(yr + j) = o;
    }
  }
}

template <typename T, int VEC, int NC>
__global__ __launch_bounds__(LN_ROWS_PER_BLOCK* kWave) void layernorm_bwd_dx_cached_kernel(
    const T* __restrict__ dy, const T* __restrict__ x, const float* __restrict__ stats,
    const T* __restrict__ gamma, const T* __restrict__ res, T* __restrict__ dx, int64_t rows, int h) {
  typedef typename RawVec<T, VEC>::type Raw;
  const int lane = threadIdx.x % kWave;
  const int64_t row = (int64_t)blockIdx.x * LN_ROWS_PER_BLOCK + threadIdx.x / kWave;
  if (row >= rows) return;
  const float mean = stats[row], rstd = stats[rows + row];
  const T* xr = x + row * h;
  const T* dyr = dy + row * h;
  Raw xc[NC], dc[NC];   // the row of x and of dy; gamma is re-read (it stays in cache)
  float s1 = 0.f, s2 = 0.f;
#pragma unroll
  for (int it = 0; it < NC; ++it) {
    const int j = (it * kWave + lane) * VEC;
    if (j < h) {
      xc[it] = *reinterpret_cast<const Raw*>(xr + j);
      dc[it] = *reinterpret_cast<const Raw*>(dyr + j);
      const Raw g = *reinterpret_cast<const Raw*>(gamma + j);
#pragma unroll
      for (int i = 0; i < VEC; ++i) {
        const float dxh = to_f32(dc[it][i]) * to_f32(g[i]);
        s1 += dxh;
        s2 += dxh * ((to_f32(xc[it][i]) - mean) * rstd);
      }
    }
  }
  const float m1 = wave_sum(s1) / (float)h, m2 = wave_sum(s2) / (float)h;
  const T* rr = res + row * h;
  T* dxr = dx + row * h;
#pragma unroll
  for (int it = 0; it < NC; ++it) {
    const int j = (it * kWave + lane) * VEC;
    if (j < h) {
      const Raw g = *reinterpret_cast<const Raw*>(gamma + j), r = *reinterpret_cast<const Raw*>(rr + j);
      Raw o;
#pragma unroll
      for (int i = 0; i < VEC; ++i) {
        const float xh = (to_f32(xc[it][i]) - mean) * rstd;
        o[i] = from_f32<T>(to_f32(r[i]) + rstd * (to_f32(dc[it][i]) * to_f32(g[i]) - m1 - xh * m2));
      }
      *reinterpret_cast<Raw*>(dxr + j) = o;
    }
  }
}

// Stage 1 of a column reduction over rows [chunk*CR_CHUNK, +CR_CHUNK).
// LNMODE 0: partial[chunk][c] = sum_t a[t,c].
// LNMODE 1: partial[chunk][c] = sum_t a[t,c]*xhat[t,c] (dgamma) and
//           partial[chunk][n+c] = sum_t a[t,c] (dbeta), xhat from x and stats.
template <typename T, int LNMODE>
__global__ __launch_bounds__(CR_COLS* CR_ROWLANES) void colreduce_partial_kernel(
    const T* __restrict__ a, const T* __restrict__ x, const float* __restrict__ stats,
    float* __restrict__ partial, int64_t rows, int64_t n) {
  __shared__ float sh[2][CR_ROWLANES][CR_COLS];
  const int c = threadIdx.x % CR_COLS, rl = threadIdx.x / CR_COLS;
  const int64_t col = (int64_t)blockIdx.x * CR_COLS + c;
  const int64_t r0 = (int64_t)blockIdx.y * CR_CHUNK;
  const int64_t r1 = (r0 + CR_CHUNK < rows) ? r0 + CR_CHUNK : rows;
  float s0 = 0.f, s1 = 0.f;
  if (col < n) {
    for (int64_t t = r0 + rl; t < r1; t += CR_ROWLANES) {
      float v = to_f32(a[t * n + col]);
      if (LNMODE) {
        float xh = (to_f32(x[t * n + col]) - stats[t]) * stats[rows + t];
        s0 += v * xh;
        s1 += v;
      } else {
        s0 += v;
      }
    }
  }
  sh[0][rl][c] = s0;
  sh[1][rl][c] = s1;
  __syncthreads();
  if (rl == 0 && col < n) {
    float t0 = 0.f, t1 = 0.f;
#pragma unroll
    for (int i = 0; i < CR_ROWLANES; ++i) { t0 += sh[0][i][c]; t1 += sh[1][i][c]; }
    const int64_t width = LNMODE ? 2 * n : n;
    partial[(int64_t)blockIdx.y * width + col] = t0;
    if (LNMODE) partial[(int64_t)blockIdx.y * width + n + col] = t1;
  }
}

// Stage 2: out0[c] += sum_chunks partial[chunk][c]; with out1, also the second half.
__global__ __launch_bounds__(256) void colreduce_final_kernel(const float* __restrict__ partial,
                                                              int nchunks, int64_t n,
                                                              float* __restrict__ out0,
                                                              float* __restrict__ out1) {
  const int64_t col = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (col >= n) return;
  const int64_t width = out1 ? 2 * n : n;
  float t0 = 0.f, t1 = 0.f;
  for (int k = 0; k < nchunks; ++k) {
    t0 += partial[(int64_t)k * width + col];
    if (out1) t1 += partial[(int64_t)k * width + n + col];
  }
  out0[col] += t0;
  if (out1) out1[col] += t1;
}

template <typename T> constexpr int ln_vec() { return 16 / (int)sizeof(T); }
inline bool ln_aligned16(std::initializer_list<const void*> ps) {
  for (const void* p : ps)
    if (reinterpret_cast<uintptr_t>(p) & 15) return false;
  return true;
}

template <typename T>
inline hipError_t launch_layernorm_fwd(const T* x, const T* gamma, const T* beta, T* y, float* stats,
                                       int64_t rows, int h, float eps, hipStream_t st) {
  dim3 grid((unsigned)((rows + LN_ROWS_PER_BLOCK - 1) / LN_ROWS_PER_BLOCK)), block(LN_ROWS_PER_BLOCK * kWave);
  constexpr int V = ln_vec<T>();
  if (h % V == 0 && ln_aligned16({x, gamma, beta, y})) {
    const int nv = (h / V + kWave - 1) / kWave;  // 16-byte vectors per lane
    if (nv <= 4) hipLaunchKernelGGL((layernorm_fwd_cached_kernel<T, V, 4>), grid, block, 0, st, x, gamma, beta, y, stats, rows, h, eps);
    else if (nv <= 8) hipLaunchKernelGGL((layernorm_fwd_cached_kernel<T, V, 8>), grid, block, 0, st, x, gamma, beta, y, stats, rows, h, eps);
    else if (nv <= 16) hipLaunchKernelGGL((layernorm_fwd_cached_kernel<T, V, 16>), grid, block, 0, st, x, gamma, beta, y, stats, rows, h, eps);
    else hipLaunchKernelGGL((layernorm_fwd_kernel<T, V>), grid, block, 0, st, x, gamma, beta, y, stats, rows, h, eps);
  } else
    hipLaunchKernelGGL((layernorm_fwd_kernel<T, 1>), grid, block, 0, st, x, gamma, beta, y, stats, rows, h, eps);
  return hipGetLastError();
}

// The same partial column sums with 16-byte accesses: 32 column groups of VEC columns x 8
// row lanes per block; a wavefront reads two 512-byte row segments per instruction.
template <typename T, int LNMODE, int VEC>
__global__ __launch_bounds__(256) void colreduce_partial_vec_kernel(
    const T* __restrict__ a, const T* __restrict__ x, const float* __restrict__ stats,
    float* __restrict__ partial, int64_t rows, int64_t n) {
  constexpr int CG = 32, RL = 8;
  __shared__ float sh[2][RL][CG * VEC];
  const int cg = threadIdx.x % CG, rl = threadIdx.x / CG;
  const int64_t col = ((int64_t)blockIdx.x * CG + cg) * VEC;
  const int64_t r0 = (int64_t)blockIdx.y * CR_CHUNK;
  const int64_t r1 = (r0 + CR_CHUNK < rows) ? r0 + CR_CHUNK : rows;
  float s0[VEC], s1[VEC];
#pragma unroll
  for (int i = 0; i < VEC; ++i) { s0[i] = 0.f; s1[i] = 0.f; }
  if (col < n) {
    for (int64_t t = r0 + rl; t < r1; t += RL) {
      float v[VEC];
      VecLoad<T, VEC>::load(a + t * n + col, v);
      if (LNMODE) {
        float xv[VEC];
        VecLoad<T, VEC>::load(x + t * n + col, xv);
        const float mu = stats[t], rs = stats[rows + t];
#pragma unroll
        for (int i = 0; i < VEC; ++i) { s0[i] += v[i] * ((xv[i] - mu) * rs); s1[i] += v[i]; }
      } else {
#pragma unroll
        for (int i = 0; i < VEC; ++i) s0[i] += v[i];
      }
    }
  }
#pragma unroll
  for (int i = 0; i < VEC; ++i) { sh[0][rl][cg * VEC + i] = s0[i]; if (LNMODE) sh[1][rl][cg * VEC + i] = s1[i]; }
  __syncthreads();
  const int64_t width = LNMODE ? 2 * n : n;
  for (int c = threadIdx.x; c < CG * VEC; c += 256) {
    const int64_t gc = (int64_t)blockIdx.x * CG * VEC + c;
    if (gc >= n) continue;
    float t0 = 0.f, t1 = 0.f;
#pragma unroll
    for (int i = 0; i < RL; ++i) { t0 += sh[0][i][c]; if (LNMODE) t1 += sh[1][i][c]; }
    partial[(int64_t)blockIdx.y * width + gc] = t0;
    if (LNMODE) partial[(int64_t)blockIdx.y * width + n + gc] = t1;
  }
}

template <typename T, int LNMODE>
inline void launch_colreduce_partial(const T* a, const T* x, const float* stats, float* partial, int64_t rows, int64_t n,
                                     hipStream_t st) {
  const int nch = (int)((rows + CR_CHUNK - 1) / CR_CHUNK);
  constexpr int VEC = 16 / sizeof(T);
  const bool aligned = (reinterpret_cast<uintptr_t>(a) % 16 == 0) && (x == nullptr || reinterpret_cast<uintptr_t>(x) % 16 == 0);
  if (n % VEC == 0 && aligned) {
    dim3 g((unsigned)((n + 32 * VEC - 1) / (32 * VEC)), (unsigned)nch);
    hipLaunchKernelGGL((colreduce_partial_vec_kernel<T, LNMODE, VEC>), g, dim3(256), 0, st, a, x, stats, partial, rows, n);
  } else {
    dim3 g((unsigned)((n + CR_COLS - 1) / CR_COLS), (unsigned)nch);
    hipLaunchKernelGGL((colreduce_partial_kernel<T, LNMODE>), g, dim3(CR_COLS * CR_ROWLANES), 0, st, a, x, stats, partial, rows, n);
  }
}

inline int colreduce_chunks(int64_t rows) { return (int)((rows + CR_CHUNK - 1) / CR_CHUNK); }

// dx = res + LN'(dy) alone (one launch).
template <typename T>
inline hipError_t launch_layernorm_bwd_dx(const T* dy, const T* x, const float* stats, const T* gamma,
                                          const T* res, T* dx, int64_t rows, int h, hipStream_t st) {
  dim3 grid((unsigned)((rows + LN_ROWS_PER_BLOCK - 1) / LN_ROWS_PER_BLOCK)), block(LN_ROWS_PER_BLOCK * kWave);
  constexpr int V = ln_vec<T>();
  if (h % V == 0 && ln_aligned16({dy, x, gamma, res, dx})) {
    const int nv = (h / V + kWave - 1) / kWave;
    if (nv <= 4) hipLaunchKernelGGL((layernorm_bwd_dx_cached_kernel<T, V, 4>), grid, block, 0, st, dy, x, stats, gamma, res, dx, rows, h);
    else if (nv <= 8) hipLaunchKernelGGL((layernorm_bwd_dx_cached_kernel<T, V, 8>), grid, block, 0, st, dy, x, stats, gamma, res, dx, rows, h);
    else if (nv <= 16) hipLaunchKernelGGL((layernorm_bwd_dx_cached_kernel<T, V, 16>), grid, block, 0, st, dy, x, stats, gamma, res, dx, rows, h);
    else hipLaunchKernelGGL((layernorm_bwd_dx_kernel<T, V>), grid, block, 0, st, dy, x, stats, gamma, res, dx, rows, h);
  } else
    hipLaunchKernelGGL((layernorm_bwd_dx_kernel<T, 1>), grid, block, 0, st, dy, x, stats, gamma, res, dx, rows, h);
  return hipGetLastError();
}

// dgamma += sum_t dy * xhat, dbeta += sum_t dy (two launches; they read dy, x and the statistics only,
// so they need not run on the stream that carries dx).
template <typename T>
inline hipError_t launch_layernorm_bwd_params(const T* dy, const T* x, const float* stats, float* dgamma, float* dbeta,
                                              float* partial, int64_t rows, int h, hipStream_t st) {
  const int nch = colreduce_chunks(rows);
  launch_colreduce_partial<T, 1>(dy, x, stats, partial, rows, (int64_t)h, st);
  hipLaunchKernelGGL(colreduce_final_kernel, dim3((unsigned)((h + 255) / 256)), dim3(256), 0, st, partial, nch, (int64_t)h, dgamma, dbeta);
  return hipGetLastError();
}

// dx plus the gamma/beta gradient accumulation (three launches).
template <typename T>
inline hipError_t launch_layernorm_bwd(const T* dy, const T* x, const float* stats, const T* gamma,
                                       const T* res, T* dx, float* dgamma, float* dbeta,
                                       float* partial, int64_t rows, int h, hipStream_t st) {
  hipError_t e = launch_layernorm_bwd_dx<T>(dy, x, stats, gamma, res, dx, rows, h, st);
  if (e != hipSuccess) return e;
  return launch_layernorm_bwd_params<T>(dy, x, stats, dgamma, dbeta, partial, rows, h, st);
}

template <typename T>
inline hipError_t launch_colsum(const T* a, float* out, float* partial, int64_t rows, int64_t n, hipStream_t st) {
  const int nch = colreduce_chunks(rows);
  launch_colreduce_partial<T, 0>(a, (const T*)nullptr, (const float*)nullptr, partial, rows, n, st);
  hipLaunchKernelGGL(colreduce_final_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, partial, nch, n, out, (float*)nullptr);
  return hipGetLastError();
}

// out = dropout(in) with the mask of one site (backward of a residual-branch dropout: the
// gradient that enters the branch's GEMMs and bias reduction).  One thread per 4 columns of a
// row = one mask word.
template <typename T>
__global__ __launch_bounds__(256) void dropout_apply_kernel(const T* __restrict__ in, T* __restrict__ out, int64_t rows,
                                                            int64_t cols, DropArgs drop) {
  const int64_t cpr = (cols + 3) / 4;  // column patches per row
  const int64_t total = rows * cpr;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t r = i / cpr, cp = i % cpr;
    const uint32_t w = drop_row_word(drop, (uint32_t)r, (uint32_t)cp);
    const int64_t base = r * cols + cp * 4;
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (cp * 4 + e < cols)
        out[base + e] = drop_keep(drop, w, e) ? from_f32<T>(to_f32(in[base + e]) * drop.scale) : from_f32<T>(0.f);
  }
}

template <typename T>
inline hipError_t launch_dropout_apply(const T* in, T* out, int64_t rows, int64_t cols, const DropArgs& drop, hipStream_t st) {
  const int64_t total = rows * ((cols + 3) / 4);
  int64_t nblk = (total + 255) / 256;
  if (nblk > 16384) nblk = 16384;
  if (nblk < 1) nblk = 1;
  hipLaunchKernelGGL((dropout_apply_kernel<T>), dim3((unsigned)nblk), dim3(256), 0, st, in, out, rows, cols, drop);
  return hipGetLastError();
}

}  // namespace varuna
