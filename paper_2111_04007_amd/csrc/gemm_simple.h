// Generic-stride LDS-tiled FMA GEMM with fp32 accumulation.
//   acc[m,n] = sum_k A(m,k) * B(n,k),   A(m,k) = a[m*a_ms + k*a_ks],  B(n,k) = b[n*b_ns + k*b_ks]
// It serves the fp32 path (tolerance 1e-5 rules out reduced-precision matrix
// cores) and any bf16 shape the MFMA kernel's tile constraints do not cover.
// Any M, N, K; every access is bounds-checked.
#pragma once
#include "common.h"

namespace varuna {

constexpr int SG_BM = 64, SG_BN = 64, SG_BK = 16, SG_THREADS = 256;

template <typename T, int MODE>
__global__ __launch_bounds__(SG_THREADS) void gemm_simple_kernel(
    const T* __restrict__ a, int64_t a_ms, int64_t a_ks, const T* __restrict__ b, int64_t b_ns,
    int64_t b_ks, int64_t M, int64_t N, int64_t K, EpiArgs<T> epi) {
  __shared__ float sa[SG_BK][SG_BM + 4];
  __shared__ float sb[SG_BK][SG_BN + 4];
  const int tid = threadIdx.x;
  const int tx = tid % 16, ty = tid / 16;  // 16x16 threads, each a 4x4 patch
  const int64_t m0 = (int64_t)blockIdx.y * SG_BM, n0 = (int64_t)blockIdx.x * SG_BN;
  float acc[4][4] = {};

  // Loader mapping: 64 rows x 16 k = 1024 elements, 4 per thread.  When the
  // operand is contiguous along k, adjacent threads walk k; otherwise rows.
  const bool a_kfast = (a_ks == 1), b_kfast = (b_ks == 1);
  for (int64_t k0 = 0; k0 < K; k0 += SG_BK) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int e = tid + i * SG_THREADS;
      int r = a_kfast ? e / SG_BK : e % SG_BM;
      int kk = a_kfast ? e % SG_BK : e / SG_BM;
      int64_t gm = m0 + r, gk = k0 + kk;
      sa[kk][r] = (gm < M && gk < K) ? to_f32(a[gm * a_ms + gk * a_ks]) : 0.0f;
      r = b_kfast ? e / SG_BK : e % SG_BN;
      kk = b_kfast ? e % SG_BK : e / SG_BN;
      int64_t gn = n0 + r;
      gk = k0 + kk;
      sb[kk][r] = (gn < N && gk < K) ? to_f32(b[gn * b_ns + gk * b_ks]) : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < SG_BK; ++kk) {
      float av[4], bv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) av[i] = sa[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) bv[j] = sb[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int64_t m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int64_t n = n0 + tx * 4 + j;
      if (n < N) epilogue_store<T, MODE>(epi, m, n, acc[i][j]);
    }
  }
}

template <typename T>
inline hipError_t launch_gemm_simple(int mode, const T* a, int64_t a_ms, int64_t a_ks, const T* b,
                                     int64_t b_ns, int64_t b_ks, int64_t M, int64_t N, int64_t K,
                                     const EpiArgs<T>& epi, hipStream_t st) {
  dim3 grid((unsigned)((N + SG_BN - 1) / SG_BN), (unsigned)((M + SG_BM - 1) / SG_BM));
  dim3 block(SG_THREADS);
#define VARUNA_SG_CASE(MODE_)                                                                   \
  case MODE_:                                                                                   \
    hipLaunchKernelGGL((gemm_simple_kernel<T, MODE_>), grid, block, 0, st, a, a_ms, a_ks, b,    \
                       b_ns, b_ks, M, N, K, epi);                                               \
    break;
  switch (mode) {
    VARUNA_SG_CASE(EPI_BIAS)
    VARUNA_SG_CASE(EPI_BIAS_GELU)
    VARUNA_SG_CASE(EPI_BIAS_RES)
    VARUNA_SG_CASE(EPI_DGELU)
    VARUNA_SG_CASE(EPI_PLAIN)
    VARUNA_SG_CASE(EPI_ACCUM_F32)
    default:
      return hipErrorInvalidValue;
  }
#undef VARUNA_SG_CASE
  return hipGetLastError();
}

}  // namespace varuna
