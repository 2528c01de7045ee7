// bf16 MFMA GEMM for gfx950 with fp32 accumulation and fused epilogues.
//
//   acc[m,n] = sum_k A(m,k) * B(n,k)
//   A_KMAJOR: A(m,k) = a[m*lda + k]   else (m-major): A(m,k) = a[k*lda + m]
//   B_KMAJOR: B(n,k) = b[n*ldb + k]   else (n-major): B(n,k) = b[k*ldb + n]
//
// The three products of a linear layer map onto it as
//   forward  Y  = X W^T   : A = X  (k-major), B = W  (k-major)
//   dgrad    dX = dY W    : A = dY (k-major), B = W  (n-major)
//   wgrad    dW += dY^T X : A = dY (m-major), B = X  (n-major)
//
// Structure: one workgroup owns a BM x BN output tile; the K loop advances in
// steps of 64, staging A and B tiles through registers into a double-buffered,
// XOR-swizzled LDS layout in which each tile row holds its 64 k-values
// contiguously (8 chunks of 16 B).  Operands that are not k-major in memory
// are transposed in registers (8x8 blocks) on the way in, so the MFMA inner
// loop is the same for all three products.  Each wavefront computes a
// (BM/WGM) x (BN/WGN) sub-tile with v_mfma_f32_32x32x16_bf16.  The MFMA is
// issued with the operands swapped (B fragment as the row operand) so that a
// lane ends up holding 4 consecutive n of one output row: the epilogue then
// works on 8-byte (bf16) / 16-byte (fp32) vectors.
//
// Requires M % BM == 0, N % BN == 0, K % 64 == 0, lda/ldb % 8 == 0 and
// 16-byte aligned bases; the host wrapper checks this.
#pragma once
#include "common.h"

namespace varuna {

constexpr int MG_BK = 64;

// LDS element offset of 16-byte chunk c (0..7) of tile row r.
__device__ __forceinline__ int mg_lds_off(int r, int c) {
  return r * MG_BK + (((c ^ r ^ (r >> 3)) & 7) << 3);
}

template <int MODE>
__device__ __forceinline__ void mg_epilogue4(const EpiArgs<bf16>& e, int64_t m, int64_t n, const float* acc) {
  const int64_t idx = m * e.ldc + n;
  if (MODE == EPI_ACCUM_F32) {
    floatx4* p = reinterpret_cast<floatx4*>(e.out_f32 + idx);
    floatx4 v = *p;
    v[0] += acc[0]; v[1] += acc[1]; v[2] += acc[2]; v[3] += acc[3];
    *p = v;
    return;
  }
  float o[4] = {acc[0], acc[1], acc[2], acc[3]};
  if (MODE == EPI_BIAS || MODE == EPI_BIAS_GELU || MODE == EPI_BIAS_RES) {
    bf16x4 bv = *reinterpret_cast<const bf16x4*>(e.bias + n);
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] += (float)bv[i];
  }
  if (MODE == EPI_BIAS_GELU) {
    if (e.aux_out) {
      bf16x4 uv;
#pragma unroll
      for (int i = 0; i < 4; ++i) uv[i] = (bf16)o[i];
      *reinterpret_cast<bf16x4*>(e.aux_out + idx) = uv;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = gelu_logistic_f(o[i]);
  }
  if (MODE == EPI_BIAS_RES) {
    if (e.drop.thr != 0) {  // n is a multiple of 4: one patch row covers the four columns
      const uint32_t w = drop_row_word(e.drop, (uint32_t)m, (uint32_t)(n >> 2));
#pragma unroll
      for (int i = 0; i < 4; ++i) o[i] = drop_keep(e.drop, w, i) ? o[i] * e.drop.scale : 0.f;
    }
    bf16x4 rv = *reinterpret_cast<const bf16x4*>(e.aux_in + idx);
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] += (float)rv[i];
  }
  if (MODE == EPI_DGELU) {
    bf16x4 uv = *reinterpret_cast<const bf16x4*>(e.aux_in + idx);
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] *= gelu_logistic_grad_f((float)uv[i]);
  }
  bf16x4 ov;
#pragma unroll
  for (int i = 0; i < 4; ++i) ov[i] = (bf16)o[i];
  *reinterpret_cast<bf16x4*>(e.out + idx) = ov;
}

// Eight consecutive columns of one output row.
template <int MODE>
__device__ __forceinline__ void mg_epilogue8(const EpiArgs<bf16>& e, int64_t m, int64_t n, const float* acc) {
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

// Global -> register staging of one ROWS x 64 operand tile, and register -> LDS.
// The transposing path (operand not k-major in memory) gives each thread blocks
// of KB k-rows x 8 tile-rows: KB 16-byte loads, a register transpose, then 8
// LDS writes of KB consecutive k-values each.
template <int ROWS, int NT, bool KMAJOR>
struct MgStage {
  static constexpr int NCH = ROWS * 8 / NT;  // 16-byte chunks per thread
  static constexpr int KB = (NCH >= 8) ? 8 : 4;
  static constexpr int NB = NCH / KB;
  static_assert(ROWS * 8 % NT == 0, "tile/threads mismatch");
  static_assert(KMAJOR || (NCH % KB == 0 && NCH >= 4), "transposing loader: unsupported tile/threads");
  bf16x8 v[NCH];

  __device__ __forceinline__ void load(const bf16* __restrict__ g, int64_t ld, int64_t row0, int64_t k0, int tid) {
    if (KMAJOR) {
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        const int q = tid + i * NT, r = q >> 3, c = q & 7;
        v[i] = *reinterpret_cast<const bf16x8*>(g + (row0 + r) * ld + k0 + c * 8);
      }
    } else {
#pragma unroll
      for (int i = 0; i < NB; ++i) {
        const int q = tid + i * NT, rb = q % (ROWS / 8), kb = q / (ROWS / 8);
#pragma unroll
        for (int kk = 0; kk < KB; ++kk)
          v[i * KB + kk] = *reinterpret_cast<const bf16x8*>(g + (k0 + kb * KB + kk) * ld + row0 + rb * 8);
      }
    }
  }

  __device__ __forceinline__ void store(bf16* __restrict__ lds, int tid) const {
    if (KMAJOR) {
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        const int q = tid + i * NT, r = q >> 3, c = q & 7;
        *reinterpret_cast<bf16x8*>(lds + mg_lds_off(r, c)) = v[i];
      }
    } else {
#pragma unroll
      for (int i = 0; i < NB; ++i) {
        const int q = tid + i * NT, rb = q % (ROWS / 8), kb = q / (ROWS / 8);
        const int koff = kb * KB;
#pragma unroll
        for (int rr = 0; rr < 8; ++rr) {
          // tile row rb*8+rr receives the KB k-values of column rr of the block
          bf16* dst = lds + mg_lds_off(rb * 8 + rr, koff >> 3) + (koff & 7);
          if (KB == 8) {
            bf16x8 t;
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) t[kk] = v[i * KB + kk][rr];
            *reinterpret_cast<bf16x8*>(dst) = t;
          } else {
            bf16x4 t;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) t[kk] = v[i * KB + kk][rr];
            *reinterpret_cast<bf16x4*>(dst) = t;
          }
        }
      }
    }
  }
};

template <int BM, int BN, int WGM, int WGN, bool A_KMAJOR, bool B_KMAJOR, int MODE>
__global__ __launch_bounds__(WGM* WGN* kWave) void gemm_mfma_kernel(
    const bf16* __restrict__ a, int64_t lda, const bf16* __restrict__ b, int64_t ldb, int K,
    int tiles_m, int tiles_n, EpiArgs<bf16> epi) {
  constexpr int NT = WGM * WGN * kWave;
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 32, TN = WN / 32;
  static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile must be a multiple of 32x32");
  extern __shared__ __attribute__((aligned(16))) unsigned char mg_smem[];
  bf16* sa = reinterpret_cast<bf16*>(mg_smem);   // [2][BM*64]
  bf16* sb = sa + 2 * BM * MG_BK;                // [2][BN*64]

  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int wm = wave / WGN, wn = wave % WGN;

  // Workgroup -> tile.  Consecutive workgroup ids go round-robin over the 8 XCDs;
  // give every XCD a contiguous range of logical tiles, walked in groups of 8
  // tile rows so the A and B panels an XCD touches stay in its L2.
  int logical = blockIdx.x;
  const int nblk = gridDim.x;
  if ((nblk & 7) == 0) logical = (blockIdx.x & 7) * (nblk >> 3) + (blockIdx.x >> 3);
  constexpr int GROUP = 8;
  const int width = GROUP * tiles_n;
  const int grp = logical / width;
  const int first_m = grp * GROUP;
  const int gsize = (tiles_m - first_m < GROUP) ? tiles_m - first_m : GROUP;
  const int tile_m = first_m + (logical % width) % gsize;
  const int tile_n = (logical % width) / gsize;
  const int64_t m0 = (int64_t)tile_m * BM, n0 = (int64_t)tile_n * BN;

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  MgStage<BM, NT, A_KMAJOR> ga;
  MgStage<BN, NT, B_KMAJOR> gb;
  const int nk = K / MG_BK;
  ga.load(a, lda, m0, 0, tid);
  gb.load(b, ldb, n0, 0, tid);
  ga.store(sa, tid);
  gb.store(sb, tid);
  __syncthreads();

  const int frow = lane & 31, fchunk = lane >> 5;
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) {
      ga.load(a, lda, m0, (int64_t)(kt + 1) * MG_BK, tid);
      gb.load(b, ldb, n0, (int64_t)(kt + 1) * MG_BK, tid);
    }
    const bf16* ca = sa + cur * BM * MG_BK;
    const bf16* cb = sb + cur * BN * MG_BK;
#pragma unroll
    for (int ks = 0; ks < MG_BK / 16; ++ks) {
      bf16x8 fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        fa[i] = *reinterpret_cast<const bf16x8*>(ca + mg_lds_off(wm * WM + i * 32 + frow, ks * 2 + fchunk));
#pragma unroll
      for (int j = 0; j < TN; ++j)
        fb[j] = *reinterpret_cast<const bf16x8*>(cb + mg_lds_off(wn * WN + j * 32 + frow, ks * 2 + fchunk));
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) {
      ga.store(sa + (cur ^ 1) * BM * MG_BK, tid);
      gb.store(sb + (cur ^ 1) * BN * MG_BK, tid);
    }
    __syncthreads();
  }

  // acc[i][j][r]: row m = lane%32 of the 32x32 tile, column n = 8*(r/4) + 4*(lane/32) + r%4.
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int64_t m = m0 + wm * WM + i * 32 + frow;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int64_t n = n0 + wn * WN + j * 32 + g * 8 + fchunk * 4;
        float v[4] = {acc[i][j][g * 4 + 0], acc[i][j][g * 4 + 1], acc[i][j][g * 4 + 2], acc[i][j][g * 4 + 3]};
        mg_epilogue4<MODE>(epi, m, n, v);
      }
    }
  }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
enum GemmOp : int { GEMM_FWD = 0, GEMM_DGRAD = 1, GEMM_WGRAD = 2 };

struct MgTile { int bm, bn; };
// variant ids: 1: 256x256 / 4 waves, 2: 256x256 / 8 waves, 3: 256x128 / 4 waves, 4: 128x128 / 4 waves
inline bool mg_variant_tile(int variant, MgTile* t) {
  switch (variant) {
    case 1: case 2: *t = {256, 256}; return true;
    case 3: *t = {256, 128}; return true;
    case 4: *t = {128, 128}; return true;
    default: return false;
  }
}

inline bool mg_shape_ok(int variant, int64_t M, int64_t N, int64_t K, int64_t lda, int64_t ldb) {
  MgTile t;
  if (!mg_variant_tile(variant, &t)) return false;
  return M % t.bm == 0 && N % t.bn == 0 && K % MG_BK == 0 && K >= MG_BK && lda % 8 == 0 && ldb % 8 == 0 &&
         (M / t.bm) * (N / t.bn) < (1ll << 31);
}

// Picks the largest tile that divides the problem and still fills the 256 CUs.
inline int mg_choose_variant(int64_t M, int64_t N, int64_t K, int64_t lda, int64_t ldb) {
  const int order[3] = {2, 3, 4};
  int fallback = 0;
  for (int v : order) {
    if (!mg_shape_ok(v, M, N, K, lda, ldb)) continue;
    MgTile t;
    mg_variant_tile(v, &t);
    if (!fallback) fallback = v;
    if ((M / t.bm) * (N / t.bn) >= 256) return v;
  }
  // nothing fills the chip: take the smallest tile that fits (most workgroups)
  for (int i = 2; i >= 0; --i)
    if (mg_shape_ok(order[i], M, N, K, lda, ldb)) return order[i];
  return fallback;
}

template <int BM, int BN, int WGM, int WGN, bool AK, bool BK_, int MODE>
inline hipError_t mg_launch_one(const bf16* a, int64_t lda, const bf16* b, int64_t ldb, int64_t M, int64_t N,
                                int64_t K, const EpiArgs<bf16>& epi, hipStream_t st) {
  auto kern = gemm_mfma_kernel<BM, BN, WGM, WGN, AK, BK_, MODE>;
  constexpr size_t smem = (size_t)2 * (BM + BN) * MG_BK * sizeof(bf16);
  static bool attr_set = false;  // per instantiation
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int tm = (int)(M / BM), tn = (int)(N / BN);
  hipLaunchKernelGGL(kern, dim3((unsigned)(tm * tn)), dim3(WGM * WGN * kWave), smem, st, a, lda, b, ldb,
                     (int)K, tm, tn, epi);
  return hipGetLastError();
}

template <bool AK, bool BK_, int MODE>
inline hipError_t mg_launch_variant(int variant, const bf16* a, int64_t lda, const bf16* b, int64_t ldb,
                                    int64_t M, int64_t N, int64_t K, const EpiArgs<bf16>& epi, hipStream_t st) {
  switch (variant) {
    case 1: return mg_launch_one<256, 256, 2, 2, AK, BK_, MODE>(a, lda, b, ldb, M, N, K, epi, st);
    case 2: return mg_launch_one<256, 256, 2, 4, AK, BK_, MODE>(a, lda, b, ldb, M, N, K, epi, st);
    case 3: return mg_launch_one<256, 128, 2, 2, AK, BK_, MODE>(a, lda, b, ldb, M, N, K, epi, st);
    case 4: return mg_launch_one<128, 128, 2, 2, AK, BK_, MODE>(a, lda, b, ldb, M, N, K, epi, st);
    default: return hipErrorInvalidValue;
  }
}

// op/mode dispatch.  Returns hipErrorInvalidValue for combinations that do not exist.
inline hipError_t launch_gemm_mfma(int op, int mode, int variant, const bf16* a, int64_t lda, const bf16* b,
                                   int64_t ldb, int64_t M, int64_t N, int64_t K, const EpiArgs<bf16>& epi,
                                   hipStream_t st) {
  if (op == GEMM_FWD) {
    if (mode == EPI_BIAS) return mg_launch_variant<true, true, EPI_BIAS>(variant, a, lda, b, ldb, M, N, K, epi, st);
    if (mode == EPI_BIAS_GELU) return mg_launch_variant<true, true, EPI_BIAS_GELU>(variant, a, lda, b, ldb, M, N, K, epi, st);
    if (mode == EPI_BIAS_RES) return mg_launch_variant<true, true, EPI_BIAS_RES>(variant, a, lda, b, ldb, M, N, K, epi, st);
  } else if (op == GEMM_DGRAD) {
    if (mode == EPI_PLAIN) return mg_launch_variant<true, false, EPI_PLAIN>(variant, a, lda, b, ldb, M, N, K, epi, st);
    if (mode == EPI_DGELU) return mg_launch_variant<true, false, EPI_DGELU>(variant, a, lda, b, ldb, M, N, K, epi, st);
  } else if (op == GEMM_WGRAD) {
    if (mode == EPI_ACCUM_F32) return mg_launch_variant<false, false, EPI_ACCUM_F32>(variant, a, lda, b, ldb, M, N, K, epi, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace varuna
