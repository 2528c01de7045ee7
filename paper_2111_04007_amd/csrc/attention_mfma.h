// bf16 MFMA flash-style attention for gfx950: forward, and a two-kernel
// deterministic backward (no atomics).  Head dim D in {64, 96, 128}, sequence
// length a multiple of 128.  qkv is [b*s, 3h] (Q | K | V column blocks, head j at
// column j*D of each), ctx / dctx are [b*s, h], lse / delta are [b, heads, s] fp32.
//
// All three kernels keep two 64-row tiles in LDS (rows of D values, padded pitch)
// and hold the other operands in registers.  Products use
// v_mfma_f32_32x32x16_bf16 whose operand layout is: row operand lane L -> row
// L%32, k = 8*(L/32)..+7; column operand likewise; result lane L -> column L%32,
// rows 8*(r/4) + 4*(L/32) + r%4 for the 16 registers r.  Scores are computed
// "transposed" (tile rows as the MFMA row operand) so that a lane ends up with 16
// scores of ONE softmax row per 32x32 block: row statistics need one cross-half
// shuffle, and the probabilities are already laid out as the column operand of
// the following product, whose other operand comes out of LDS through the
// transposing read ds_read_b64_tr_b16 (the k-slot order of the two operands
// then agrees by construction).
//
//   forward (per 128-query workgroup, 32 queries per wave; K, V tiles in LDS):
//     S^T = K Q^T ; online softmax in base 2 ; O^T += V^T P^T
//   backward dQ (same geometry): S^T, dP^T = V dO^T ; dS = P (dP - delta) ;
//     dQ^T += K^T dS^T ; also writes delta = rowsum(dO * O)
//   backward dK/dV (per 128-key workgroup, 32 keys per wave; Q, dO tiles in LDS):
//     S = Q K^T, dP = dO V^T ; dV^T += dO^T P ; dK^T += Q^T dS
#pragma once
#include "common.h"

namespace varuna {

typedef short at_shortx4 __attribute__((ext_vector_type(4)));

template <int D>
struct AttnCfg {
  static_assert(D == 64 || D == 96 || D == 128, "head dim");
  // Row pitch in elements: pitch bytes = 13*16 (D=64) or 19*16 (D=96,128).  An odd number
  // of 16-byte units spreads 16 consecutive rows over all banks for ds_read_b128, and
  // 4 consecutive rows' 32-byte segments do not overlap for the transposing reads.
  static constexpr int PITCH = (D == 64) ? 104 : 152;
  static constexpr int CH = D / 8;             // 16-byte chunks per row
  static constexpr int CPT = 64 * CH / 256;    // chunks per thread for a 64-row tile, 256 threads
  static constexpr int TILE = 64 * PITCH;      // elements per LDS tile
  static constexpr int KD = D / 16;            // k-steps over the head dim
  static constexpr int DB = D / 32;            // 32-wide blocks of the head dim
};

// 64 x D tile: global -> registers -> LDS, 256 threads.
template <int D>
struct AttnTileRegs {
  bf16x8 v[AttnCfg<D>::CPT];
  __device__ __forceinline__ void load(const bf16* __restrict__ base, int64_t row_stride, int tid) {
#pragma unroll
    for (int i = 0; i < AttnCfg<D>::CPT; ++i) {
      const int id = tid + i * 256, r = id / AttnCfg<D>::CH, c = id % AttnCfg<D>::CH;
      v[i] = *reinterpret_cast<const bf16x8*>(base + r * row_stride + c * 8);
    }
  }
  __device__ __forceinline__ void store(bf16* __restrict__ lds, int tid) const {
#pragma unroll
    for (int i = 0; i < AttnCfg<D>::CPT; ++i) {
      const int id = tid + i * 256, r = id / AttnCfg<D>::CH, c = id % AttnCfg<D>::CH;
      *reinterpret_cast<bf16x8*>(lds + r * AttnCfg<D>::PITCH + c * 8) = v[i];
    }
  }
};

// Row operand from an LDS tile: row (row_base + lane%32), columns col0 + 8*(lane/32) .. +7.
template <int D>
__device__ __forceinline__ bf16x8 at_row_frag(const bf16* tile, int row_base, int col0, int lane) {
  return *reinterpret_cast<const bf16x8*>(tile + (row_base + (lane & 31)) * AttnCfg<D>::PITCH + col0 + 8 * (lane >> 5));
}

// Transposed row operand: operand row = tile column (col_base + lane%32); its 8 k-slots are
// tile rows r0 + 4*(lane/32) + {0..3} and r0 + 8 + 4*(lane/32) + {0..3} -- the order in
// which a lane holds the rows of a 32x32 MFMA result, i.e. of P / dS.
template <int D>
__device__ __forceinline__ bf16x8 at_tr_frag(const bf16* tile, int r0, int col_base, int lane) {
  const int j = lane & 15;
  const bf16* p = tile + (r0 + 4 * (lane >> 5) + (j >> 2)) * AttnCfg<D>::PITCH + col_base + ((lane >> 4) & 1) * 16 + 4 * (j & 3);
  at_shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) at_shortx4*)p);
  at_shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) at_shortx4*)(p + 8 * AttnCfg<D>::PITCH));
  union { struct { at_shortx4 a, b; } s; bf16x8 v; } u;
  u.s.a = lo; u.s.b = hi;
  return u.v;
}

// acc += A B with the accumulator pinned to the accumulation registers.  With one wave per
// SIMD the dK/dV kernel spreads over both halves of the register file, and left to itself the
// compiler keeps these long-lived accumulators in the ordinary half and copies all 16
// registers across around every product.  The product is opaque to the compiler here, so the
// wait states a later read of the result needs are inserted by hand (at_mfma_settle).
__device__ __forceinline__ void at_mfma_acc(floatx16& acc, const bf16x8& a, const bf16x8& b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}
__device__ __forceinline__ void at_mfma_settle() { asm volatile("s_nop 15\n\ts_nop 15" ::: "memory"); }

// Value of lane (4*(lane/4) + j) of the same lane quad, j known at compile time after
// unrolling (a DPP quad permutation: no LDS, no wait).
__device__ __forceinline__ uint32_t at_quad_bcast(uint32_t v, int j) {
  switch (j & 3) {
    case 0: return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x00, 0xf, 0xf, false);
    case 1: return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x55, 0xf, 0xf, false);
    case 2: return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xaa, 0xf, 0xf, false);
    default: return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xff, 0xf, 0xf, false);
  }
}

// Dropout mask words for a lane that owns ONE mask row (its query) and, per 32-key block, the
// four 4-key groups g = 0..3 of that row.  The four lanes of a quad own the four rows of the
// same 4x4 mask patches, so each lane generates only the patch of group g = lane%4 and the
// quad exchanges words: out[g] = word (lane%4) of the patch generated by quad lane g.
// row_patch must be the same in all four lanes; col_patch0 is group 0's patch column, group g
// lies two patch columns further per step.
__device__ __forceinline__ void at_drop_row_words(const DropArgs& drop, uint32_t row_patch, uint32_t col_patch0, int lane,
                                                  uint32_t out[4]) {
  const int ql = lane & 3;
  uint32_t own[4];
  drop_patch(drop, row_patch, col_patch0 + 2u * (uint32_t)ql, own);
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    const uint32_t t0 = at_quad_bcast(own[0], g), t1 = at_quad_bcast(own[1], g);
    const uint32_t t2 = at_quad_bcast(own[2], g), t3 = at_quad_bcast(own[3], g);
    out[g] = ql == 0 ? t0 : (ql == 1 ? t1 : (ql == 2 ? t2 : t3));
  }
}

__device__ __forceinline__ bf16x8 at_pack8(const float* p) {
  bf16x8 r;
#pragma unroll
  for (int i = 0; i < 8; ++i) r[i] = (bf16)p[i];
  return r;
}

// ---------------------------------------------------------------------------
// forward
// ---------------------------------------------------------------------------
template <int D, bool CAUSAL, bool DROP>
__global__ __launch_bounds__(256, 2) void attn_fwd_mfma_kernel(const bf16* __restrict__ qkv, bf16* __restrict__ ctx,
                                                            float* __restrict__ lse, int s, int heads,
                                                            float scale_log2e, DropArgs drop) {
  using C = AttnCfg<D>;
  __shared__ __attribute__((aligned(16))) bf16 sk[C::TILE];
  __shared__ __attribute__((aligned(16))) bf16 sv[C::TILE];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hf = lane >> 5;
  // Grid: x = (batch, head), y = query block.  Workgroups are dispatched in x-fastest order,
  // so under the causal mask every head's longest (latest) query blocks start first and only
  // short ones are left at the end of the launch; and because consecutive workgroups go round
  // the 8 XCDs, all query blocks of one head (same x mod 8) share one XCD's L2 for K and V.
  const int qb = gridDim.y - 1 - blockIdx.y;
  const int head = blockIdx.x % heads, bi = blockIdx.x / heads;
  const int h = heads * D;
  const int64_t ld = 3 * (int64_t)h;
  const bf16* base = qkv + (int64_t)bi * s * ld + head * D;
  const int q0 = qb * 128, qw = q0 + wave * 32;  // this wave's first query
  const int query = qw + (lane & 31);

  bf16x8 qf[C::KD];
#pragma unroll
  for (int t = 0; t < C::KD; ++t)
    qf[t] = *reinterpret_cast<const bf16x8*>(base + (int64_t)query * ld + 16 * t + 8 * hf);

  floatx16 o[C::DB];
#pragma unroll
  for (int i = 0; i < C::DB; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[i][r] = 0.f;
  float m = -INFINITY, l = 0.f;

  const int nkb = CAUSAL ? (q0 + 128) / 64 : s / 64;
  AttnTileRegs<D> rk, rv;
  rk.load(base + h, ld, tid);
  rv.load(base + 2 * h, ld, tid);
  for (int kb = 0; kb < nkb; ++kb) {
    if (kb) __syncthreads();
    rk.store(sk, tid);
    rv.store(sv, tid);
    __syncthreads();
    if (kb + 1 < nkb) {
      rk.load(base + (int64_t)(kb + 1) * 64 * ld + h, ld, tid);
      rv.load(base + (int64_t)(kb + 1) * 64 * ld + 2 * h, ld, tid);
    }
    const int k0 = kb * 64;
    if (CAUSAL && k0 > qw + 31) continue;  // whole key block is in this wave's future
    floatx16 sc[2];
#pragma unroll
    for (int sb = 0; sb < 2; ++sb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) sc[sb][r] = 0.f;
      // fragments fetched as one batch ahead of their products (see the dK/dV kernel)
      bf16x8 kfr[C::KD];
#pragma unroll
      for (int t = 0; t < C::KD; ++t) kfr[t] = at_row_frag<D>(sk, sb * 32, 16 * t, lane);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int t = 0; t < C::KD; ++t)
        sc[sb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[t], qf[t], sc[sb], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    // V^T fragments of the first 32 keys: in flight during the softmax arithmetic
    bf16x8 vtr[2][C::DB];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int db = 0; db < C::DB; ++db) vtr[t][db] = at_tr_frag<D>(sv, 16 * t, db * 32, lane);
    __builtin_amdgcn_sched_barrier(0);
    // Raw scores stay in the accumulators until the exponential: the row maximum is taken on
    // them (the scale is positive), and scale and shift fold into one fused multiply-add.
    // Only key blocks that straddle the diagonal pay for the mask.
    float p[2][16];
    float mx = -INFINITY;
    if (CAUSAL && k0 + 63 > qw) {
#pragma unroll
      for (int sb = 0; sb < 2; ++sb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = k0 + sb * 32 + 8 * (r >> 2) + 4 * hf + (r & 3);
          if (key > query) sc[sb][r] = -INFINITY;
        }
    }
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sc[sb][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    // The running reference m only moves when a row's maximum grows by more than 2^8: until
    // then the exponentials are taken against the old reference (they stay below 256, l and
    // the output carry the same factor and the final division removes it), and the block
    // skips rescaling the output accumulators.  Key 0 is visible to every query, so the
    // first block always sets a finite reference.
    const float m_cand = fmaxf(m, mx * scale_log2e);
    const bool grow = m_cand > m + 8.0f;
    if (__builtin_amdgcn_ballot_w64(grow) != 0) {
      const float m_new = grow ? m_cand : m;
      const float alpha = __builtin_amdgcn_exp2f(m - m_new);
      m = m_new;
      l *= alpha;
#pragma unroll
      for (int i = 0; i < C::DB; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[i][r] *= alpha;
    }
    float psum = 0.f;
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        p[sb][r] = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[sb][r], scale_log2e, -m));
        psum += p[sb][r];
      }
    l += psum;   // the softmax is normalised before the dropout
    if (DROP) {
      // this lane's 16 probabilities of a 32-key block are 4 groups of 4 consecutive keys of
      // ONE mask row (its query): one generator call per block, shared within the lane quad
      const uint32_t drow = (uint32_t)(((int64_t)bi * heads + head) * s + query);
#pragma unroll
      for (int sb = 0; sb < 2; ++sb) {
        uint32_t w[4];
        at_drop_row_words(drop, drow >> 2, (uint32_t)(k0 + sb * 32 + 4 * hf) >> 2, lane, w);
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (!drop_keep(drop, w[g], e)) p[sb][4 * g + e] = 0.f;
      }
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int sb = 0; sb < 2; ++sb) {
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const bf16x8 pf = at_pack8(&p[sb][8 * t]);
#pragma unroll
        for (int db = 0; db < C::DB; ++db)
          o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vtr[t][db], pf, o[db], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
      if (sb == 0) {  // the second 32 keys' fragments, into the same registers
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int db = 0; db < C::DB; ++db) vtr[t][db] = at_tr_frag<D>(sv, 32 + 16 * t, db * 32, lane);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
  l += __shfl_xor(l, 32, 64);
  const float inv = (DROP ? drop.scale : 1.0f) / l;
  if (lse && hf == 0) lse[((int64_t)bi * heads + head) * s + query] = (m + log2f(l)) * 0.6931471805599453f;
  bf16* crow = ctx + ((int64_t)bi * s + query) * h + head * D;
#pragma unroll
  for (int db = 0; db < C::DB; ++db)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      bf16x4 v;
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = (bf16)(o[db][4 * g + e] * inv);
      *reinterpret_cast<bf16x4*>(crow + db * 32 + 8 * g + 4 * hf) = v;
    }
}

// ---------------------------------------------------------------------------
// backward, query side: dQ and delta
// ---------------------------------------------------------------------------
template <int D, bool CAUSAL, bool DROP>
__global__ __launch_bounds__(256, 2) void attn_bwd_dq_mfma_kernel(const bf16* __restrict__ qkv, const bf16* __restrict__ ctx,
                                                               const float* __restrict__ lse,
                                                               const bf16* __restrict__ dctx, bf16* __restrict__ dqkv,
                                                               float* __restrict__ delta, int s, int heads,
                                                               float scale, float scale_log2e, DropArgs drop) {
  using C = AttnCfg<D>;
  __shared__ __attribute__((aligned(16))) bf16 sk[C::TILE];
  __shared__ __attribute__((aligned(16))) bf16 sv[C::TILE];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hf = lane >> 5;
  const int qb = gridDim.y - 1 - blockIdx.y;   // grid as in the forward kernel: long query blocks of every head first
  const int head = blockIdx.x % heads, bi = blockIdx.x / heads;
  const int h = heads * D;
  const int64_t ld = 3 * (int64_t)h;
  const bf16* base = qkv + (int64_t)bi * s * ld + head * D;
  const int q0 = qb * 128, qw = q0 + wave * 32;
  const int query = qw + (lane & 31);
  const int64_t orow = ((int64_t)bi * s + query) * h + head * D;
  const int64_t sidx = ((int64_t)bi * heads + head) * s + query;

  bf16x8 qf[C::KD], gf[C::KD];
  float dl = 0.f;
#pragma unroll
  for (int t = 0; t < C::KD; ++t) {
    qf[t] = *reinterpret_cast<const bf16x8*>(base + (int64_t)query * ld + 16 * t + 8 * hf);
    gf[t] = *reinterpret_cast<const bf16x8*>(dctx + orow + 16 * t + 8 * hf);
    const bf16x8 of = *reinterpret_cast<const bf16x8*>(ctx + orow + 16 * t + 8 * hf);
#pragma unroll
    for (int e = 0; e < 8; ++e) dl += (float)gf[t][e] * (float)of[e];
  }
  dl += __shfl_xor(dl, 32, 64);
  if (hf == 0) delta[sidx] = dl;
  const float l2 = lse[sidx] * 1.4426950408889634f;  // log-sum-exp in base 2

  floatx16 dq[C::DB];
#pragma unroll
  for (int i = 0; i < C::DB; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) dq[i][r] = 0.f;

  const int nkb = CAUSAL ? (q0 + 128) / 64 : s / 64;
  AttnTileRegs<D> rk, rv;
  rk.load(base + h, ld, tid);
  rv.load(base + 2 * h, ld, tid);
  for (int kb = 0; kb < nkb; ++kb) {
    if (kb) __syncthreads();
    rk.store(sk, tid);
    rv.store(sv, tid);
    __syncthreads();
    if (kb + 1 < nkb) {
      rk.load(base + (int64_t)(kb + 1) * 64 * ld + h, ld, tid);
      rv.load(base + (int64_t)(kb + 1) * 64 * ld + 2 * h, ld, tid);
    }
    const int k0 = kb * 64;
    // (no per-wave skip of key blocks in this wave's future: the mask zeroes them, and a
    // branch around the products costs registers)
    const bool need_mask = CAUSAL && (k0 + 63 > qw);
#pragma unroll
    for (int sb = 0; sb < 2; ++sb) {
      floatx16 sc, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) { sc[r] = 0.f; dp[r] = 0.f; }
      // fragments fetched in batches ahead of their products (see the dK/dV kernel)
      constexpr int KH = (C::KD + 1) / 2;
#pragma unroll
      for (int t0 = 0; t0 < C::KD; t0 += KH) {
        bf16x8 kfr[KH], vfr[KH];
#pragma unroll
        for (int t = 0; t < KH; ++t)
          if (t0 + t < C::KD) {
            kfr[t] = at_row_frag<D>(sk, sb * 32, 16 * (t0 + t), lane);
            vfr[t] = at_row_frag<D>(sv, sb * 32, 16 * (t0 + t), lane);
          }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < KH; ++t)
          if (t0 + t < C::KD) {
            sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[t], qf[t0 + t], sc, 0, 0, 0);
            dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfr[t], gf[t0 + t], dp, 0, 0, 0);
          }
        __builtin_amdgcn_sched_barrier(0);
      }
      // K^T fragments of the last product: in flight during the arithmetic below
      bf16x8 ktr[2][C::DB];
#pragma unroll
      for (int db = 0; db < C::DB; ++db) ktr[0][db] = at_tr_frag<D>(sk, sb * 32, db * 32, lane);
      __builtin_amdgcn_sched_barrier(0);
      if (DROP) {  // dP = dropout'(dO V^T): same mask words as the forward kernel
        uint32_t w[4];
        at_drop_row_words(drop, (uint32_t)sidx >> 2, (uint32_t)(k0 + sb * 32 + 4 * hf) >> 2, lane, w);
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
          for (int e = 0; e < 4; ++e) dp[4 * g + e] = drop_keep(drop, w[g], e) ? dp[4 * g + e] * drop.scale : 0.f;
      }
      // Below d = 128 only key blocks that straddle or follow the diagonal pay for the mask
      // (a branch on the wave's position); at d = 128 the kernel sits at the register limit,
      // the branch costs a spill, and masking every block was measured faster.
      constexpr bool MASK_BRANCH = D < 128;
      if (MASK_BRANCH && need_mask) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = k0 + sb * 32 + 8 * (r >> 2) + 4 * hf + (r & 3);
          if (key > query) sc[r] = -INFINITY;
        }
      }
      float ds[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float pr = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[r], scale_log2e, -l2));
        if (!MASK_BRANCH && need_mask) {
          const int key = k0 + sb * 32 + 8 * (r >> 2) + 4 * hf + (r & 3);
          if (key > query) pr = 0.f;
        }
        ds[r] = pr * (dp[r] - dl);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int db = 0; db < C::DB; ++db) ktr[1][db] = at_tr_frag<D>(sk, sb * 32 + 16, db * 32, lane);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const bf16x8 df = at_pack8(&ds[8 * t]);
#pragma unroll
        for (int db = 0; db < C::DB; ++db)
          dq[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ktr[t][db], df, dq[db], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
  bf16* drow = dqkv + ((int64_t)bi * s + query) * ld + head * D;
#pragma unroll
  for (int db = 0; db < C::DB; ++db)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      bf16x4 v;
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = (bf16)(dq[db][4 * g + e] * scale);
      *reinterpret_cast<bf16x4*>(drow + db * 32 + 8 * g + 4 * hf) = v;
    }
}

// ---------------------------------------------------------------------------
// backward, key side: dK and dV
// ---------------------------------------------------------------------------
template <int D, bool CAUSAL, bool DROP>
__global__ __launch_bounds__(256) void attn_bwd_dkv_mfma_kernel(const bf16* __restrict__ qkv, const float* __restrict__ lse,
                                                                const bf16* __restrict__ dctx,
                                                                const float* __restrict__ delta, bf16* __restrict__ dqkv,
                                                                int s, int heads, float scale, float scale_log2e,
                                                                DropArgs drop) {
  using C = AttnCfg<D>;
  __shared__ __attribute__((aligned(16))) bf16 sq[C::TILE];
  __shared__ __attribute__((aligned(16))) bf16 sg[C::TILE];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hf = lane >> 5;
  // grid: x = (batch, head), y = key block; early key blocks (most queries under the causal
  // mask) of every head are dispatched first
  const int kblk = blockIdx.y;
  const int head = blockIdx.x % heads, bi = blockIdx.x / heads;
  const int h = heads * D;
  const int64_t ld = 3 * (int64_t)h;
  const bf16* base = qkv + (int64_t)bi * s * ld + head * D;
  const bf16* gbase = dctx + (int64_t)bi * s * h + head * D;
  const int kb0 = kblk * 128, kw = kb0 + wave * 32;  // this wave's first key
  const int key = kw + (lane & 31);
  const int64_t sbase = ((int64_t)bi * heads + head) * s;

  bf16x8 kf[C::KD], vf[C::KD];
#pragma unroll
  for (int t = 0; t < C::KD; ++t) {
    kf[t] = *reinterpret_cast<const bf16x8*>(base + (int64_t)key * ld + h + 16 * t + 8 * hf);
    vf[t] = *reinterpret_cast<const bf16x8*>(base + (int64_t)key * ld + 2 * h + 16 * t + 8 * hf);
  }
  floatx16 dk[C::DB], dv[C::DB];
#pragma unroll
  for (int i = 0; i < C::DB; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dk[i][r] = 0.f; dv[i][r] = 0.f; }

  // Per 64-query tile the statistics lse (scaled to base 2) and delta ride along with the
  // Q / dO tiles: threads 0..63 prefetch lse, 64..127 delta, into registers and then LDS,
  // so the inner loop never waits on a global load.
  __shared__ __attribute__((aligned(16))) float sstat[2][64];
  const int qs = CAUSAL ? kb0 / 64 : 0, nqb = s / 64;
  AttnTileRegs<D> rq, rg;
  float rstat = 0.f;
  auto load_stat = [&](int qb) {
    if (tid < 64) rstat = lse[sbase + qb * 64 + tid] * 1.4426950408889634f;
    else if (tid < 128) rstat = delta[sbase + qb * 64 + tid - 64];
  };
  rq.load(base + (int64_t)qs * 64 * ld, ld, tid);
  rg.load(gbase + (int64_t)qs * 64 * h, h, tid);
  load_stat(qs);
  for (int qb = qs; qb < nqb; ++qb) {
    if (qb > qs) __syncthreads();
    rq.store(sq, tid);
    rg.store(sg, tid);
    if (tid < 128) sstat[tid >> 6][tid & 63] = rstat;
    __syncthreads();
    if (qb + 1 < nqb) {
      rq.load(base + (int64_t)(qb + 1) * 64 * ld, ld, tid);
      rg.load(gbase + (int64_t)(qb + 1) * 64 * h, h, tid);
      load_stat(qb + 1);
    }
    const int q0 = qb * 64;
    // (A wave whose keys all follow the tile's queries is not skipped: that happens in a
    // workgroup's first tile only, the mask zeroes its contribution, and a branch around the
    // products makes the compiler copy all accumulators.)
    const bool need_mask = CAUSAL && (q0 < kw + 31);
    // Order of one 64-query tile (one wave per SIMD: nothing but this order overlaps the LDS
    // with the matrix pipe).  Per 32-query half `sb`: the row fragments of Q and dO for S and
    // dP (all k-steps) and the first half of the transposed fragments for dV/dK go out as one
    // batch; S and dP are multiplied while the tail of that batch is still landing; the second
    // half of the transposed fragments is fetched under the softmax arithmetic; and the row
    // fragments of the NEXT half are fetched before this half's dV/dK products are issued, so
    // they land under those products.  The scheduling fences keep it that way (left alone,
    // the compiler pairs every read with its product and waits for each one).
    bf16x8 qfr[C::KD], gfr[C::KD];
    auto fetch_rows = [&](int sb) {
#pragma unroll
      for (int t = 0; t < C::KD; ++t) {
        qfr[t] = at_row_frag<D>(sq, sb * 32, 16 * t, lane);
        gfr[t] = at_row_frag<D>(sg, sb * 32, 16 * t, lane);
      }
    };
    // (At d = 64 the kernel fits two waves per SIMD, which overlap by themselves; fetching a
    // half ahead would cost the registers that allow it.)
    constexpr bool AHEAD = D > 64;
    if (AHEAD) fetch_rows(0);
#pragma unroll
    for (int sb = 0; sb < 2; ++sb) {
      if (!AHEAD) fetch_rows(sb);
      bf16x8 gtr[2][C::DB], qtr[2][C::DB];
#pragma unroll
      for (int db = 0; db < C::DB; ++db) {
        gtr[0][db] = at_tr_frag<D>(sg, sb * 32, db * 32, lane);
        qtr[0][db] = at_tr_frag<D>(sq, sb * 32, db * 32, lane);
      }
      __builtin_amdgcn_sched_barrier(0);
      floatx16 sc, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) { sc[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
      for (int t = 0; t < C::KD; ++t) {
        sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qfr[t], kf[t], sc, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gfr[t], vf[t], dp, 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int db = 0; db < C::DB; ++db) {
        gtr[1][db] = at_tr_frag<D>(sg, sb * 32 + 16, db * 32, lane);
        qtr[1][db] = at_tr_frag<D>(sq, sb * 32 + 16, db * 32, lane);
      }
      __builtin_amdgcn_sched_barrier(0);
      float pr[16], ds[16];
      // Each group g of 4 consecutive queries is the 4 rows of one mask patch and this lane's
      // key one of its columns; the four lanes of a quad share the patch column, so each
      // generates the patch of group g = lane%4 only and the quad exchanges the words.
      uint32_t own[4];
      if (DROP) drop_patch(drop, ((uint32_t)(sbase + q0 + sb * 32 + 4 * hf) >> 2) + 2u * (uint32_t)(lane & 3), (uint32_t)key >> 2, own);
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int ql = sb * 32 + 8 * g + 4 * hf;  // 4 consecutive queries of the tile
        const floatx4 l4 = *reinterpret_cast<const floatx4*>(&sstat[0][ql]);
        const floatx4 d4 = *reinterpret_cast<const floatx4*>(&sstat[1][ql]);
        uint32_t mw[4];
        if (DROP) {
#pragma unroll
          for (int e = 0; e < 4; ++e) mw[e] = at_quad_bcast(own[e], g);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int r = 4 * g + e;
          float p = __builtin_amdgcn_exp2f(sc[r] * scale_log2e - l4[e]);
          if (need_mask && (q0 + ql + e < key)) p = 0.f;
          float f = 1.0f;
          if (DROP) f = drop_keep(drop, mw[e], key & 3) ? drop.scale : 0.f;
          pr[r] = p * f;
          ds[r] = p * (dp[r] * f - d4[e]);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      if (AHEAD && sb == 0) {  // the second half's row fragments: in flight during this half's dV/dK products
        fetch_rows(1);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const bf16x8 pf = at_pack8(&pr[8 * t]);
        const bf16x8 df = at_pack8(&ds[8 * t]);
#pragma unroll
        for (int db = 0; db < C::DB; ++db) {
          at_mfma_acc(dv[db], gtr[t][db], pf);
          at_mfma_acc(dk[db], qtr[t][db], df);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    // The products above are opaque to the compiler, which therefore adds no wait states
    // between them and anything it may place around the loop's back-edge that reads dk / dv
    // (a copy, a spill).  Settle once per tile: the accumulators are architecturally current
    // at every point outside the run of products.
    at_mfma_settle();
    __builtin_amdgcn_sched_barrier(0);
  }
  at_mfma_settle();
  __builtin_amdgcn_sched_barrier(0);  // the reads of dK/dV below stay below the wait
  bf16* krow = dqkv + ((int64_t)bi * s + key) * ld + h + head * D;
  bf16* vrow = krow + h;
#pragma unroll
  for (int db = 0; db < C::DB; ++db)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      bf16x4 a, c;
#pragma unroll
      for (int e = 0; e < 4; ++e) { a[e] = (bf16)(dk[db][4 * g + e] * scale); c[e] = (bf16)dv[db][4 * g + e]; }
      *reinterpret_cast<bf16x4*>(krow + db * 32 + 8 * g + 4 * hf) = a;
      *reinterpret_cast<bf16x4*>(vrow + db * 32 + 8 * g + 4 * hf) = c;
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
inline bool attn_mfma_supported(int s, int d) { return (d == 64 || d == 96 || d == 128) && s >= 128 && s % 128 == 0; }

template <int D, bool DROP>
inline hipError_t attn_fwd_mfma_d(const bf16* qkv, bf16* ctx, float* lse, int b, int s, int heads, int causal,
                                  const DropArgs& drop, hipStream_t st) {
  dim3 grid((unsigned)(heads * b), (unsigned)(s / 128));
  const float sl = 1.4426950408889634f / sqrtf((float)D);
  if (causal) hipLaunchKernelGGL((attn_fwd_mfma_kernel<D, true, DROP>), grid, dim3(256), 0, st, qkv, ctx, lse, s, heads, sl, drop);
  else hipLaunchKernelGGL((attn_fwd_mfma_kernel<D, false, DROP>), grid, dim3(256), 0, st, qkv, ctx, lse, s, heads, sl, drop);
  return hipGetLastError();
}

inline hipError_t launch_attention_fwd_mfma(const bf16* qkv, bf16* ctx, float* lse, int b, int s, int heads, int d,
                                            int causal, const DropArgs& drop, hipStream_t st) {
  const bool dr = drop.thr != 0;
  if (d == 64) return dr ? attn_fwd_mfma_d<64, true>(qkv, ctx, lse, b, s, heads, causal, drop, st) : attn_fwd_mfma_d<64, false>(qkv, ctx, lse, b, s, heads, causal, drop, st);
  if (d == 96) return dr ? attn_fwd_mfma_d<96, true>(qkv, ctx, lse, b, s, heads, causal, drop, st) : attn_fwd_mfma_d<96, false>(qkv, ctx, lse, b, s, heads, causal, drop, st);
  if (d == 128) return dr ? attn_fwd_mfma_d<128, true>(qkv, ctx, lse, b, s, heads, causal, drop, st) : attn_fwd_mfma_d<128, false>(qkv, ctx, lse, b, s, heads, causal, drop, st);
  return hipErrorInvalidConfiguration;
}

template <int D, bool DROP>
inline hipError_t attn_bwd_mfma_d(const bf16* qkv, const bf16* ctx, const float* lse, const bf16* dctx, bf16* dqkv,
                                  float* delta, int b, int s, int heads, int causal, const DropArgs& drop, hipStream_t st) {
  dim3 grid((unsigned)(heads * b), (unsigned)(s / 128));
  const float sc = 1.0f / sqrtf((float)D), sl = 1.4426950408889634f * sc;
  if (causal) {
    hipLaunchKernelGGL((attn_bwd_dq_mfma_kernel<D, true, DROP>), grid, dim3(256), 0, st, qkv, ctx, lse, dctx, dqkv, delta, s, heads, sc, sl, drop);
    hipLaunchKernelGGL((attn_bwd_dkv_mfma_kernel<D, true, DROP>), grid, dim3(256), 0, st, qkv, lse, dctx, delta, dqkv, s, heads, sc, sl, drop);
  } else {
    hipLaunchKernelGGL((attn_bwd_dq_mfma_kernel<D, false, DROP>), grid, dim3(256), 0, st, qkv, ctx, lse, dctx, dqkv, delta, s, heads, sc, sl, drop);
    hipLaunchKernelGGL((attn_bwd_dkv_mfma_kernel<D, false, DROP>), grid, dim3(256), 0, st, qkv, lse, dctx, delta, dqkv, s, heads, sc, sl, drop);
  }
  return hipGetLastError();
}

inline hipError_t launch_attention_bwd_mfma(const bf16* qkv, const bf16* ctx, const float* lse, const bf16* dctx,
                                            bf16* dqkv, float* delta, int b, int s, int heads, int d, int causal,
                                            const DropArgs& drop, hipStream_t st) {
  const bool dr = drop.thr != 0;
  if (d == 64) return dr ? attn_bwd_mfma_d<64, true>(qkv, ctx, lse, dctx, dqkv, delta, b, s, heads, causal, drop, st) : attn_bwd_mfma_d<64, false>(qkv, ctx, lse, dctx, dqkv, delta, b, s, heads, causal, drop, st);
  if (d == 96) return dr ? attn_bwd_mfma_d<96, true>(qkv, ctx, lse, dctx, dqkv, delta, b, s, heads, causal, drop, st) : attn_bwd_mfma_d<96, false>(qkv, ctx, lse, dctx, dqkv, delta, b, s, heads, causal, drop, st);
  if (d == 128) return dr ? attn_bwd_mfma_d<128, true>(qkv, ctx, lse, dctx, dqkv, delta, b, s, heads, causal, drop, st) : attn_bwd_mfma_d<128, false>(qkv, ctx, lse, dctx, dqkv, delta, b, s, heads, causal, drop, st);
  return hipErrorInvalidConfiguration;
}

}  // namespace varuna
