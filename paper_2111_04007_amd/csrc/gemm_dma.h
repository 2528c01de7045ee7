// bf16 MFMA GEMM for gfx950: operands go from global memory straight into LDS
// (buffer_load_dwordx4 ... lds, no register staging) into stages of 64 k (two per
// operand, or two of A and three of B: template parameter LS), and MFMA fragments
// are software-pipelined in registers across k-steps and across k-tiles, with one
// workgroup barrier per k-tile.
//
//   acc[m,n] = sum_k A(m,k) * B(n,k)
//   A_KMAJOR: A(m,k) = a[m*lda + k]   else (m-major): A(m,k) = a[k*lda + m]
//   B_KMAJOR: B(n,k) = b[n*ldb + k]   else (n-major): B(n,k) = b[k*ldb + n]
//
// LDS layouts (each wave-level direct load deposits 64 lanes x 16 B contiguously,
// so swizzles are applied by choosing which global chunk a lane fetches):
//   k-major operand : [row][64 k]  (128 B per row, 8 chunks of 16 B),
//                     physical chunk = c ^ ((row ^ (row >> 3)) & 7); fragments by ds_read_b128.
//   m/n-major operand: [k][ROWS]   (ROWS*2 B per k-row), physical chunk within each
//                     group of 16 = c ^ dg_tr_swizzle(k); fragments by the transposing
//                     LDS read ds_read_b64_tr_b16 (16 lanes x 4 k-rows -> each lane
//                     gets 4 consecutive k of its own row), two per 8-k operand.
// Both give a lane the 8 consecutive k-values (lane/32)*8.. of tile row lane%32,
// which is the operand layout of v_mfma_f32_32x32x16_bf16.
#pragma once
#include <type_traits>

#include "common.h"
#include "gemm_epilogue.h"

namespace varuna {

constexpr int DG_BK = 64;      // k per LDS stage: 128-byte row segments keep the L1/L2 path efficient
constexpr int DG_STAGES = 2;

typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* glb_ptr_t;

// s_waitcnt immediates (gfx9 encoding: vmcnt [3:0]+[15:14], expcnt [6:4], lgkmcnt [11:8]).
#define DG_WAIT_VM(n) (((n) & 0xf) | (((n) >> 4) << 14) | (7 << 4) | (15 << 8))
#define DG_WAIT_VM0_LGKM0 (7 << 4)
#define DG_WAIT_LGKM0 (0xf | (3 << 14) | (7 << 4))

// Direct global->LDS staging of one operand tile (ROWS x 64).
//   k-major  : LDS [row][64 k], 8 chunks of 16 B per row, physical chunk = c ^ ((row ^ (row >> 3)) & 7)
//   m/n-major: LDS [k][ROWS],   physical chunk (within each aligned group of 16) = c ^ dg_tr_swizzle(k)
// A transposing read takes, per 16 lanes, 32 B from each of 4 consecutive k-rows, and per 32 lanes 64 B
// from each; k-rows are a multiple of 256 B apart, so unswizzled all four start in the same bank.  The
// XOR values 0, 6, 12, 10 differ both in bits 1-2 and in bits 2-3 of the chunk number: the four rows'
// 32-byte pieces fall into different quarters of 128 B and their 64-byte pieces into different quarters
// of 256 B, which is free of bank conflicts whether the LDS serves 16 or 32 lanes of such a read at once.
__device__ __forceinline__ constexpr int dg_tr_swizzle(int k) { return ((k & 1) * 6) ^ (((k >> 1) & 1) * 12); }

template <int ROWS, int NW, bool KMAJOR>
struct DgLoader {
  static constexpr int NINS = ROWS * DG_BK * 2 / 1024;  // wave-level 1 KB loads per tile
  static constexpr int LPT = NINS / NW;                  // per wave
  static_assert(NINS % NW == 0 && LPT >= 1, "tile rows / waves mismatch");
  static_assert(KMAJOR || ROWS % 128 == 0, "the m/n-major swizzle permutes groups of 16 chunks");
  const bf16* base;             // the whole operand is one buffer; loads beyond its extent return zero
  uint32_t extent;
  uint32_t voff[LPT];           // per-lane byte offset of each of this wave's loads (k-tile 0)
  uint32_t step;                // bytes to advance per k-tile

  __device__ __forceinline__ void init(const bf16* g, int64_t ld, int64_t row0, int wave, int lane, uint32_t extent_bytes) {
    base = g;
    extent = extent_bytes;
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
      const int q = wave + i * NW;
      if (KMAJOR) {
        const int row = q * 8 + (lane >> 3), p = lane & 7;
        const int c = p ^ ((row ^ (row >> 3)) & 7);
        voff[i] = (uint32_t)(((row0 + row) * ld + c * 8) * 2);
      } else {
        constexpr int CPR = ROWS / 8;  // chunks per k-row
        const int slot = q * 64 + lane, krow = slot / CPR, p = slot % CPR;
        const int c = p ^ dg_tr_swizzle(krow);
        voff[i] = (uint32_t)(((int64_t)krow * ld + row0 + c * 8) * 2);
      }
    }
    step = (uint32_t)((KMAJOR ? (int64_t)DG_BK : (int64_t)DG_BK * ld) * 2);
  }

  __device__ __forceinline__ void issue(bf16* lds_tile, int kt, int wave) const {
#if defined(__HIP_DEVICE_COMPILE__)  // the buffer builtins exist in the device pass only
    const uint32_t soff = (uint32_t)kt * step;
    const auto rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16*>(base), 0, extent, 0x00020000);
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
      const int q = wave + i * NW;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_ptr_t)(lds_tile + q * 512), 16, voff[i], soff, 0, 0);
    }
#endif
  }
  // Load number I of this wave alone.  With live == false the descriptor covers zero bytes: every
  // lane is out of range, no memory request is made and the load only deposits zeros, so a
  // k-tile past the end of the reduction costs no branch in the middle of a run of products.
  template <int I>
  __device__ __forceinline__ void issue_one(bf16* lds_tile, int kt, int wave, bool live) const {
#if defined(__HIP_DEVICE_COMPILE__)
    static_assert(I >= 0 && I < LPT, "load index");
    const uint32_t soff = (uint32_t)kt * step;
    const auto rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16*>(base), 0, live ? extent : 0u, 0x00020000);
    const int q = wave + I * NW;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_ptr_t)(lds_tile + q * 512), 16, voff[I], live ? soff : 0u, 0, 0);
#endif
  }
};

// One MFMA operand fragment in registers.  In a kernel whose operands are both k-major the
// fragments are plain 16-byte LDS loads that the compiler tracks and schedules (HAND = false).
// A kernel with an m/n-major operand issues ALL its fragment reads as inline assembly
// (HAND = true): the compiler treats the transposing-read builtin as a possible alias of the
// direct-to-LDS loads and puts a wait for all of them (vmcnt(0)) in front of the first such
// read after every issue of the next k-tile, which exposes the full memory latency once per
// k-tile.  Reads it does not see cost no such wait; their completion is waited for by hand
// (settle() before the first use), and issue order is source order.
template <bool KMAJOR, bool HAND> struct DgFragReg;
template <> struct DgFragReg<true, false> { bf16x8 v; };
template <> struct DgFragReg<true, true> { bf16x8 v; };
template <> struct DgFragReg<false, true> { shortx4 lo, hi; };

template <bool HAND> __device__ __forceinline__ bf16x8 dg_value(const DgFragReg<true, HAND>& f) { return f.v; }
__device__ __forceinline__ bf16x8 dg_value(const DgFragReg<false, true>& f) {
  union { struct { shortx4 a, b; } s; bf16x8 v; } u;
  u.s.a = f.lo; u.s.b = f.hi;
  return u.v;
}
// Waits until every LDS read this wave has issued so far has returned; tied to the fragment's
// registers so that no use of them can be scheduled above it.
__device__ __forceinline__ void dg_settle(DgFragReg<true, false>&) {}
__device__ __forceinline__ void dg_settle(DgFragReg<true, true>& f) { asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f.v)); }
__device__ __forceinline__ void dg_settle(DgFragReg<false, true>& f) {
  asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f.lo), "+v"(f.hi));
}
// The same for a whole array of fragments with one wait.
template <int N> __device__ __forceinline__ void dg_settle_all(DgFragReg<true, false> (&)[N]) {}
template <int N> __device__ __forceinline__ void dg_settle_all(DgFragReg<true, true> (&f)[N]) {
  if constexpr (N == 2) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0].v), "+v"(f[1].v));
  else if constexpr (N == 4) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0].v), "+v"(f[1].v), "+v"(f[2].v), "+v"(f[3].v));
  else {
#pragma unroll
    for (int i = 0; i < N; ++i) dg_settle(f[i]);
  }
}
template <int N> __device__ __forceinline__ void dg_settle_all(DgFragReg<false, true> (&f)[N]) {
  if constexpr (N == 2) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0].lo), "+v"(f[0].hi), "+v"(f[1].lo), "+v"(f[1].hi));
  else if constexpr (N == 4)
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0].lo), "+v"(f[0].hi), "+v"(f[1].lo), "+v"(f[1].hi), "+v"(f[2].lo), "+v"(f[2].hi),
                 "+v"(f[3].lo), "+v"(f[3].hi));
  else {
#pragma unroll
    for (int i = 0; i < N; ++i) dg_settle(f[i]);
  }
}

// Fragment reader: the 8 consecutive k-values KS*16 + (lane/32)*8 .. of row lane%32 of fragment number IDX
// (32 rows each) of the wave's sub-tile, whose first row is wave_base (a multiple of 64).  Fragment number
// and k-step are compile-time values: in the hand-issued forms whatever part of the address they contribute
// additively goes into the instruction's offset field instead of into an address computation.
template <int ROWS, bool KMAJOR, bool HAND>
struct DgFrag {
  template <int IDX, int KS>
  static __device__ __forceinline__ void fetch(DgFragReg<KMAJOR, HAND>& f, const bf16* lds_tile, int wave_base,
                                               std::integral_constant<int, IDX>, std::integral_constant<int, KS>, int lane) {
    if constexpr (KMAJOR) {
      // the swizzle depends on the fragment number through its parity only: row bits 3..5 are 4*IDX + lane bits
      const int row = wave_base + (IDX & 1) * 32 + (lane & 31), c = KS * 2 + (lane >> 5);
      const bf16* p0 = lds_tile + row * DG_BK + ((c ^ ((row ^ (row >> 3)) & 7)) << 3);
      constexpr int IMM = (IDX >> 1) * 64 * DG_BK * 2;   // bytes
      if constexpr (HAND) {
        const uint32_t a0 = (uint32_t)(uintptr_t)(lds_ptr_t)const_cast<bf16*>(p0);
        asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(f.v) : "v"(a0), "n"(IMM));
      } else {
        f.v = *reinterpret_cast<const bf16x8*>(reinterpret_cast<const unsigned char*>(p0) + IMM);
      }
    } else {
      const int blk = lane >> 4, j = lane & 15;
      const int m = wave_base + IDX * 32 + (blk & 1) * 16 + 4 * (j & 3);
      const int kq = j >> 2;  // k-row within its group of 4 == (krow & 3)
      const int c = m >> 3, phys = c ^ dg_tr_swizzle(kq);
      const bf16* p0 = lds_tile + ((blk >> 1) * 8 + kq) * ROWS + phys * 8 + (m & 7);
      const uint32_t a0 = (uint32_t)(uintptr_t)(lds_ptr_t)const_cast<bf16*>(p0);
      constexpr int IMM0 = KS * 16 * ROWS * 2, IMM1 = IMM0 + 4 * ROWS * 2;   // bytes
      static_assert(IMM1 < 65536, "offset field");
      asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(f.lo) : "v"(a0), "n"(IMM0));
      asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(f.hi) : "v"(a0), "n"(IMM1));
    }
  }
};

// Scheduling hints for one k-step: MFMA, then RPM LDS reads (and one direct load if any
// are pending in this step), MFMA, ...
template <int Q, int NMFMA, int NREAD, int RPM, int NVMEM>
struct DgInterleave {
  static __device__ __forceinline__ void hint() {
    if constexpr (Q < NMFMA) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      if constexpr (Q * RPM < NREAD)
        __builtin_amdgcn_sched_group_barrier(0x100, (Q * RPM + RPM <= NREAD) ? RPM : NREAD - Q * RPM, 0);
      if constexpr (Q < NVMEM) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
      DgInterleave<Q + 1, NMFMA, NREAD, RPM, NVMEM>::hint();
    }
  }
};

// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>), unrolled at compile time.
template <int N, typename F>
__device__ __forceinline__ void dg_static_for(F&& f) {
  if constexpr (N > 0) {
    dg_static_for<N - 1>(f);
    f(std::integral_constant<int, N - 1>{});
  }
}
// A half-open range of load numbers handed to one k-step.
template <int LO, int HI> struct DgLoads { static constexpr int lo = LO, hi = HI; };
// Load number J (LO <= J < HI) goes out right after product number dg_load_slot of the k-step's NMFMA.
constexpr int dg_load_slot(int j, int lo, int hi, int nmfma) { return ((j - lo) * nmfma) / (hi - lo); }
constexpr uint32_t dg_load_mask(int lo, int hi, int nmfma) {
  uint32_t m = 0;
  for (int j = lo; j < hi; ++j) m |= 1u << dg_load_slot(j, lo, hi, nmfma);
  return m;
}
// Scheduling hints for one k-step whose direct loads sit after the products named in VMASK.
template <int Q, int NMFMA, int NREAD, int RPM, uint32_t VMASK>
struct DgInterleaveMask {
  static __device__ __forceinline__ void hint() {
    if constexpr (Q < NMFMA) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      if constexpr (Q * RPM < NREAD)
        __builtin_amdgcn_sched_group_barrier(0x100, (Q * RPM + RPM <= NREAD) ? RPM : NREAD - Q * RPM, 0);
      if constexpr ((VMASK >> Q) & 1u) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
      DgInterleaveMask<Q + 1, NMFMA, NREAD, RPM, VMASK>::hint();
    }
  }
};

// bf16 epilogue of one wave's (TM*32) x WN sub-tile whose first output is (row0, col0), through a
// private LDS buffer of 32 rows x WN floats.  acc[i][j][r] is row m = lane%32 of the 32x32 block,
// column n = 8*(r/4) + 4*(lane/32) + r%4.
template <int MODE, int TM, int TN, int WN>
__device__ __forceinline__ void dg_epilogue_bf16(floatx16 (&acc)[TM][TN], unsigned char* buf, const EpiArgs<bf16>& epi,
                                                 int64_t row0, int64_t col0, int lane) {
  constexpr int ROWB = WN * 4;              // bytes per staged fp32 row
  constexpr int LPR = WN / 8;               // lanes per output row (8 columns each)
  constexpr int RPI = 64 / LPR;             // rows per store instruction
  const int frow = lane & 31, fchunk = lane >> 5;
  const int rrow = lane / LPR, rcol = (lane % LPR) * 8;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int c = j * 8 + g * 2 + fchunk;
        floatx4 v = {acc[i][j][g * 4 + 0], acc[i][j][g * 4 + 1], acc[i][j][g * 4 + 2], acc[i][j][g * 4 + 3]};
        *reinterpret_cast<floatx4*>(buf + frow * ROWB + (((c & ~15) | ((c ^ frow) & 15)) << 4)) = v;
      }
    __builtin_amdgcn_s_waitcnt(DG_WAIT_LGKM0);  // own writes landed (the buffer is private to the wave)
#pragma unroll
    for (int sub = 0; sub < 32 / RPI; ++sub) {
      const int r = sub * RPI + rrow, c0 = rcol / 4;
      const floatx4 lo = *reinterpret_cast<const floatx4*>(buf + r * ROWB + (((c0 & ~15) | ((c0 ^ r) & 15)) << 4));
      const floatx4 hi = *reinterpret_cast<const floatx4*>(buf + r * ROWB + ((((c0 + 1) & ~15) | (((c0 + 1) ^ r) & 15)) << 4));
      float v[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      gemm_epilogue8<MODE>(epi, row0 + i * 32 + r, col0 + rcol, v);
    }
    __builtin_amdgcn_s_waitcnt(DG_WAIT_LGKM0);  // reads done before the next pass overwrites
  }
}

// Dynamic LDS of one workgroup: the operand stages, or the epilogue's per-wave staging where that is larger.
template <int BM, int BN, int WGM, int WGN, int MODE, int LS>
constexpr size_t dg_smem_bytes() {
  const size_t stages = (size_t)(LS >= 2 ? 2 * BM + 3 * BN : DG_STAGES * (BM + BN)) * DG_BK * 2;
  const size_t pass = (size_t)WGM * WGN * 32 * (BN / WGN) * 4;   // 32 rows x WN floats per wave
  const size_t epi = (MODE == EPI_ACCUM_F32 || MODE == EPI_STORE_F32) ? 2 * pass : pass;
  return stages > epi ? stages : epi;
}

// LS (load schedule): 0 = the loads of a k-tile go out in one run right after the barrier that
// frees their stage (from the upper half of the waves, or from both halves one k-step apart,
// see below); 1 = every wave sends its share one load at a time between its products, spread
// over the three k-steps that follow that barrier, so that no wave sits at the texture
// addresser's full queue while its products wait.
template <int BM, int BN, int WGM, int WGN, bool A_KMAJOR, bool B_KMAJOR, int MODE, int LS = 0>
__global__ __launch_bounds__(WGM* WGN* kWave) void gemm_dma_kernel(
    const bf16* __restrict__ a, int64_t lda, const bf16* __restrict__ b, int64_t ldb, int K,
    int tiles_m, int tiles_n, EpiArgs<bf16> epi, int xcd_remap, int group) {
  constexpr int NW = WGM * WGN;
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 32, TN = WN / 32;
  // the epilogues swizzle 16-byte chunks of a staged fp32 row by the low four bits of the row
  // number, which needs rows of whole groups of 16 chunks
  static_assert(WM % 32 == 0 && WN % 64 == 0, "wave sub-tile: rows in 32s, columns in 64s");
  constexpr int STAGE_ELEMS = (BM + BN) * DG_BK;
  extern __shared__ __attribute__((aligned(16))) unsigned char dg_smem[];
  bf16* smem = reinterpret_cast<bf16*>(dg_smem);  // [2][A tile | B tile]

  const int tid = threadIdx.x, lane = tid % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int wm = wave / WGN, wn = wave % WGN;

  // Workgroup -> tile.  Consecutive workgroup ids go round-robin over the 8 XCDs; give
  // every XCD a contiguous range of logical tiles, walked in groups of `group` tile rows
  // so the A and B panels an XCD touches stay in its L2.
  int logical = blockIdx.x;
  const int nblk = gridDim.x;
  if (xcd_remap && (nblk & 7) == 0) logical = (blockIdx.x & 7) * (nblk >> 3) + (blockIdx.x >> 3);
  const int width = group * tiles_n;
  const int grp = logical / width;
  const int first_m = grp * group;
  const int gsize = (tiles_m - first_m < group) ? tiles_m - first_m : group;
  const int tile_m = first_m + (logical % width) % gsize;
  const int tile_n = (logical % width) / gsize;
  const int64_t m0 = (int64_t)tile_m * BM, n0 = (int64_t)tile_n * BN;

  // A direct load holds its wave at issue until the texture addresser takes it (about 20
  // cycles per 1 KB load, 64 loads per k-tile and CU), and a wave held there issues no
  // products.  With two waves per SIMD the loads are therefore arranged so that while one
  // wave of a SIMD is held at issue the other keeps the matrix pipe fed (measured per kernel):
  //   both operands k-major: only the upper half of the waves (one per SIMD) sends loads,
  //     the whole k-tile right after the barrier that frees the stage;
  //   an m/n-major operand: every wave sends its share, the lower half right after that
  //     barrier, the upper half one k-step later.
  // With one wave per SIMD every wave sends its share right after the barrier.
  constexpr bool HAND = !(A_KMAJOR && B_KMAJOR);
  constexpr bool SPLIT = (NW == 8) && HAND && LS == 0;          // two issue points
  constexpr int NI = (NW == 8 && !HAND && LS == 0) ? 4 : NW;    // number of issuing waves
  const bool issuer = wave >= NW - NI;
  const int iw = wave - (NW - NI);
  const bool early = !SPLIT || wave < NW / 2;
  DgLoader<BM, NI, A_KMAJOR> la;
  DgLoader<BN, NI, B_KMAJOR> lb;
  la.init(a, lda, m0, issuer ? iw : 0, lane, (uint32_t)((A_KMAJOR ? (int64_t)tiles_m * BM : (int64_t)K) * lda * 2));
  lb.init(b, ldb, n0, issuer ? iw : 0, lane, (uint32_t)((B_KMAJOR ? (int64_t)tiles_n * BN : (int64_t)K) * ldb * 2));
  constexpr int LPT = DgLoader<BM, NI, A_KMAJOR>::LPT + DgLoader<BN, NI, B_KMAJOR>::LPT;

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // gridDim.y splits of the reduction (EPI_STORE_F32 only): this workgroup owns k-tiles kt0 .. kt0+nk-1
  const int nk = K / DG_BK / (int)gridDim.y;
  const int kt0 = (int)blockIdx.y * nk;
  // LDS map.  LS 0, 1: two stages of [A tile | B tile].  LS 2: two stages of A, then three of B.
  constexpr int A_STRIDE = (LS >= 2) ? BM * DG_BK : STAGE_ELEMS;
  constexpr int B_STRIDE = (LS >= 2) ? BN * DG_BK : STAGE_ELEMS;
  constexpr int B_BASE = (LS >= 2) ? 2 * BM * DG_BK : BM * DG_BK;
  // LS >= 2: which of a wave's loads (A's LA first, then B's LB) go out in the k-step after the barrier
  // ([0, C3)), and in k-steps 0, 1, 2 of the next tile ([C3, C0), [C0, C1), [C1, LA+LB)).
  constexpr int LA_ = DgLoader<BM, NI, A_KMAJOR>::LPT, LB_ = DgLoader<BN, NI, B_KMAJOR>::LPT;
  // (Halves of A right after the barrier and in k-step 0, halves of B in k-steps 1 and 2; sending all of A
  // right after the barrier, or three quarters of it, measured the same to half a percent.)
  constexpr int C3 = LA_ / 2, C0 = LA_, C1 = LA_ + LB_ / 2;
  auto a_stage = [&](int i) { return smem + i * A_STRIDE; };
  auto b_stage = [&](int i) { return smem + B_BASE + i * B_STRIDE; };
  if constexpr (LS == 1) {
    // tile 0 whole; of tile 1 only the loads that in the steady state go out right after a
    // barrier -- the k-loop sends the rest during tile 0's first two k-steps, as for any tile
    constexpr int LA1 = DgLoader<BM, NI, A_KMAJOR>::LPT, N31 = (LPT + 2) / 3;
    la.issue(smem, kt0, iw);
    lb.issue(smem + BM * DG_BK, kt0, iw);
    dg_static_for<N31>([&](auto j_tag) {
      constexpr int J = decltype(j_tag)::value;
      if constexpr (J < LA1) la.template issue_one<J>(smem + STAGE_ELEMS, kt0 + 1, iw, nk > 1);
      else lb.template issue_one<J - LA1>(smem + STAGE_ELEMS + BM * DG_BK, kt0 + 1, iw, nk > 1);
    });
    // (a load whose descriptor covers zero bytes makes no memory request and may retire ahead of
    // older loads still in flight: counting outstanding loads is only valid among live ones)
    if (nk > 1) __builtin_amdgcn_s_waitcnt(DG_WAIT_VM(N31)); else __builtin_amdgcn_s_waitcnt(DG_WAIT_VM(0));
  } else if constexpr (LS >= 2) {
    // A(0), B(0) whole, then B(1) whole and the loads of tile 1 that go out right after a barrier (all of
    // them A's): what the steady state has sent for tile 0's period by the time its k-step 0 starts.
    static_assert(C3 <= LA_ && C0 >= LA_, "only A's loads follow the barrier; A is complete after k-step 0");
    la.issue(a_stage(0), kt0, iw);
    lb.issue(b_stage(0), kt0, iw);
    dg_static_for<LB_>([&](auto j_tag) { lb.template issue_one<decltype(j_tag)::value>(b_stage(1), kt0 + 1, iw, nk > 1); });
    dg_static_for<C3>([&](auto j_tag) { la.template issue_one<decltype(j_tag)::value>(a_stage(1), kt0 + 1, iw, nk > 1); });
    if (nk > 1) __builtin_amdgcn_s_waitcnt(DG_WAIT_VM(LB_ + C3)); else __builtin_amdgcn_s_waitcnt(DG_WAIT_VM(0));
  } else if (issuer) {
    la.issue(smem, kt0, iw);
    lb.issue(smem + BM * DG_BK, kt0, iw);
    if (nk > 1) {
      la.issue(smem + STAGE_ELEMS, kt0 + 1, iw);
      lb.issue(smem + STAGE_ELEMS + BM * DG_BK, kt0 + 1, iw);
      __builtin_amdgcn_s_waitcnt(DG_WAIT_VM(LPT));  // tile 0 landed, tile 1 may be in flight
    } else {
      __builtin_amdgcn_s_waitcnt(DG_WAIT_VM(0));
    }
  }
  __builtin_amdgcn_s_barrier();

  DgFragReg<A_KMAJOR, HAND> fa[2][TM];
  DgFragReg<B_KMAJOR, HAND> fb[2][TN];
  static_assert(WM % 64 == 0 && WN % 64 == 0, "the fragment readers take a wave's first row as a multiple of 64");
  using KS0 = std::integral_constant<int, 0>;
  using KS1 = std::integral_constant<int, 1>;
  using KS2 = std::integral_constant<int, 2>;
  using KS3 = std::integral_constant<int, 3>;
  dg_static_for<TN>([&](auto j) { DgFrag<BN, B_KMAJOR, HAND>::fetch(fb[0][decltype(j)::value], b_stage(0), wn * WN, j, KS0{}, lane); });
  dg_static_for<TM>([&](auto i) { DgFrag<BM, A_KMAJOR, HAND>::fetch(fa[0][decltype(i)::value], a_stage(0), wm * WM, i, KS0{}, lane); });

  constexpr int NMFMA = TM * TN;
  constexpr int NREAD = (A_KMAJOR ? TM : 2 * TM) + (B_KMAJOR ? TN : 2 * TN);
  constexpr int RPM = (NREAD + NMFMA - 1) / NMFMA;
  using S0 = std::integral_constant<int, 0>;
  using S1 = std::integral_constant<int, 1>;

  if constexpr (LS == 0) {
  // One k-step of 16: multiply fragment set `cur` while set `cur^1` is fetched from
  // (tile, ks_next).  The hints pin the order MFMA, LDS read, MFMA, LDS read, ... so the
  // LDS latency hides behind the matrix pipe.
  auto kstep = [&](auto cur_tag, const bf16* ta, auto ks_next) {
    constexpr int cur = decltype(cur_tag)::value;
    const bf16* tb = ta + BM * DG_BK;
    // hand-waited fragments of set `cur` (fetched during the previous k-step) first, so the
    // wait does not cover the reads issued next
    dg_settle_all(fb[cur]);
    dg_settle_all(fa[cur]);
    dg_static_for<TN>([&](auto j) { DgFrag<BN, B_KMAJOR, HAND>::fetch(fb[cur ^ 1][decltype(j)::value], tb, wn * WN, j, ks_next, lane); });
    dg_static_for<TM>([&](auto i) { DgFrag<BM, A_KMAJOR, HAND>::fetch(fa[cur ^ 1][decltype(i)::value], ta, wm * WM, i, ks_next, lane); });
    // hand-issued reads go out before this k-step's products, so they have the whole k-step to land
    if constexpr (HAND) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dg_value(fb[cur][j]), dg_value(fa[cur][i]), acc[i][j], 0, 0, 0);
    if constexpr (!HAND) DgInterleave<0, NMFMA, NREAD, RPM, 0>::hint();
    else __builtin_amdgcn_sched_barrier(0);  // the products stay above the next k-step's wait
  };

  // Per k-tile kt (stage kt&1):
  //   k-steps 0..2 multiply while fetching the next k-step's fragments from the same tile;
  //   then every wave waits for its own reads and for its share of tile kt+1 to land, and
  //   the workgroup barrier makes both facts global: tile kt's stage may now be refilled
  //   (tile kt+2 is issued into it) and tile kt+1 may be read;
  //   k-step 3 multiplies while fetching k-step 0 of tile kt+1 (on the last tile that is a
  //   stale but in-bounds read whose result is never used).
  for (int kt = 0; kt < nk; ++kt) {
    bf16* cur = smem + (kt & 1) * STAGE_ELEMS;
    bf16* nxt = smem + ((kt & 1) ^ 1) * STAGE_ELEMS;
    kstep(S0{}, cur, KS1{});
    if (SPLIT && !early && kt >= 1 && kt + 1 < nk) {  // the late half's share of tile kt+1 (tiles 0, 1: sent above)
      la.issue(nxt, kt0 + kt + 1, iw);
      lb.issue(nxt + BM * DG_BK, kt0 + kt + 1, iw);
    }
    kstep(S1{}, cur, KS2{});
    kstep(S0{}, cur, KS3{});
    __builtin_amdgcn_s_waitcnt(DG_WAIT_VM0_LGKM0);
    __builtin_amdgcn_s_barrier();
    if (issuer && early && kt + 2 < nk) {
      la.issue(cur, kt0 + kt + 2, iw);
      lb.issue(cur + BM * DG_BK, kt0 + kt + 2, iw);
    }
    kstep(S1{}, nxt, KS0{});
  }
  } else {
  // Loads sent one at a time between products.  A wave's LT loads of a k-tile are numbered A's
  // first (LA of them), then B's.
  //   LS 1: those numbered [0, N3) go out in the k-step after the barrier that frees their stage,
  //     [N3, N3+N0) and the rest in the two k-steps after it; the k-step before the next barrier
  //     carries none, so the last ones have that long to land.
  //   LS 2: B has a third stage, so B's loads for tile kt+2 can go out while tile kt is still being
  //     read: every k-step carries the same number of loads (A's halves in the k-step after the
  //     barrier and the one after it, B's halves in the other two) and the path from L2 into LDS,
  //     which is what bounds a 256x256 tile, never runs dry between barriers.
  constexpr int LA = DgLoader<BM, NI, A_KMAJOR>::LPT, LB = DgLoader<BN, NI, B_KMAJOR>::LPT, LT = LPT;
  constexpr int N3 = (LT + 2) / 3, N0 = (LT - N3 + 1) / 2;
  auto kstep = [&](auto cur_tag, const bf16* ta, const bf16* tb, auto ks_next, auto loads, bf16* lda_stage, int lda_kt,
                   bool lda_live, bf16* ldb_stage, int ldb_kt, bool ldb_live) {
    constexpr int cur = decltype(cur_tag)::value;
    constexpr int LO = decltype(loads)::lo, HI = decltype(loads)::hi;
    dg_settle_all(fb[cur]);
    dg_settle_all(fa[cur]);
    auto fetch_one = [&](auto r_tag) {   // read number r of the next k-step's fragments: B's first, then A's
      constexpr int R = decltype(r_tag)::value;
      if constexpr (R < TN) DgFrag<BN, B_KMAJOR, HAND>::fetch(fb[cur ^ 1][R], tb, wn * WN, std::integral_constant<int, R>{}, ks_next, lane);
      else DgFrag<BM, A_KMAJOR, HAND>::fetch(fa[cur ^ 1][R - TN], ta, wm * WM, std::integral_constant<int, R - TN>{}, ks_next, lane);
    };
    if constexpr (HAND) {
      dg_static_for<TM + TN>(fetch_one);
      __builtin_amdgcn_sched_barrier(0);
    }
    dg_static_for<NMFMA>([&](auto q_tag) {
      constexpr int Q = decltype(q_tag)::value, I = Q / TN, J = Q % TN;
      acc[I][J] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dg_value(fb[cur][J]), dg_value(fa[cur][I]), acc[I][J], 0, 0, 0);
      if constexpr (!HAND) {   // source order = the order the hints ask for: product, fragment read(s), load
        constexpr int FR = (TM + TN + NMFMA - 1) / NMFMA;   // fragments per product
        dg_static_for<FR>([&](auto f_tag) {
          constexpr int R = Q * FR + decltype(f_tag)::value;
          if constexpr (R < TM + TN) fetch_one(std::integral_constant<int, R>{});
        });
      }
      if constexpr (HI > LO) {
        dg_static_for<HI - LO>([&](auto l_tag) {
          constexpr int L = LO + decltype(l_tag)::value;
          if constexpr (dg_load_slot(L, LO, HI, NMFMA) == Q) {
            if constexpr (HAND) __builtin_amdgcn_sched_barrier(0);
            if constexpr (L < LA) la.template issue_one<L>(lda_stage, lda_kt, iw, lda_live);
            else lb.template issue_one<L - LA>(ldb_stage, ldb_kt, iw, ldb_live);
            if constexpr (HAND) __builtin_amdgcn_sched_barrier(0);
          }
        });
      }
    });
    if constexpr (!HAND) DgInterleaveMask<0, NMFMA, NREAD, RPM, (HI > LO ? dg_load_mask(LO, HI, NMFMA) : 0u)>::hint();
    else __builtin_amdgcn_sched_barrier(0);
  };
  if constexpr (LS == 1) {
    for (int kt = 0; kt < nk; ++kt) {
      bf16* cur = smem + (kt & 1) * STAGE_ELEMS;
      bf16* nxt = smem + ((kt & 1) ^ 1) * STAGE_ELEMS;
      bf16* curb = cur + BM * DG_BK;
      bf16* nxtb = nxt + BM * DG_BK;
      // A load for a k-tile past the end deposits zeros into a stage nobody reads any more.
      const bool live_next = kt + 1 < nk;   // tile kt+1's remaining loads
      kstep(S0{}, cur, curb, KS1{}, DgLoads<N3, N3 + N0>{}, nxt, kt0 + kt + 1, live_next, nxtb, kt0 + kt + 1, live_next);
      kstep(S1{}, cur, curb, KS2{}, DgLoads<N3 + N0, LT>{}, nxt, kt0 + kt + 1, live_next, nxtb, kt0 + kt + 1, live_next);
      kstep(S0{}, cur, curb, KS3{}, DgLoads<0, 0>{}, nxt, 0, false, nxtb, 0, false);
      __builtin_amdgcn_s_waitcnt(DG_WAIT_VM0_LGKM0);
      __builtin_amdgcn_s_barrier();
      kstep(S1{}, nxt, nxtb, KS0{}, DgLoads<0, N3>{}, cur, kt0 + kt + 2, kt + 2 < nk, curb, kt0 + kt + 2, kt + 2 < nk);
    }
  } else {
    // One k-tile whose A stage AP (kt mod 2) and B stage BS (kt mod 3) are compile-time values.
    auto ktile = [&](auto ap_tag, auto bs_tag, int kt) {
      constexpr int AP = decltype(ap_tag)::value, BS = decltype(bs_tag)::value;
      constexpr int BS1 = (BS + 1) % 3, BS2 = (BS + 2) % 3;
      bf16* ca = a_stage(AP);
      bf16* na = a_stage(AP ^ 1);
      bf16* cb = b_stage(BS);
      bf16* nb = b_stage(BS1);
      bf16* nnb = b_stage(BS2);   // held tile kt-1: free since the last barrier
      const bool live1 = kt + 1 < nk, live2 = kt + 2 < nk;
      kstep(S0{}, ca, cb, KS1{}, DgLoads<C3, C0>{}, na, kt0 + kt + 1, live1, nnb, kt0 + kt + 2, live2);
      kstep(S1{}, ca, cb, KS2{}, DgLoads<C0, C1>{}, na, 0, false, nnb, kt0 + kt + 2, live2);
      kstep(S0{}, ca, cb, KS3{}, DgLoads<C1, LT>{}, na, 0, false, nnb, kt0 + kt + 2, live2);
      if (live2) __builtin_amdgcn_s_waitcnt(DG_WAIT_VM(LB) & DG_WAIT_LGKM0);   // (see the loop below)
      else __builtin_amdgcn_s_waitcnt(DG_WAIT_VM0_LGKM0);
      __builtin_amdgcn_s_barrier();
      kstep(S1{}, na, nb, KS0{}, DgLoads<0, C3>{}, ca, kt0 + kt + 2, live2, nnb, 0, false);
    };
    using S2 = std::integral_constant<int, 2>;
    if constexpr (LS == 4) {
      // The loop unrolled over the period of the stage pair (2 x 3 k-tiles): every LDS address of a
      // fragment read or a load's destination is then a lane-dependent register plus a constant, and
      // the address arithmetic that otherwise follows the stage pointers around the loop (about one
      // vector and one scalar instruction per product) is gone.
      int kt = 0;
      for (; kt + 6 <= nk; kt += 6) {
        ktile(S0{}, S0{}, kt);
        ktile(S1{}, S1{}, kt + 1);
        ktile(S0{}, S2{}, kt + 2);
        ktile(S1{}, S0{}, kt + 3);
        ktile(S0{}, S1{}, kt + 4);
        ktile(S1{}, S2{}, kt + 5);
      }
      if (kt < nk) { ktile(S0{}, S0{}, kt); ++kt; }
      if (kt < nk) { ktile(S1{}, S1{}, kt); ++kt; }
      if (kt < nk) { ktile(S0{}, S2{}, kt); ++kt; }
      if (kt < nk) { ktile(S1{}, S0{}, kt); ++kt; }
      if (kt < nk) { ktile(S0{}, S1{}, kt); ++kt; }
    } else {
      int bs = 0;   // B stage of tile kt (kt mod 3)
      for (int kt = 0; kt < nk; ++kt) {
        bf16* ca = a_stage(kt & 1);
        bf16* na = a_stage((kt & 1) ^ 1);
        const int bs1 = bs == 2 ? 0 : bs + 1, bs2 = bs1 == 2 ? 0 : bs1 + 1;
        bf16* cb = b_stage(bs);
        bf16* nb = b_stage(bs1);
        bf16* nnb = b_stage(bs2);   // held tile kt-1: free since the last barrier
        const bool live1 = kt + 1 < nk, live2 = kt + 2 < nk;
        kstep(S0{}, ca, cb, KS1{}, DgLoads<C3, C0>{}, na, kt0 + kt + 1, live1, nnb, kt0 + kt + 2, live2);
        kstep(S1{}, ca, cb, KS2{}, DgLoads<C0, C1>{}, na, 0, false, nnb, kt0 + kt + 2, live2);
        kstep(S0{}, ca, cb, KS3{}, DgLoads<C1, LT>{}, na, 0, false, nnb, kt0 + kt + 2, live2);
        // tile kt+1 must have landed (A's second half went out three k-steps ago, B's a period ago); the
        // LB loads of B(kt+2) sent since then may still be in flight.  That count holds only while
        // those loads are live: past the end of the reduction they make no memory request and may
        // retire ahead of older loads, so the last two k-tiles wait for everything.
        if (live2) __builtin_amdgcn_s_waitcnt(DG_WAIT_VM(LB) & DG_WAIT_LGKM0);
        else __builtin_amdgcn_s_waitcnt(DG_WAIT_VM0_LGKM0);
        __builtin_amdgcn_s_barrier();
        kstep(S1{}, na, nb, KS0{}, DgLoads<0, C3>{}, ca, kt0 + kt + 2, live2, nnb, 0, false);
        bs = bs1;
      }
    }
  }
  }

  const int frow = lane & 31, fchunk = lane >> 5;
  if constexpr (MODE == EPI_ACCUM_F32 || MODE == EPI_STORE_F32) {
    // out_f32 += acc.  Reading the old values through registers would leave only a few KB
    // in flight per CU (the accumulators own the register file), so the old tile is
    // streamed into the now idle LDS with the same direct loads as the operands: each wave
    // pulls its own sub-tile in passes of 32 rows x WN floats, double-buffered, adds its
    // accumulators and stores.  Chunks of 16 B are XOR-swizzled by the row so that 16 lanes
    // reading one column of 16 rows hit distinct banks.
    constexpr int CPR = WN / 4;                 // 16-byte chunks per row of the pass block
    constexpr int PASS_BYTES = 32 * WN * 4;
    constexpr int NINS = PASS_BYTES / 1024;     // direct loads per pass
    static_assert(NW * 2 * PASS_BYTES <= dg_smem_bytes<BM, BN, WGM, WGN, MODE, LS>(), "epilogue staging must fit the workgroup's LDS");
    __builtin_amdgcn_s_waitcnt(DG_WAIT_VM0_LGKM0);
    __builtin_amdgcn_s_barrier();               // every wave is done with the operand stages
    unsigned char* mybuf = dg_smem + wave * (2 * PASS_BYTES);
    float* cbase = epi.out_f32 + (MODE == EPI_STORE_F32 ? (int64_t)blockIdx.y * epi.split_stride : 0) +
                   (m0 + wm * WM) * epi.ldc + n0 + wn * WN;
    auto issue_pass = [&](int pass) {
      unsigned char* buf = mybuf + (pass & 1) * PASS_BYTES;
#pragma unroll
      for (int q = 0; q < NINS; ++q) {
        const int slot = q * 64 + lane, row = slot / CPR, pc = slot % CPR;
        const int c = pc ^ (row & 15);
        __builtin_amdgcn_global_load_lds((glb_ptr_t)(cbase + (int64_t)(pass * 32 + row) * epi.ldc + c * 4),
                                         (lds_ptr_t)(buf + q * 1024), 16, 0, 0);
      }
    };
    if constexpr (MODE == EPI_ACCUM_F32) {
      issue_pass(0);
      if (TM > 1) issue_pass(1);
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      if constexpr (MODE == EPI_ACCUM_F32) {
        if (i + 1 < TM) __builtin_amdgcn_s_waitcnt(DG_WAIT_VM(NINS)); else __builtin_amdgcn_s_waitcnt(DG_WAIT_VM(0));
      }
      const unsigned char* buf = mybuf + (i & 1) * PASS_BYTES;
      float* crow = cbase + (int64_t)(i * 32 + frow) * epi.ldc;
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int c = j * 8 + g * 2 + fchunk;
          floatx4 v = {0.f, 0.f, 0.f, 0.f};   // EPI_STORE_F32: a partial sum of its own, nothing to add to
          if constexpr (MODE == EPI_ACCUM_F32)
            v = *reinterpret_cast<const floatx4*>(buf + frow * (WN * 4) + ((c ^ (frow & 15)) << 4));
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] += acc[i][j][g * 4 + e];
          *reinterpret_cast<floatx4*>(crow + c * 4) = v;
        }
      if (MODE == EPI_ACCUM_F32 && i + 2 < TM) {
        __builtin_amdgcn_s_waitcnt(DG_WAIT_LGKM0);  // this buffer's LDS reads are done before it is refilled
        issue_pass(i + 2);
      }
    }
  } else {
    // bf16 outputs.  acc[i][j][r] is row m = lane%32 of the 32x32 tile, column
    // n = 8*(r/4) + 4*(lane/32) + r%4: storing straight from that layout writes 8-byte
    // pieces of many rows per instruction and was measured to amplify HBM write traffic
    // 2-3x.  Instead each wave transposes its sub-tile through the idle LDS, 32 rows at a
    // time (fp32, chunk-XOR-swizzled), and re-reads it with consecutive lanes along a row,
    // so bias / residual / pre-GeLU reads and all stores are 16 bytes per lane and whole
    // 128-byte lines per row.
    static_assert(NW * 32 * WN * 4 <= dg_smem_bytes<BM, BN, WGM, WGN, MODE, LS>(), "epilogue staging must fit the workgroup's LDS");
    __builtin_amdgcn_s_waitcnt(DG_WAIT_VM0_LGKM0);
    __builtin_amdgcn_s_barrier();             // every wave is done with the operand stages
    dg_epilogue_bf16<MODE, TM, TN, WN>(acc, dg_smem + wave * (32 * WN * 4), epi, m0 + wm * WM, n0 + wn * WN, lane);
  }
}

// ---------------------------------------------------------------------------
// host side.  Variant ids (0 is "the library's choice", -1 the plain FMA kernel):
//   5: 256x256 tile, 8 waves   6: 256x256, 4 waves   7: 128x128, 4 waves   8: 256x128, 4 waves
//   9: as 5 with the spread load schedule   10: as 7 with the spread load schedule   11: as 6 with it
//   12: as 5 with three stages of B and loads in every k-step   13: as 6 with that   14: as 7 with that
//   15: 128x256, 8 waves, that schedule   16: 256x128, 8 waves, that schedule
//   17: as 13 with the k-tile loop unrolled over the stage period   18: as 12 with that
//   19, 20, 21: as 14, 15, 16 with that
// ---------------------------------------------------------------------------
inline bool dg_variant_tile(int variant, GemmTile* t) {
  switch (variant) {
    case 5: case 6: case 9: case 11: case 12: case 13: case 17: case 18: *t = {256, 256}; return true;
    case 7: case 10: case 14: case 19: *t = {128, 128}; return true;
    case 8: case 16: case 21: *t = {256, 128}; return true;
    case 15: case 20: *t = {128, 256}; return true;
    default: return false;
  }
}

inline bool dg_shape_ok(int variant, int64_t M, int64_t N, int64_t K, int64_t lda, int64_t ldb) {
  GemmTile t;
  if (!dg_variant_tile(variant, &t)) return false;
  // operands are addressed with 32-bit byte offsets from their base (buffer loads)
  const int64_t a_bytes = (M > K ? M : K) * lda * 2, b_bytes = (N > K ? N : K) * ldb * 2;
  return M % t.bm == 0 && N % t.bn == 0 && K % DG_BK == 0 && K >= DG_BK && lda % 8 == 0 && ldb % 8 == 0 &&
         (M / t.bm) * (N / t.bn) < (1ll << 31) && a_bytes < (1ll << 32) && b_bytes < (1ll << 32);
}

// Picks between the 256x256 (one workgroup per CU) and 128x128 (two per CU) tiles by the
// number of full-chip rounds each needs; 0 if neither fits the shape.
inline int dg_choose_variant(int64_t M, int64_t N, int64_t K, int64_t lda, int64_t ldb) {
  const bool ok5 = dg_shape_ok(5, M, N, K, lda, ldb), ok7 = dg_shape_ok(7, M, N, K, lda, ldb);
  if (!ok7) return 0;  // anything divisible by 256 is divisible by 128
  if (!ok5) return 7;
  const int64_t t5 = (M / 256) * (N / 256), t7 = (M / 128) * (N / 128);
  const double cost5 = (double)((t5 + 255) / 256) * 4.0 / 1.15;
  const double cost7 = (double)((t7 + 511) / 512) * 2.0;
  return cost5 <= cost7 ? 5 : 7;
}

// Kernel configuration for a product once the tile size is chosen (tile_variant 5: 256x256, 7:
// 128x128), picked by timing whole stage steps with each combination in one process (the chip
// runs the step at its board power limit, so what counts is energy per product, not the rate of
// a kernel alone): the 256x256 forward product runs on 4 waves (128x128 per wave: a third fewer
// LDS reads per product) with a third B stage and loads in every k-step; dgrad keeps 8 waves
// (two per SIMD hide each other's waits on the two-instruction transposed reads) with the same
// load schedule, and so does wgrad (both operands read transposed); all of them with the k-tile
// loop unrolled over the stage period, which removes the address arithmetic from the loop and was
// worth 4.4 % of the C5 step and 1.4-2.6 % of the smaller stages' in same-process A/B.
struct DgFlavours { int fwd256 = 17, bwd256 = 18, fwd128 = 19, dgrad128 = 19, wgrad128 = 19, wgrad256 = 18; bool pair128 = true; };
inline DgFlavours& dg_flavours() { static DgFlavours f; return f; }   // tuning hook: varuna_debug_set_gemm_kernels
inline int dg_flavour(int tile_variant, int op) {
  const DgFlavours& f = dg_flavours();
  if (tile_variant == 5) return op == GEMM_FWD ? f.fwd256 : (op == GEMM_DGRAD ? f.bwd256 : f.wgrad256);
  if (tile_variant == 7) return op == GEMM_FWD ? f.fwd128 : (op == GEMM_DGRAD ? f.dgrad128 : f.wgrad128);
  return tile_variant;
}

// The library's choice for one product.  On top of the tile size and its kernel configuration:
// two 128x128 workgroups on a CU are bound by the CU's path from L2 (64 B per clock), so forward
// and dgrad products may run on 128x256 (else 256x128) tiles of 8 waves instead, one per CU: a pair
// of tiles that shares one operand panel through LDS, a quarter less L2->LDS traffic, measured 8 %
// faster per product.  The merged tiles come in whole rounds of one per CU.  A 128x128 workgroup alone
// on a CU runs at nearly twice the speed (0.55 of a full round's time for a product of at most 256
// tiles), one CU holding two makes the round a full one, and beyond 512 tiles the slots refill as
// they drain; in units of one full round of 512 tiles the two cost 0.55 / 1 / (tiles / 512) and
// 0.92 * ceil(tiles / 2 / 256).
inline int dg_pick(int op, int64_t M, int64_t N, int64_t K, int64_t lda, int64_t ldb) {
  const int tile = dg_choose_variant(M, N, K, lda, ldb);
  if (tile == 7 && op != GEMM_WGRAD && dg_flavours().pair128) {
    const int64_t t = (M / 128) * (N / 128);
    const int wide = dg_shape_ok(20, M, N, K, lda, ldb) ? 20 : (dg_shape_ok(21, M, N, K, lda, ldb) ? 21 : 0);
    if (wide != 0) {
      const double c128 = t <= 256 ? 0.55 : (t <= 512 ? 1.0 : (double)t / 512.0);
      const double cw = 0.92 * (double)((t / 2 + 255) / 256);
      if (cw < c128 - 0.01) return wide;
    }
  }
  return dg_flavour(tile, op);
}

template <int BM, int BN, int WGM, int WGN, bool AK, bool BK_, int MODE, int LS = 0>
inline hipError_t dg_launch_one(const bf16* a, int64_t lda, const bf16* b, int64_t ldb, int64_t M, int64_t N,
                                int64_t K, const EpiArgs<bf16>& epi, int splits, hipStream_t st) {
  auto kern = gemm_dma_kernel<BM, BN, WGM, WGN, AK, BK_, MODE, LS>;
  constexpr size_t smem = dg_smem_bytes<BM, BN, WGM, WGN, MODE, LS>();
  static_assert(smem <= 160 * 1024, "one workgroup's LDS");
  // the first call raises the kernel's dynamic LDS limit (thread-safe: initialisation of a local static)
  static const hipError_t attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (attr_err != hipSuccess) return attr_err;
  const int tm = (int)(M / BM), tn = (int)(N / BN);
  constexpr int xcd_remap = 1, group = 8;   // tile order: contiguous range per XCD, walked in groups of 8 tile rows
  if (splits < 1 || (MODE != EPI_STORE_F32 && splits != 1) || (K / DG_BK) % splits != 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(kern, dim3((unsigned)(tm * tn), (unsigned)splits), dim3(WGM * WGN * kWave), smem, st, a, lda, b, ldb,
                     (int)K, tm, tn, epi, xcd_remap, group);
  return hipGetLastError();
}

template <bool AK, bool BK_, int MODE>
inline hipError_t dg_launch_variant(int variant, const bf16* a, int64_t lda, const bf16* b, int64_t ldb,
                                    int64_t M, int64_t N, int64_t K, const EpiArgs<bf16>& epi, int splits, hipStream_t st) {
  switch (variant) {
    case 5: return dg_launch_one<256, 256, 2, 4, AK, BK_, MODE>(a, lda, b, ldb, M, N, K, epi, splits, st);
    case 6: return dg_launch_one<256, 256, 2, 2, AK, BK_, MODE>(a, lda, b, ldb, M, N, K, epi, splits, st);
    case 7: return dg_launch_one<128, 128, 2, 2, AK, BK_, MODE>(a, lda, b, ldb, M, N, K, epi, splits, st);
    case 8: return dg_launch_one<256, 128, 2, 2, AK, BK_, MODE>(a, lda, b, ldb, M, N, K, epi, splits, st);
    case 9: return dg_launch_one<256, 256, 2, 4, AK, BK_, MODE, 1>(a, lda, b, ldb, M, N, K, epi, splits, st);
    case 10: return dg_launch_one<128, 128, 2, 2, AK, BK_, MODE, 1>(a, lda, b, ldb, M, N, K, epi, splits, st);
    case 11: return dg_launch_one<256, 256, 2, 2, AK, BK_, MODE, 1>(a, lda, b, ldb, M, N, K, epi, splits, st);
    case 12: return dg_launch_one<256, 256, 2, 4, AK, BK_, MODE, 2>(a, lda, b, ldb, M, N, K, epi, splits, st);
    case 13: return dg_launch_one<256, 256, 2, 2, AK, BK_, MODE, 2>(a, lda, b, ldb, M, N, K, epi, splits, st);
    case 14: return dg_launch_one<128, 128, 2, 2, AK, BK_, MODE, 2>(a, lda, b, ldb, M, N, K, epi, splits, st);
    case 15: return dg_launch_one<128, 256, 2, 4, AK, BK_, MODE, 2>(a, lda, b, ldb, M, N, K, epi, splits, st);
    case 16: return dg_launch_one<256, 128, 4, 2, AK, BK_, MODE, 2>(a, lda, b, ldb, M, N, K, epi, splits, st);
    case 17: return dg_launch_one<256, 256, 2, 2, AK, BK_, MODE, 4>(a, lda, b, ldb, M, N, K, epi, splits, st);
    case 18: return dg_launch_one<256, 256, 2, 4, AK, BK_, MODE, 4>(a, lda, b, ldb, M, N, K, epi, splits, st);
    case 19: return dg_launch_one<128, 128, 2, 2, AK, BK_, MODE, 4>(a, lda, b, ldb, M, N, K, epi, splits, st);
    case 20: return dg_launch_one<128, 256, 2, 4, AK, BK_, MODE, 4>(a, lda, b, ldb, M, N, K, epi, splits, st);
    case 21: return dg_launch_one<256, 128, 4, 2, AK, BK_, MODE, 4>(a, lda, b, ldb, M, N, K, epi, splits, st);
    default: return hipErrorInvalidValue;
  }
}

// Split-K for weight-gradient GEMMs whose output has too few tiles to fill the chip: the
// reduction is cut into `splits` equal parts, each workgroup row of the grid writes its
// partial tile (EPI_STORE_F32) and splitk_reduce adds the partials to the accumulator in a
// fixed order, so the result stays run-to-run deterministic.  Returns 1 when no split pays.
inline int dg_wgrad_splits(int64_t M, int64_t N, int64_t K) {
  const int v = dg_choose_variant(M, N, K, M, N);
  GemmTile t;
  if (v == 0 || !dg_variant_tile(v, &t)) return 1;
  const int64_t tiles = (M / t.bm) * (N / t.bn), slots = (v == 5) ? 256 : 512, nk = K / DG_BK;
  int64_t s = slots / tiles;
  if (s > 8) s = 8;
  while (s > 1 && (nk % s != 0 || nk / s < 8)) --s;
  return (int)(s < 1 ? 1 : s);
}

__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ partial, int splits, int64_t n,
                                                            float* __restrict__ out) {
  const int64_t n4 = n / 4;  // n is a multiple of 4 (tile sizes)
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (int64_t)gridDim.x * blockDim.x) {
    floatx4 acc = reinterpret_cast<floatx4*>(out)[i];
    for (int s = 0; s < splits; ++s) {
      const floatx4 p = reinterpret_cast<const floatx4*>(partial + (int64_t)s * n)[i];
      acc[0] += p[0]; acc[1] += p[1]; acc[2] += p[2]; acc[3] += p[3];
    }
    reinterpret_cast<floatx4*>(out)[i] = acc;
  }
}

inline hipError_t launch_splitk_reduce(const float* partial, int splits, int64_t n, float* out, hipStream_t st) {
  int64_t nblk = (n / 4 + 255) / 256;
  if (nblk > 8192) nblk = 8192;
  if (nblk < 1) nblk = 1;
  hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)nblk), dim3(256), 0, st, partial, splits, n, out);
  return hipGetLastError();
}

inline hipError_t launch_gemm_dma(int op, int mode, int variant, const bf16* a, int64_t lda, const bf16* b,
                                  int64_t ldb, int64_t M, int64_t N, int64_t K, const EpiArgs<bf16>& epi,
                                  hipStream_t st, int splits = 1) {
  if (op == GEMM_FWD) {
    if (mode == EPI_BIAS) return dg_launch_variant<true, true, EPI_BIAS>(variant, a, lda, b, ldb, M, N, K, epi, splits, st);
    if (mode == EPI_BIAS_GELU) return dg_launch_variant<true, true, EPI_BIAS_GELU>(variant, a, lda, b, ldb, M, N, K, epi, splits, st);
    if (mode == EPI_BIAS_RES) return dg_launch_variant<true, true, EPI_BIAS_RES>(variant, a, lda, b, ldb, M, N, K, epi, splits, st);
  } else if (op == GEMM_DGRAD) {
    if (mode == EPI_PLAIN) return dg_launch_variant<true, false, EPI_PLAIN>(variant, a, lda, b, ldb, M, N, K, epi, splits, st);
    if (mode == EPI_DGELU) return dg_launch_variant<true, false, EPI_DGELU>(variant, a, lda, b, ldb, M, N, K, epi, splits, st);
  } else if (op == GEMM_WGRAD) {
    if (mode == EPI_ACCUM_F32) return dg_launch_variant<false, false, EPI_ACCUM_F32>(variant, a, lda, b, ldb, M, N, K, epi, splits, st);
    if (mode == EPI_STORE_F32) return dg_launch_variant<false, false, EPI_STORE_F32>(variant, a, lda, b, ldb, M, N, K, epi, splits, st);
    if (mode == EPI_PLAIN) return dg_launch_variant<false, false, EPI_PLAIN>(variant, a, lda, b, ldb, M, N, K, epi, splits, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace varuna
