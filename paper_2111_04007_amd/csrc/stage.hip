// Stage driver and C ABI (see include/varuna_stage.h for the contract).
//
// Host side only enqueues kernels on the caller's stream.  The layer loop:
//   forward   : LN1 -> QKV GEMM(+bias) -> attention -> proj GEMM(+bias+residual)
//               -> LN2 -> MLP1 GEMM(+bias+GeLU) -> MLP2 GEMM(+bias+residual)
//   recompute : the same launches, additionally storing LN statistics, the
//               log-sum-exp and the pre-GeLU values, each layer into its own
//               region of the workspace (the last layer's MLP2 is not needed by
//               the backward pass and is skipped)
//   backward  : per layer, top down: MLP2 dgrad(+GeLU') / wgrad, MLP1 dgrad /
//               wgrad, LN2 backward, proj dgrad / wgrad, attention backward,
//               QKV dgrad / wgrad, LN1 backward; bias / gamma / beta gradients by
//               two-stage column reductions.  Every parameter gradient is added
//               to the caller's fp32 buffer.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <type_traits>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/varuna_stage.h"
#include "attention_mfma.h"
#include "attention_simple.h"
#include "common.h"
#include "gemm_dma.h"
#include "gemm_simple.h"
#include "mfma_probe.h"
#include "norm_reduce.h"
#include "optimizer.h"

using namespace varuna;

namespace {

thread_local char g_err[512] = "";

varuna_status_t fail(varuna_status_t code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

#define HIP_TRY(expr)                                                                          \
  do {                                                                                         \
    hipError_t e_ = (expr);                                                                    \
    if (e_ != hipSuccess)                                                                      \
      return fail(VARUNA_EHIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
  } while (0)

inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

struct Dims {
  int L, h, a, d, s, b, M, f, causal, dtype, G;
  float eps;
  int64_t T, E, F;  // tokens, T*h, T*f
  size_t es;        // bytes per activation / parameter element
  uint32_t drop_thr;  // dropout: an element is kept iff its random byte >= drop_thr (0: no dropout)
  float drop_scale;   // 256 / (256 - drop_thr)
};

varuna_status_t make_dims(const varuna_stage_config_t* c, Dims* o) {
  if (!c) return fail(VARUNA_EINVAL, "config is NULL");
  if (c->n_layers < 1 || c->hidden < 1 || c->n_heads < 1 || c->seq_len < 1 || c->micro_batch < 1 ||
      c->n_micro_batches < 1 || c->mlp_hidden < 0)
    return fail(VARUNA_EINVAL, "non-positive dimension in config");
  if (c->hidden % c->n_heads != 0)
    return fail(VARUNA_EINVAL, "hidden (%d) is not a multiple of n_heads (%d)", c->hidden, c->n_heads);
  if (c->dtype != VARUNA_F32 && c->dtype != VARUNA_BF16) return fail(VARUNA_EINVAL, "unknown dtype %d", c->dtype);
  if (c->causal != 0 && c->causal != 1) return fail(VARUNA_EINVAL, "causal must be 0 or 1");
  if (!(c->ln_eps >= 0.0f)) return fail(VARUNA_EINVAL, "ln_eps must be >= 0");
  o->L = c->n_layers; o->h = c->hidden; o->a = c->n_heads; o->d = c->hidden / c->n_heads;
  o->s = c->seq_len; o->b = c->micro_batch; o->M = c->n_micro_batches;
  o->f = c->mlp_hidden ? c->mlp_hidden : 4 * c->hidden;
  o->causal = c->causal; o->dtype = c->dtype;
  if (c->wgrad_group < 0 || c->wgrad_group > 64) return fail(VARUNA_EINVAL, "wgrad_group must be in [0, 64]");
  o->G = c->wgrad_group > 1 ? c->wgrad_group : 1;
  // the MFMA GEMMs address an operand with 32-bit byte offsets: a stacked ring of G slots must stay below 4 GiB
  if (c->dtype == VARUNA_BF16 && o->G > 1 &&
      (int64_t)o->G * c->micro_batch * c->seq_len * (int64_t)(c->mlp_hidden ? c->mlp_hidden : 4 * c->hidden) * 2 >= (1ll << 32))
    return fail(VARUNA_EUNSUPPORTED, "wgrad_group %d: %d stacked micro-batches of the [tokens, mlp_hidden] operand reach 4 GiB",
                c->wgrad_group, o->G);
  o->eps = c->ln_eps > 0.0f ? c->ln_eps : 1e-5f;
  o->T = (int64_t)o->b * o->s; o->E = o->T * o->h; o->F = o->T * o->f;
  o->es = c->dtype == VARUNA_F32 ? 4 : 2;
  if (!(c->dropout_p >= 0.0f) || !(c->dropout_p < 1.0f)) return fail(VARUNA_EINVAL, "dropout_p must lie in [0, 1)");
  o->drop_thr = (uint32_t)lrintf(256.0f * c->dropout_p);
  if (o->drop_thr > 255) return fail(VARUNA_EINVAL, "dropout_p %g rounds to probability 1", (double)c->dropout_p);
  o->drop_scale = 256.0f / (256.0f - (float)o->drop_thr);
  if ((int64_t)o->b * o->a * o->s >= (1ll << 32)) return fail(VARUNA_EUNSUPPORTED, "batch * heads * seq_len exceeds 2^32");
  if (o->s > ATS_MAX_S) return fail(VARUNA_EUNSUPPORTED, "seq_len %d exceeds the supported maximum %d", o->s, ATS_MAX_S);
  if (o->d > ATS_MAX_D) return fail(VARUNA_EUNSUPPORTED, "head dim %d exceeds the supported maximum %d", o->d, ATS_MAX_D);
  if (o->T > (1ll << 24) || (int64_t)o->h > (1 << 20) || (int64_t)o->f > (1 << 22))
    return fail(VARUNA_EUNSUPPORTED, "dimension too large");
  return VARUNA_OK;
}

// element offsets of the 12 parameter tensors inside one layer
struct ParamOffsets { size_t off[VARUNA_PARAMS_PER_LAYER]; size_t n[VARUNA_PARAMS_PER_LAYER]; size_t per_layer; };
ParamOffsets param_offsets(const Dims& D) {
  const size_t h = D.h, f = D.f;
  const size_t n[VARUNA_PARAMS_PER_LAYER] = {h, h, 3 * h * h, 3 * h, h * h, h, h, h, f * h, f, h * f, h};
  ParamOffsets p;
  size_t o = 0;
  for (int i = 0; i < VARUNA_PARAMS_PER_LAYER; ++i) { p.off[i] = o; p.n[i] = n[i]; o += n[i]; }
  p.per_layer = o;
  return p;
}

// byte offsets inside the workspace.
// The operands of the weight-gradient GEMMs (xn1, ctx, xn2, g and dy, du, dx1, dqkv of every
// layer) are rings of G micro-batch slots stacked along the token dimension, so that one
// GEMM with reduction length cnt*T covers the cnt micro-batches gathered since the last
// flush (G = 1: plain per-micro-batch accumulation).
struct LayerArea {
  size_t stats1, qkv, lse, x1, stats2, u, y;   // one copy
  size_t xn1, ctx, xn2, g;                     // rings written by the recompute pass
  size_t dy, du, dx1, dqkv;                    // rings written by the backward pass
  size_t dyd, dx1d;                            // with dropout: dy, dx1 after the branch masks (rings)
};
struct Workspace {
  std::vector<LayerArea> layer;  // per layer: saved activations and backward rings
  LayerArea fwd;                 // scratch of the forward pass (nothing of it is kept)
  size_t saved_begin, saved_end;
  size_t ping[2];                // forward layer outputs (discarded)
  size_t dxn, dxn_b, dctx, delta, partial;   // dxn: gradient of LN2's output, dxn_b: of LN1's
  size_t partial_side;           // reduction partials of the bias-gradient sums that run on the side stream
  size_t stat_partial;           // partial sums of the gradient statistics (doubles)
  size_t splitk, splitk_size;    // partial weight gradients of split-K GEMMs (fp32); size 0 if no GEMM splits
  size_t total;
};
// Largest split-K partial buffer any of the four weight-gradient GEMMs can ask for, over all
// reduction lengths cnt*T (cnt = 1..G micro-batches gathered).
size_t splitk_bytes(const Dims& D) {
  if (D.dtype != VARUNA_BF16) return 0;
  const int64_t shapes[4][2] = {{D.h, D.f}, {D.f, D.h}, {D.h, D.h}, {3 * (int64_t)D.h, D.h}};
  size_t best = 0;
  for (int cnt = 1; cnt <= D.G; ++cnt)
    for (const auto& mn : shapes) {
      const int s = dg_wgrad_splits(mn[0], mn[1], (int64_t)cnt * D.T);
      if (s > 1) best = std::max(best, (size_t)s * mn[0] * mn[1] * sizeof(float));
    }
  return best;
}

Workspace carve(const Dims& D) {
  Workspace w;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t r = o; o = align_up(o + bytes); return r; };
  const size_t E = (size_t)D.E * D.es, F = (size_t)D.F * D.es;
  const size_t lse = (size_t)D.b * D.a * D.s * sizeof(float), st = (size_t)2 * D.T * sizeof(float);
  auto area = [&](size_t G, bool with_backward) {
    LayerArea a{};
    a.stats1 = take(st); a.xn1 = take(G * E); a.qkv = take(3 * E); a.lse = take(lse); a.ctx = take(G * E);
    a.x1 = take(E); a.stats2 = take(st); a.xn2 = take(G * E); a.u = take(F); a.g = take(G * F); a.y = take(E);
    if (with_backward) { a.dy = take(G * E); a.du = take(G * F); a.dx1 = take(G * E); a.dqkv = take(G * 3 * E); }
    return a;
  };
  w.saved_begin = o;
  for (int l = 0; l < D.L; ++l) w.layer.push_back(area((size_t)D.G, false));
  w.saved_end = o;
  for (int l = 0; l < D.L; ++l) {
    LayerArea& a = w.layer[l];
    a.dy = take((size_t)D.G * E); a.du = take((size_t)D.G * F); a.dx1 = take((size_t)D.G * E); a.dqkv = take((size_t)D.G * 3 * E);
    if (D.drop_thr) { a.dyd = take((size_t)D.G * E); a.dx1d = take((size_t)D.G * E); }
    else { a.dyd = a.dy; a.dx1d = a.dx1; }
  }
  w.fwd = area(1, false);
  w.ping[0] = take(E); w.ping[1] = take(E);
  w.dxn = take(E); w.dxn_b = take(E); w.dctx = take(E);
  w.delta = take(lse);
  int64_t widest = 3 * (int64_t)D.h;
  if (D.f > widest) widest = D.f;
  w.partial = take((size_t)colreduce_chunks(D.T) * widest * sizeof(float));
  w.partial_side = take((size_t)colreduce_chunks(D.T) * widest * sizeof(float));
  w.stat_partial = take((size_t)kStatBlocks * 2 * sizeof(double));
  w.splitk_size = splitk_bytes(D);
  w.splitk = take(w.splitk_size);
  w.total = o;
  return w;
}

constexpr int kMaxEvents = 4096;

}  // namespace

struct varuna_stage {
  Dims D;
  ParamOffsets po;
  Workspace ws;
  const char* params;
  float* grads;
  char* boundary;
  char* work;
  std::vector<char> forwarded;
  int pending = 0;  // micro-batches whose weight-gradient GEMMs have not been issued yet
  int kept_mb = -1;  // micro-batch whose internals forward_keep left in the layer areas (-1: none)
  int kept_slot = 0; // ring slot they were written to
  uint64_t seed = 0;  // dropout seed (varuna_stage_set_dropout_seed)
  // The bias-gradient column sums of the backward pass depend on nothing downstream and are
  // HBM-bound: when the caller has handed over a second stream (varuna_stage_set_side_stream)
  // they run there beside the GEMM chain, forked and joined with events inside every backward
  // call; otherwise on the caller's stream, in order.
  hipStream_t side = nullptr;
  hipEvent_t ev_fork = nullptr, ev_join = nullptr;
  bool side_used = false;  // work was forked in the current call and has not been joined yet
  // profiler
  bool prof_on = false;
  std::vector<hipEvent_t> ev;  // pairs
  struct Rec { int cls; double flops, bytes; };
  std::vector<Rec> recs;
};

namespace {

__global__ void fill_zero_f32_kernel(float* p, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = 0.f;
}

// RAII-free profiling bracket: records start/stop events around one launch group.
struct Bracket {
  varuna_stage* st; hipStream_t s; bool active;
  Bracket(varuna_stage* st_, hipStream_t s_, int cls, double flops, double bytes) : st(st_), s(s_), active(false) {
    if (st && st->prof_on && st->recs.size() * 2 + 2 <= st->ev.size()) {
      active = true;
      (void)hipEventRecord(st->ev[st->recs.size() * 2], s);
      st->recs.push_back({cls, flops, bytes});
    }
  }
  ~Bracket() { if (active) (void)hipEventRecord(st->ev[(st->recs.size() - 1) * 2 + 1], s); }
};

// ---- typed operations ------------------------------------------------------

template <typename T> struct GemmDispatch;

template <> struct GemmDispatch<float> {
  static hipError_t run(int op, int mode, int variant, int64_t M, int64_t N, int64_t K, const float* a,
                        const float* b, const EpiArgs<float>& e, hipStream_t s, int splits = 1) {
    (void)variant;
    if (splits != 1) return hipErrorInvalidConfiguration;
    if (op == GEMM_FWD) return launch_gemm_simple<float>(mode, a, K, 1, b, K, 1, M, N, K, e, s);
    if (op == GEMM_DGRAD) return launch_gemm_simple<float>(mode, a, K, 1, b, 1, N, M, N, K, e, s);
    return launch_gemm_simple<float>(mode, a, 1, M, b, 1, N, M, N, K, e, s);
  }
};

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

template <> struct GemmDispatch<bf16> {
  // variant 0: library's choice; -1: force the simple kernel; >0: that MFMA configuration
  static hipError_t run(int op, int mode, int variant, int64_t M, int64_t N, int64_t K, const bf16* a,
                        const bf16* b, const EpiArgs<bf16>& e, hipStream_t s, int splits = 1) {
    const int64_t lda = (op == GEMM_WGRAD) ? M : K;
    const int64_t ldb = (op == GEMM_FWD) ? K : N;
    const bool ptr_ok = aligned16(a) && aligned16(b) && aligned16(e.bias) && aligned16(e.aux_in) &&
                        aligned16(e.out) && aligned16(e.aux_out) && aligned16(e.out_f32) && (N % 8 == 0);
    int v = variant;
    if (v == 0) {
      v = ptr_ok ? dg_pick(op, M, N, K, lda, ldb) : -1;
      if (v == 0) v = -1;
    }
    if (v >= 5) {
      if (!ptr_ok || !dg_shape_ok(v, M, N, K, lda, ldb)) return hipErrorInvalidConfiguration;
      return launch_gemm_dma(op, mode, v, a, lda, b, ldb, M, N, K, e, s, splits);
    }
    if (splits != 1 || v != -1) return hipErrorInvalidConfiguration;
    if (op == GEMM_FWD) return launch_gemm_simple<bf16>(mode, a, K, 1, b, K, 1, M, N, K, e, s);
    if (op == GEMM_DGRAD) return launch_gemm_simple<bf16>(mode, a, K, 1, b, 1, N, M, N, K, e, s);
    return launch_gemm_simple<bf16>(mode, a, 1, M, b, 1, N, M, N, K, e, s);
  }
};

template <typename T> struct AttnDispatch {
  static hipError_t fwd(int variant, const T* qkv, T* ctx, float* lse, int b, int s, int a, int d, int causal,
                        const DropArgs& drop, hipStream_t st) {
    (void)variant;
    return launch_attention_fwd_simple<T>(qkv, ctx, lse, b, s, a, d, causal, drop, st);
  }
  static hipError_t bwd(int variant, const T* qkv, const T* ctx, const float* lse, const T* dctx, T* dqkv,
                        float* delta, int b, int s, int a, int d, int causal, const DropArgs& drop, hipStream_t st) {
    (void)variant;
    return launch_attention_bwd_simple<T>(qkv, ctx, lse, dctx, dqkv, delta, b, s, a, d, causal, drop, st);
  }
};

template <> struct AttnDispatch<bf16> {
  // variant 0: library's choice; -1: simple kernels; 1: MFMA kernels
  static hipError_t fwd(int variant, const bf16* qkv, bf16* ctx, float* lse, int b, int s, int a, int d, int causal,
                        const DropArgs& drop, hipStream_t st) {
    int v = variant;
    if (v == 0) v = attn_mfma_supported(s, d) ? 1 : -1;
    if (v == 1) {
      if (!attn_mfma_supported(s, d)) return hipErrorInvalidConfiguration;
      return launch_attention_fwd_mfma(qkv, ctx, lse, b, s, a, d, causal, drop, st);
    }
    return launch_attention_fwd_simple<bf16>(qkv, ctx, lse, b, s, a, d, causal, drop, st);
  }
  static hipError_t bwd(int variant, const bf16* qkv, const bf16* ctx, const float* lse, const bf16* dctx, bf16* dqkv,
                        float* delta, int b, int s, int a, int d, int causal, const DropArgs& drop, hipStream_t st) {
    int v = variant;
    if (v == 0) v = attn_mfma_supported(s, d) ? 1 : -1;
    if (v == 1) {
      if (!attn_mfma_supported(s, d)) return hipErrorInvalidConfiguration;
      return launch_attention_bwd_mfma(qkv, ctx, lse, dctx, dqkv, delta, b, s, a, d, causal, drop, st);
    }
    return launch_attention_bwd_simple<bf16>(qkv, ctx, lse, dctx, dqkv, delta, b, s, a, d, causal, drop, st);
  }
};

// ---- the stage passes -------------------------------------------------------

template <typename T>
struct StageOps {
  varuna_stage* S;
  hipStream_t st;
  const Dims& D;
  StageOps(varuna_stage* s_, hipStream_t st_) : S(s_), st(st_), D(s_->D) {}

  const T* param(int l, int which) const {
    return reinterpret_cast<const T*>(S->params) + (size_t)l * S->po.per_layer + S->po.off[which];
  }
  float* grad(int l, int which) const { return S->grads + (size_t)l * S->po.per_layer + S->po.off[which]; }
  template <typename U> U* wsp(size_t off) const { return reinterpret_cast<U*>(S->work + off); }

  // Dropout arguments of `site` in layer l for micro-batch mb (thr = 0 when the stage has no dropout).
  DropArgs drop_args(uint32_t site, int l, int mb) const {
    return DropArgs{D.drop_thr, D.drop_scale, (uint32_t)(S->seed & 0xffffffffu), (uint32_t)(S->seed >> 32),
                    site + 256u * (uint32_t)l, (uint32_t)mb};
  }

  hipError_t gemm(int cls, int op, int mode, int64_t M, int64_t N, int64_t K, const T* a, const T* b, const T* bias,
                  const T* aux_in, T* out, T* aux_out, float* out_f32, const DropArgs& drop = DropArgs{}) {
    EpiArgs<T> e{bias, aux_in, out, aux_out, out_f32, N, drop};
    double bytes = (double)(M * K + N * K) * sizeof(T) + (double)M * N * (out_f32 ? 8.0 : (double)sizeof(T));
    Bracket br(S, st, cls, 2.0 * M * N * K, bytes);
    return GemmDispatch<T>::run(op, mode, 0, M, N, K, a, b, e, st);
  }

  double attn_flops_fwd() const {
    double dense = 4.0 * D.b * D.a * (double)D.s * D.s * D.d;
    return D.causal ? dense * 0.5 : dense;
  }

  // One layer forward.  rs: ring slot of the wgrad operands (xn1, ctx, xn2, g).
  // save: also store stats, lse, u.  skip_mlp2: stop after GeLU.
  hipError_t layer_forward(int l, int mb, const T* x, T* y, const LayerArea& A, int rs, bool save, bool skip_mlp2) {
    hipError_t e;
    const int64_t T_ = D.T;
    T* xn1 = wsp<T>(A.xn1) + (size_t)rs * D.E; T* qkv = wsp<T>(A.qkv); T* ctx = wsp<T>(A.ctx) + (size_t)rs * D.E;
    T* x1 = wsp<T>(A.x1); T* xn2 = wsp<T>(A.xn2) + (size_t)rs * D.E; T* u = wsp<T>(A.u);
    T* g = wsp<T>(A.g) + (size_t)rs * D.F;
    float* stats1 = save ? wsp<float>(A.stats1) : nullptr;
    float* stats2 = save ? wsp<float>(A.stats2) : nullptr;
    float* lse = save ? wsp<float>(A.lse) : nullptr;
    {
      Bracket br(S, st, VARUNA_K_LN_FWD, 0, 2.0 * D.E * sizeof(T));
      if ((e = launch_layernorm_fwd<T>(x, param(l, VARUNA_P_LN1_G), param(l, VARUNA_P_LN1_B), xn1, stats1, T_, D.h, D.eps, st))) return e;
    }
    if ((e = gemm(VARUNA_K_GEMM_FWD, GEMM_FWD, EPI_BIAS, T_, 3 * D.h, D.h, xn1, param(l, VARUNA_P_WQKV), param(l, VARUNA_P_BQKV), nullptr, qkv, nullptr, nullptr))) return e;
    {
      Bracket br(S, st, VARUNA_K_ATTN_FWD, attn_flops_fwd(), 4.0 * D.E * sizeof(T));
      if ((e = AttnDispatch<T>::fwd(0, qkv, ctx, lse, D.b, D.s, D.a, D.d, D.causal, drop_args(DROP_SITE_ATTN, l, mb), st))) return e;
    }
    if ((e = gemm(VARUNA_K_GEMM_FWD, GEMM_FWD, EPI_BIAS_RES, T_, D.h, D.h, ctx, param(l, VARUNA_P_WO), param(l, VARUNA_P_BO), x, x1, nullptr, nullptr, drop_args(DROP_SITE_PROJ, l, mb)))) return e;
    {
      Bracket br(S, st, VARUNA_K_LN_FWD, 0, 2.0 * D.E * sizeof(T));
      if ((e = launch_layernorm_fwd<T>(x1, param(l, VARUNA_P_LN2_G), param(l, VARUNA_P_LN2_B), xn2, stats2, T_, D.h, D.eps, st))) return e;
    }
    if ((e = gemm(VARUNA_K_GEMM_FWD, GEMM_FWD, EPI_BIAS_GELU, T_, D.f, D.h, xn2, param(l, VARUNA_P_W1), param(l, VARUNA_P_B1), nullptr, g, save ? u : nullptr, nullptr))) return e;
    if (skip_mlp2) return hipSuccess;
    return gemm(VARUNA_K_GEMM_FWD, GEMM_FWD, EPI_BIAS_RES, T_, D.h, D.f, g, param(l, VARUNA_P_W2), param(l, VARUNA_P_B2), x1, y, nullptr, nullptr, drop_args(DROP_SITE_MLP, l, mb));
  }

  // Runs `launch(stream, partial scratch)` beside the GEMM chain when the caller has handed over a
  // side stream: everything the launch reads is complete at this point of the caller's stream,
  // and nothing on that stream depends on its result before the next join_side().
  template <typename F>
  hipError_t on_side(int cls, double bytes, F&& launch) {
    if (S->prof_on || S->side == nullptr) {  // per-kernel timing wants everything on one stream
      Bracket br(S, st, cls, 0, bytes);
      return launch(st, wsp<float>(S->ws.partial));
    }
    hipError_t e;
    if ((e = hipEventRecord(S->ev_fork, st))) return e;
    if ((e = hipStreamWaitEvent(S->side, S->ev_fork, 0))) return e;
    S->side_used = true;
    return launch(S->side, wsp<float>(S->ws.partial_side));
  }
  hipError_t colsum(const T* a, float* out, int64_t n) {
    return on_side(VARUNA_K_COLREDUCE, (double)D.T * n * sizeof(T),
                   [&](hipStream_t s, float* partial) { return launch_colsum<T>(a, out, partial, D.T, n, s); });
  }
  // gamma / beta gradients of one LayerNorm (reads dy, x, statistics)
  hipError_t ln_params(const T* dyn, const T* x, const float* stats, float* dgamma, float* dbeta) {
    return on_side(VARUNA_K_COLREDUCE, 2.0 * D.E * sizeof(T), [&](hipStream_t s, float* partial) {
      return launch_layernorm_bwd_params<T>(dyn, x, stats, dgamma, dbeta, partial, D.T, D.h, s);
    });
  }

  // The caller's stream waits for everything forked since the last join.
  hipError_t join_side() {
    if (!S->side_used) return hipSuccess;
    S->side_used = false;
    hipError_t e;
    if ((e = hipEventRecord(S->ev_join, S->side))) return e;
    return hipStreamWaitEvent(st, S->ev_join, 0);
  }

  // One layer backward for ring slot rs.  x: the layer's input; the gradient of its output
  // already sits in slot rs of the layer's dy ring; dx: gradient of its input.  The four
  // weight-gradient GEMMs are not issued here (see flush_wgrads): this pass leaves their
  // operands in the rings.
  hipError_t layer_backward(int l, int mb, const T* x, T* dx, const LayerArea& A, int rs) {
    hipError_t e;
    const int64_t T_ = D.T;
    const Workspace& W = S->ws;
    const T* qkv = wsp<T>(A.qkv); const T* ctx = wsp<T>(A.ctx) + (size_t)rs * D.E;
    const T* x1 = wsp<T>(A.x1); const T* u = wsp<T>(A.u);
    const float* stats1 = wsp<float>(A.stats1); const float* stats2 = wsp<float>(A.stats2);
    const float* lse = wsp<float>(A.lse);
    const T* dy = wsp<T>(A.dy) + (size_t)rs * D.E;
    T* du = wsp<T>(A.du) + (size_t)rs * D.F; T* dx1 = wsp<T>(A.dx1) + (size_t)rs * D.E;
    T* dqkv = wsp<T>(A.dqkv) + (size_t)rs * 3 * D.E;
    T* dxn = wsp<T>(W.dxn); T* dxn_b = wsp<T>(W.dxn_b); T* dctx = wsp<T>(W.dctx);
    float* delta = wsp<float>(W.delta);

    // With dropout the gradient entering a residual branch is the masked one (dyd, dx1d); the
    // residual path itself keeps dy / dx1.
    const bool dr = D.drop_thr != 0;
    const T* dyd = dy;
    if (dr) {
      T* o = wsp<T>(A.dyd) + (size_t)rs * D.E;
      Bracket br(S, st, VARUNA_K_OTHER, 0, 2.0 * D.E * sizeof(T));
      if ((e = launch_dropout_apply<T>(dy, o, T_, D.h, drop_args(DROP_SITE_MLP, l, mb), st))) return e;
      dyd = o;
    }
    // MLP2: du = (dyd W2) * GeLU'(u); db2 += colsum(dyd)
    if ((e = gemm(VARUNA_K_GEMM_DGRAD, GEMM_DGRAD, EPI_DGELU, T_, D.f, D.h, dyd, param(l, VARUNA_P_W2), nullptr, u, du, nullptr, nullptr))) return e;
    if ((e = colsum(dyd, grad(l, VARUNA_P_B2), D.h))) return e;
    // MLP1: dxn2 = du W1; db1 += colsum(du)
    if ((e = gemm(VARUNA_K_GEMM_DGRAD, GEMM_DGRAD, EPI_PLAIN, T_, D.h, D.f, du, param(l, VARUNA_P_W1), nullptr, nullptr, dxn, nullptr, nullptr))) return e;
    if ((e = colsum(du, grad(l, VARUNA_P_B1), D.f))) return e;
    // LN2: dx1 = dy + LN'(dxn2)
    {
      Bracket br(S, st, VARUNA_K_LN_BWD, 0, 4.0 * D.E * sizeof(T));
      if ((e = launch_layernorm_bwd_dx<T>(dxn, x1, stats2, param(l, VARUNA_P_LN2_G), dy, dx1, T_, D.h, st))) return e;
    }
    if ((e = ln_params(dxn, x1, stats2, grad(l, VARUNA_P_LN2_G), grad(l, VARUNA_P_LN2_B)))) return e;
    const T* dx1d = dx1;
    if (dr) {
      T* o = wsp<T>(A.dx1d) + (size_t)rs * D.E;
      Bracket br(S, st, VARUNA_K_OTHER, 0, 2.0 * D.E * sizeof(T));
      if ((e = launch_dropout_apply<T>(dx1, o, T_, D.h, drop_args(DROP_SITE_PROJ, l, mb), st))) return e;
      dx1d = o;
    }
    // proj: dctx = dx1d Wo; dbo += colsum(dx1d)
    if ((e = gemm(VARUNA_K_GEMM_DGRAD, GEMM_DGRAD, EPI_PLAIN, T_, D.h, D.h, dx1d, param(l, VARUNA_P_WO), nullptr, nullptr, dctx, nullptr, nullptr))) return e;
    if ((e = colsum(dx1d, grad(l, VARUNA_P_BO), D.h))) return e;
    // attention
    {
      Bracket br(S, st, VARUNA_K_ATTN_BWD, 2.5 * attn_flops_fwd(), 9.0 * D.E * sizeof(T));
      if ((e = AttnDispatch<T>::bwd(0, qkv, ctx, lse, dctx, dqkv, delta, D.b, D.s, D.a, D.d, D.causal, drop_args(DROP_SITE_ATTN, l, mb), st))) return e;
    }
    // QKV: dxn1 = dqkv Wqkv; dbqkv += colsum(dqkv)
    if ((e = gemm(VARUNA_K_GEMM_DGRAD, GEMM_DGRAD, EPI_PLAIN, T_, D.h, 3 * D.h, dqkv, param(l, VARUNA_P_WQKV), nullptr, nullptr, dxn_b, nullptr, nullptr))) return e;
    if ((e = colsum(dqkv, grad(l, VARUNA_P_BQKV), 3 * D.h))) return e;
    // LN1: dx = dx1 + LN'(dxn1)
    {
      Bracket br(S, st, VARUNA_K_LN_BWD, 0, 4.0 * D.E * sizeof(T));
      if ((e = launch_layernorm_bwd_dx<T>(dxn_b, x, stats1, param(l, VARUNA_P_LN1_G), dx1, dx, T_, D.h, st))) return e;
    }
    if ((e = ln_params(dxn_b, x, stats1, grad(l, VARUNA_P_LN1_G), grad(l, VARUNA_P_LN1_B)))) return e;
    // the next layer down rewrites dxn / dxn_b and this layer's rings: the side stream's reads come first
    return join_side();
  }

  // One weight gradient dW[M,N] += A^T B over K tokens.  bf16 shapes with too few output
  // tiles for the chip cut the reduction into splits whose partial results are added to dW in
  // a fixed order (deterministic).
  hipError_t wgrad(int64_t M, int64_t N, int64_t K, const T* a, const T* b, float* dw) {
    if constexpr (std::is_same<T, bf16>::value) {
      const int splits = dg_wgrad_splits(M, N, K);
      if (splits > 1 && (size_t)splits * M * N * sizeof(float) <= S->ws.splitk_size && aligned16(a) && aligned16(b) && aligned16(dw)) {
        float* part = wsp<float>(S->ws.splitk);
        hipError_t e;
        {
          EpiArgs<T> ea{nullptr, nullptr, nullptr, nullptr, part, N, DropArgs{}, M * N};
          Bracket br(S, st, VARUNA_K_GEMM_WGRAD, 2.0 * M * N * K, (double)(M * K + N * K) * sizeof(T) + (double)M * N * 4.0 * splits);
          if ((e = GemmDispatch<T>::run(GEMM_WGRAD, EPI_STORE_F32, 0, M, N, K, a, b, ea, st, splits))) return e;
        }
        Bracket br(S, st, VARUNA_K_OTHER, 0, (double)M * N * 4.0 * (splits + 2));
        return launch_splitk_reduce(part, splits, M * N, dw, st);
      }
    }
    return gemm(VARUNA_K_GEMM_WGRAD, GEMM_WGRAD, EPI_ACCUM_F32, M, N, K, a, b, nullptr, nullptr, nullptr, nullptr, dw);
  }

  // dW += dY^T X for the four matrices of every layer, over the `cnt` micro-batches whose
  // operands sit in ring slots 0..cnt-1: the slots are stacked along the token dimension,
  // so each is ONE GEMM with reduction length cnt*T and one fp32 read-modify-write of dW.
  hipError_t flush_wgrads(int cnt) {
    hipError_t e;
    const int64_t K = (int64_t)cnt * D.T;
    for (int l = D.L - 1; l >= 0; --l) {
      const LayerArea& A = S->ws.layer[l];
      if ((e = wgrad(D.h, D.f, K, wsp<T>(A.dyd), wsp<T>(A.g), grad(l, VARUNA_P_W2)))) return e;
      if ((e = wgrad(D.f, D.h, K, wsp<T>(A.du), wsp<T>(A.xn2), grad(l, VARUNA_P_W1)))) return e;
      if ((e = wgrad(D.h, D.h, K, wsp<T>(A.dx1d), wsp<T>(A.ctx), grad(l, VARUNA_P_WO)))) return e;
      if ((e = wgrad(3 * D.h, D.h, K, wsp<T>(A.dqkv), wsp<T>(A.xn1), grad(l, VARUNA_P_WQKV)))) return e;
    }
    return hipSuccess;
  }

  T* slot(int mb) const { return reinterpret_cast<T*>(S->boundary) + (size_t)mb * D.E; }

  hipError_t store_boundary(int mb, const T* x_in) {
    if (x_in == slot(mb)) return hipSuccess;
    Bracket br(S, st, VARUNA_K_OTHER, 0, 2.0 * D.E * sizeof(T));
    return hipMemcpyAsync(slot(mb), x_in, (size_t)D.E * sizeof(T), hipMemcpyDeviceToDevice, st);
  }

  // Forward that keeps nothing but the boundary slot: every layer reuses the forward scratch.
  hipError_t forward(int mb, const T* x_in, T* y_out) {
    hipError_t e;
    if ((e = store_boundary(mb, x_in))) return e;
    const T* x = slot(mb);
    for (int l = 0; l < D.L; ++l) {
      T* y = (l == D.L - 1) ? y_out : wsp<T>(S->ws.ping[l & 1]);
      if ((e = layer_forward(l, mb, x, y, S->ws.fwd, 0, false, false))) return e;
      x = y;
    }
    return hipSuccess;
  }

  // Recompute from the boundary slot into the per-layer areas, ring slot rs.  With y_out
  // the stage output is produced too (the debug hook wants it; the backward pass does not).
  hipError_t recompute(int mb, T* y_out, int rs) {
    hipError_t e;
    const T* x = slot(mb);
    for (int l = 0; l < D.L; ++l) {
      const bool last = (l == D.L - 1);
      T* y = last ? y_out : wsp<T>(S->ws.layer[l].y);
      if ((e = layer_forward(l, mb, x, y, S->ws.layer[l], rs, true, last && y_out == nullptr))) return e;
      x = y;
    }
    return hipSuccess;
  }

  // Backward of micro-batch mb into ring slot `pending`; with recompute_first the internals
  // are first re-derived from the boundary slot, otherwise they must already sit there.
  hipError_t backward(int mb, const T* dy_in, T* dx_out, bool recompute_first) {
    hipError_t e;
    const int rs = S->pending;
    if (recompute_first && (e = recompute(mb, nullptr, rs))) return e;
    {  // the upstream gradient joins the top layer's dy ring
      Bracket br(S, st, VARUNA_K_OTHER, 0, 2.0 * D.E * sizeof(T));
      if ((e = hipMemcpyAsync(wsp<T>(S->ws.layer[D.L - 1].dy) + (size_t)rs * D.E, dy_in, (size_t)D.E * sizeof(T), hipMemcpyDeviceToDevice, st))) return e;
    }
    for (int l = D.L - 1; l >= 0; --l) {
      const T* x = (l == 0) ? slot(mb) : wsp<T>(S->ws.layer[l - 1].y);
      T* dx = (l == 0) ? dx_out : wsp<T>(S->ws.layer[l - 1].dy) + (size_t)rs * D.E;
      if ((e = layer_backward(l, mb, x, dx, S->ws.layer[l], rs))) return e;
    }
    if ((e = join_side())) return e;   // the bias gradients are complete when this call's work is
    if (++S->pending == D.G) {
      if ((e = flush_wgrads(S->pending))) return e;
      S->pending = 0;
    }
    return hipSuccess;
  }

  hipError_t flush() {
    if (S->pending == 0) return hipSuccess;
    hipError_t e = flush_wgrads(S->pending);
    S->pending = 0;
    return e;
  }
};

varuna_status_t check_call(varuna_stage_t* st, int32_t mb, const void* in, void* out) {
  if (!st) return fail(VARUNA_EINVAL, "stage handle is NULL");
  if (mb < 0 || mb >= st->D.M) return fail(VARUNA_EINVAL, "micro-batch slot %d out of range [0, %d)", mb, st->D.M);
  if (!in || !out) return fail(VARUNA_EINVAL, "NULL tensor pointer");
  return VARUNA_OK;
}

varuna_status_t hip_result(hipError_t e, const char* what) {
  if (e == hipSuccess) return VARUNA_OK;
  if (e == hipErrorInvalidConfiguration) return fail(VARUNA_EUNSUPPORTED, "%s: kernel configuration does not support this shape", what);
  return fail(VARUNA_EHIP, "%s: %s", what, hipGetErrorString(e));
}

// Forward through the per-layer areas (the recompute pass with the stage output produced).
varuna_status_t keep_forward(varuna_stage_t* st, int32_t mb, const void* x_in, void* y_out, void* hip_stream, const char* what) {
  varuna_status_t rc = check_call(st, mb, x_in, y_out);
  if (rc) return rc;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipError_t e;
  st->kept_mb = -1;
  if (st->D.dtype == VARUNA_F32) {
    StageOps<float> ops(st, s);
    e = ops.store_boundary(mb, static_cast<const float*>(x_in));
    if (e == hipSuccess) e = ops.recompute(mb, static_cast<float*>(y_out), st->pending);
  } else {
    StageOps<bf16> ops(st, s);
    e = ops.store_boundary(mb, static_cast<const bf16*>(x_in));
    if (e == hipSuccess) e = ops.recompute(mb, static_cast<bf16*>(y_out), st->pending);
  }
  if ((rc = hip_result(e, what))) return rc;
  st->forwarded[mb] = 1;
  return VARUNA_OK;
}

}  // namespace

// ============================================================================
// C ABI
// ============================================================================
extern "C" {

const char* varuna_last_error(void) { return g_err; }

varuna_status_t varuna_stage_query_sizes(const varuna_stage_config_t* cfg, size_t* param_bytes, size_t* grad_bytes,
                                         size_t* boundary_bytes, size_t* workspace_bytes) {
  Dims D;
  varuna_status_t rc = make_dims(cfg, &D);
  if (rc) return rc;
  ParamOffsets po = param_offsets(D);
  if (param_bytes) *param_bytes = po.per_layer * D.L * D.es;
  if (grad_bytes) *grad_bytes = po.per_layer * D.L * sizeof(float);
  if (boundary_bytes) *boundary_bytes = (size_t)D.M * D.E * D.es;
  if (workspace_bytes) *workspace_bytes = carve(D).total;
  return VARUNA_OK;
}

varuna_status_t varuna_stage_param_offset(const varuna_stage_config_t* cfg, int32_t layer, int32_t which,
                                          size_t* offset_elems, size_t* n_elems) {
  Dims D;
  varuna_status_t rc = make_dims(cfg, &D);
  if (rc) return rc;
  if (layer < 0 || layer >= D.L) return fail(VARUNA_EINVAL, "layer %d out of range [0, %d)", layer, D.L);
  if (which < 0 || which >= VARUNA_PARAMS_PER_LAYER) return fail(VARUNA_EINVAL, "parameter index %d out of range", which);
  ParamOffsets po = param_offsets(D);
  if (offset_elems) *offset_elems = (size_t)layer * po.per_layer + po.off[which];
  if (n_elems) *n_elems = po.n[which];
  return VARUNA_OK;
}

varuna_status_t varuna_stage_create(const varuna_stage_config_t* cfg, const void* params, void* grads_f32,
                                    void* boundary, void* workspace, varuna_stage_t** out) {
  if (!out) return fail(VARUNA_EINVAL, "out handle pointer is NULL");
  *out = nullptr;
  Dims D;
  varuna_status_t rc = make_dims(cfg, &D);
  if (rc) return rc;
  if (!params || !grads_f32 || !boundary || !workspace) return fail(VARUNA_EINVAL, "NULL device buffer");
  const void* ptrs[4] = {params, grads_f32, boundary, workspace};
  for (const void* p : ptrs)
    if (reinterpret_cast<uintptr_t>(p) % 256 != 0) return fail(VARUNA_EINVAL, "device buffers must be 256-byte aligned");
  varuna_stage* st = new (std::nothrow) varuna_stage();
  if (!st) return fail(VARUNA_ENOMEM, "out of host memory");
  st->D = D;
  st->po = param_offsets(D);
  st->ws = carve(D);
  st->params = static_cast<const char*>(params);
  st->grads = static_cast<float*>(grads_f32);
  st->boundary = static_cast<char*>(boundary);
  st->work = static_cast<char*>(workspace);
  st->forwarded.assign(D.M, 0);
  *out = st;
  return VARUNA_OK;
}

varuna_status_t varuna_stage_destroy(varuna_stage_t* st) {
  if (!st) return fail(VARUNA_EINVAL, "stage handle is NULL");
  for (hipEvent_t e : st->ev) (void)hipEventDestroy(e);
  if (st->ev_fork) (void)hipEventDestroy(st->ev_fork);   // the side stream itself is the caller's
  if (st->ev_join) (void)hipEventDestroy(st->ev_join);
  delete st;
  return VARUNA_OK;
}

varuna_status_t varuna_stage_set_side_stream(varuna_stage_t* st, void* side_stream) {
  if (!st) return fail(VARUNA_EINVAL, "stage handle is NULL");
  if (side_stream && !st->ev_fork) {
    HIP_TRY(hipEventCreateWithFlags(&st->ev_fork, hipEventDisableTiming));
    HIP_TRY(hipEventCreateWithFlags(&st->ev_join, hipEventDisableTiming));
  }
  st->side = static_cast<hipStream_t>(side_stream);
  return VARUNA_OK;
}

varuna_status_t varuna_stage_forward(varuna_stage_t* st, int32_t mb, const void* x_in, void* y_out, void* hip_stream) {
  varuna_status_t rc = check_call(st, mb, x_in, y_out);
  if (rc) return rc;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipError_t e = (st->D.dtype == VARUNA_F32)
                     ? StageOps<float>(st, s).forward(mb, static_cast<const float*>(x_in), static_cast<float*>(y_out))
                     : StageOps<bf16>(st, s).forward(mb, static_cast<const bf16*>(x_in), static_cast<bf16*>(y_out));
  if ((rc = hip_result(e, "varuna_stage_forward"))) return rc;
  st->forwarded[mb] = 1;
  return VARUNA_OK;
}

varuna_status_t varuna_stage_debug_forward_save(varuna_stage_t* st, int32_t mb, const void* x_in, void* y_out, void* hip_stream) {
  return keep_forward(st, mb, x_in, y_out, hip_stream, "varuna_stage_debug_forward_save");
}

varuna_status_t varuna_stage_debug_saved_region(const varuna_stage_t* st, size_t* offset_bytes, size_t* n_bytes) {
  if (!st) return fail(VARUNA_EINVAL, "stage handle is NULL");
  if (offset_bytes) *offset_bytes = st->ws.saved_begin;
  if (n_bytes) *n_bytes = st->ws.saved_end - st->ws.saved_begin;
  return VARUNA_OK;
}

varuna_status_t varuna_stage_backward_recompute(varuna_stage_t* st, int32_t mb, const void* dy_in, void* dx_out, void* hip_stream) {
  varuna_status_t rc = check_call(st, mb, dy_in, dx_out);
  if (rc) return rc;
  if (!st->forwarded[mb]) return fail(VARUNA_ESTATE, "backward_recompute(%d) without a forward of that slot", mb);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipError_t e = (st->D.dtype == VARUNA_F32)
                     ? StageOps<float>(st, s).backward(mb, static_cast<const float*>(dy_in), static_cast<float*>(dx_out), true)
                     : StageOps<bf16>(st, s).backward(mb, static_cast<const bf16*>(dy_in), static_cast<bf16*>(dx_out), true);
  st->kept_mb = -1;  // the recompute pass overwrote the layer areas
  if ((rc = hip_result(e, "varuna_stage_backward_recompute"))) return rc;
  st->forwarded[mb] = 0;
  return VARUNA_OK;
}

varuna_status_t varuna_stage_forward_keep(varuna_stage_t* st, int32_t mb, const void* x_in, void* y_out, void* hip_stream) {
  varuna_status_t rc = keep_forward(st, mb, x_in, y_out, hip_stream, "varuna_stage_forward_keep");
  if (rc) return rc;
  st->kept_mb = mb;
  st->kept_slot = st->pending;
  return VARUNA_OK;
}

varuna_status_t varuna_stage_backward_stored(varuna_stage_t* st, int32_t mb, const void* dy_in, void* dx_out, void* hip_stream) {
  varuna_status_t rc = check_call(st, mb, dy_in, dx_out);
  if (rc) return rc;
  if (st->kept_mb != mb || st->kept_slot != st->pending || !st->forwarded[mb])
    return fail(VARUNA_ESTATE, "backward_stored(%d): the workspace does not hold that micro-batch's activations "
                "(needs varuna_stage_forward_keep(%d) directly before)", mb, mb);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipError_t e = (st->D.dtype == VARUNA_F32)
                     ? StageOps<float>(st, s).backward(mb, static_cast<const float*>(dy_in), static_cast<float*>(dx_out), false)
                     : StageOps<bf16>(st, s).backward(mb, static_cast<const bf16*>(dy_in), static_cast<bf16*>(dx_out), false);
  st->kept_mb = -1;
  if ((rc = hip_result(e, "varuna_stage_backward_stored"))) return rc;
  st->forwarded[mb] = 0;
  return VARUNA_OK;
}

varuna_status_t varuna_stage_grad_accum_reset(varuna_stage_t* st, void* hip_stream) {
  if (!st) return fail(VARUNA_EINVAL, "stage handle is NULL");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const size_t n = st->po.per_layer * st->D.L;
  st->pending = 0;  // operands gathered for a not yet issued weight-gradient group are dropped
  st->kept_mb = -1;
  Bracket br(st, s, VARUNA_K_OTHER, 0, 4.0 * n);
  hipLaunchKernelGGL(fill_zero_f32_kernel, dim3(2048), dim3(256), 0, s, st->grads, n);
  return hip_result(hipGetLastError(), "varuna_stage_grad_accum_reset");
}

varuna_status_t varuna_stage_grad_flush(varuna_stage_t* st, void* hip_stream) {
  if (!st) return fail(VARUNA_EINVAL, "stage handle is NULL");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipError_t e = (st->D.dtype == VARUNA_F32) ? StageOps<float>(st, s).flush() : StageOps<bf16>(st, s).flush();
  return hip_result(e, "varuna_stage_grad_flush");
}

varuna_status_t varuna_stage_set_dropout_seed(varuna_stage_t* st, uint64_t seed) {
  if (!st) return fail(VARUNA_EINVAL, "stage handle is NULL");
  for (char f : st->forwarded)
    if (f) return fail(VARUNA_ESTATE, "the dropout seed cannot change between a forward and its backward");
  st->seed = seed;
  st->kept_mb = -1;
  return VARUNA_OK;
}

varuna_status_t varuna_stage_grad_stats(varuna_stage_t* st, float* out2, void* hip_stream) {
  if (!st) return fail(VARUNA_EINVAL, "stage handle is NULL");
  if (!out2) return fail(VARUNA_EINVAL, "NULL output pointer");
  if (st->pending != 0)
    return fail(VARUNA_ESTATE, "%d micro-batches of weight gradients are gathered but not accumulated yet: call "
                "varuna_stage_grad_flush first", st->pending);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const size_t n = st->po.per_layer * st->D.L;
  Bracket br(st, s, VARUNA_K_OTHER, 0, 4.0 * n);
  return hip_result(launch_grad_stats(st->grads, n, reinterpret_cast<double*>(st->work + st->ws.stat_partial), out2, s),
                    "varuna_stage_grad_stats");
}

varuna_status_t varuna_stage_adam_step(varuna_stage_t* st, const varuna_adam_t* hp, void* params_out, float* master_f32,
                                       float* m_f32, float* v_f32, const float* skip_if_nonzero, void* hip_stream) {
  if (!st) return fail(VARUNA_EINVAL, "stage handle is NULL");
  if (!hp || !params_out || !master_f32 || !m_f32 || !v_f32) return fail(VARUNA_EINVAL, "NULL pointer");
  if (hp->step < 1) return fail(VARUNA_EINVAL, "Adam step number must be >= 1, got %d", hp->step);
  if (!(hp->beta1 >= 0.f && hp->beta1 < 1.f) || !(hp->beta2 >= 0.f && hp->beta2 < 1.f))
    return fail(VARUNA_EINVAL, "Adam betas must lie in [0, 1)");
  const void* ptrs[4] = {params_out, master_f32, m_f32, v_f32};
  for (const void* p : ptrs)
    if (reinterpret_cast<uintptr_t>(p) % 16 != 0) return fail(VARUNA_EINVAL, "optimizer buffers must be 16-byte aligned");
  if (st->pending != 0)
    return fail(VARUNA_ESTATE, "%d micro-batches of weight gradients are gathered but not accumulated yet: call "
                "varuna_stage_grad_flush first", st->pending);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const size_t n = st->po.per_layer * st->D.L;
  AdamArgs a{hp->lr, hp->beta1, hp->beta2, hp->eps, hp->weight_decay, hp->grad_scale,
             (float)(1.0 / (1.0 - pow((double)hp->beta1, (double)hp->step))),
             (float)(1.0 / (1.0 - pow((double)hp->beta2, (double)hp->step)))};
  Bracket br(st, s, VARUNA_K_OTHER, 0, (28.0 + st->D.es) * n);
  hipError_t e = (st->D.dtype == VARUNA_F32)
                     ? launch_adam<float>(st->grads, master_f32, m_f32, v_f32, static_cast<float*>(params_out), n, a, skip_if_nonzero, s)
                     : launch_adam<bf16>(st->grads, master_f32, m_f32, v_f32, static_cast<bf16*>(params_out), n, a, skip_if_nonzero, s);
  st->kept_mb = -1;  // the parameters changed: kept activations no longer belong to them
  return hip_result(e, "varuna_stage_adam_step");
}

varuna_status_t varuna_stage_profile_enable(varuna_stage_t* st, int32_t on) {
  if (!st) return fail(VARUNA_EINVAL, "stage handle is NULL");
  if (on && st->ev.empty()) {
    st->ev.reserve(2 * kMaxEvents);
    for (int i = 0; i < 2 * kMaxEvents; ++i) {
      hipEvent_t e;
      HIP_TRY(hipEventCreate(&e));
      st->ev.push_back(e);
    }
  }
  st->prof_on = on != 0;
  return VARUNA_OK;
}

varuna_status_t varuna_stage_profile_collect(varuna_stage_t* st, double* ms, int64_t* launches, double* flops, double* bytes) {
  if (!st) return fail(VARUNA_EINVAL, "stage handle is NULL");
  for (int i = 0; i < VARUNA_K_COUNT; ++i) {
    if (ms) ms[i] = 0;
    if (launches) launches[i] = 0;
    if (flops) flops[i] = 0;
    if (bytes) bytes[i] = 0;
  }
  for (size_t i = 0; i < st->recs.size(); ++i) {
    HIP_TRY(hipEventSynchronize(st->ev[2 * i + 1]));
    float t = 0.f;
    HIP_TRY(hipEventElapsedTime(&t, st->ev[2 * i], st->ev[2 * i + 1]));
    const int c = st->recs[i].cls;
    if (ms) ms[c] += t;
    if (launches) launches[c] += 1;
    if (flops) flops[c] += st->recs[i].flops;
    if (bytes) bytes[c] += st->recs[i].bytes;
  }
  st->recs.clear();
  return VARUNA_OK;
}

// ---- single operations -------------------------------------------------------

varuna_status_t varuna_op_gemm(int32_t dtype, int32_t op, int32_t epi, int32_t variant, int64_t M, int64_t N, int64_t K,
                               const void* a, const void* b, const void* bias, const void* aux_in, void* out,
                               void* aux_out, void* hip_stream) {
  if (M < 1 || N < 1 || K < 1 || M > (1ll << 30) || N > (1ll << 30) || K > (1ll << 30)) return fail(VARUNA_EINVAL, "bad GEMM size");
  if (!a || !b || !out) return fail(VARUNA_EINVAL, "NULL operand");
  int mode;
  if (op == GEMM_FWD && epi >= 0 && epi <= 2) mode = epi;
  else if (op == GEMM_DGRAD && (epi == 0 || epi == 3)) mode = epi == 0 ? EPI_PLAIN : EPI_DGELU;
  else if (op == GEMM_WGRAD && epi == 0) mode = EPI_ACCUM_F32;
  else if (op == GEMM_WGRAD && epi == 4 && dtype == VARUNA_BF16 && variant >= 5) mode = EPI_PLAIN;  // tuning aid: no accumulate
  else return fail(VARUNA_EINVAL, "unknown op/epilogue combination %d/%d", op, epi);
  if (op == GEMM_FWD && !bias) return fail(VARUNA_EINVAL, "forward GEMM needs a bias");
  if ((mode == EPI_BIAS_RES || mode == EPI_DGELU) && !aux_in) return fail(VARUNA_EINVAL, "epilogue needs aux_in");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipError_t e;
  if (dtype == VARUNA_F32) {
    EpiArgs<float> ea{static_cast<const float*>(bias), static_cast<const float*>(aux_in), static_cast<float*>(out),
                      static_cast<float*>(aux_out), static_cast<float*>(out), N};
    e = GemmDispatch<float>::run(op, mode, variant, M, N, K, static_cast<const float*>(a), static_cast<const float*>(b), ea, s);
  } else if (dtype == VARUNA_BF16) {
    EpiArgs<bf16> ea{static_cast<const bf16*>(bias), static_cast<const bf16*>(aux_in), static_cast<bf16*>(out),
                     static_cast<bf16*>(aux_out), static_cast<float*>(out), N};
    e = GemmDispatch<bf16>::run(op, mode, variant, M, N, K, static_cast<const bf16*>(a), static_cast<const bf16*>(b), ea, s);
  } else {
    return fail(VARUNA_EINVAL, "unknown dtype %d", dtype);
  }
  return hip_result(e, "varuna_op_gemm");
}

varuna_status_t varuna_op_layernorm_fwd(int32_t dtype, int64_t rows, int64_t h, float eps, const void* x, const void* gamma,
                                        const void* beta, void* y, float* stats_f32, void* hip_stream) {
  if (rows < 1 || h < 1 || h > (1 << 20) || !x || !gamma || !beta || !y) return fail(VARUNA_EINVAL, "bad layernorm arguments");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipError_t e;
  if (dtype == VARUNA_F32)
    e = launch_layernorm_fwd<float>(static_cast<const float*>(x), static_cast<const float*>(gamma), static_cast<const float*>(beta), static_cast<float*>(y), stats_f32, rows, (int)h, eps, s);
  else if (dtype == VARUNA_BF16)
    e = launch_layernorm_fwd<bf16>(static_cast<const bf16*>(x), static_cast<const bf16*>(gamma), static_cast<const bf16*>(beta), static_cast<bf16*>(y), stats_f32, rows, (int)h, eps, s);
  else return fail(VARUNA_EINVAL, "unknown dtype %d", dtype);
  return hip_result(e, "varuna_op_layernorm_fwd");
}

varuna_status_t varuna_op_layernorm_bwd(int32_t dtype, int64_t rows, int64_t h, const void* dy, const void* x,
                                        const float* stats_f32, const void* gamma, const void* res, void* dx,
                                        float* dgamma_f32, float* dbeta_f32, float* partial_f32, void* hip_stream) {
  if (rows < 1 || h < 1 || h > (1 << 20) || !dy || !x || !stats_f32 || !gamma || !res || !dx || !dgamma_f32 || !dbeta_f32 || !partial_f32)
    return fail(VARUNA_EINVAL, "bad layernorm backward arguments");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipError_t e;
  if (dtype == VARUNA_F32)
    e = launch_layernorm_bwd<float>(static_cast<const float*>(dy), static_cast<const float*>(x), stats_f32, static_cast<const float*>(gamma), static_cast<const float*>(res), static_cast<float*>(dx), dgamma_f32, dbeta_f32, partial_f32, rows, (int)h, s);
  else if (dtype == VARUNA_BF16)
    e = launch_layernorm_bwd<bf16>(static_cast<const bf16*>(dy), static_cast<const bf16*>(x), stats_f32, static_cast<const bf16*>(gamma), static_cast<const bf16*>(res), static_cast<bf16*>(dx), dgamma_f32, dbeta_f32, partial_f32, rows, (int)h, s);
  else return fail(VARUNA_EINVAL, "unknown dtype %d", dtype);
  return hip_result(e, "varuna_op_layernorm_bwd");
}

size_t varuna_op_colreduce_scratch_bytes(int64_t rows, int64_t n) {
  if (rows < 1 || n < 1) return 0;
  return (size_t)colreduce_chunks(rows) * (size_t)n * sizeof(float);
}

varuna_status_t varuna_op_colsum(int32_t dtype, int64_t rows, int64_t n, const void* a, float* out_f32, float* partial_f32, void* hip_stream) {
  if (rows < 1 || n < 1 || !a || !out_f32 || !partial_f32) return fail(VARUNA_EINVAL, "bad colsum arguments");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipError_t e;
  if (dtype == VARUNA_F32) e = launch_colsum<float>(static_cast<const float*>(a), out_f32, partial_f32, rows, n, s);
  else if (dtype == VARUNA_BF16) e = launch_colsum<bf16>(static_cast<const bf16*>(a), out_f32, partial_f32, rows, n, s);
  else return fail(VARUNA_EINVAL, "unknown dtype %d", dtype);
  return hip_result(e, "varuna_op_colsum");
}

// ---- column sums with no allocation anywhere ------------------------------------------
// The stage-1 partial sums of varuna_op_colsum_static live in this file-scope device array
// (every GPU the library runs on holds its own copy until the process ends).  In host code
// the array's name is only a stand-in; the device address comes from hipGetSymbolAddress,
// once per device, and is what the kernels receive.
constexpr size_t kStaticScratchFloats = (size_t)1 << 20;   // 4 MiB
static __device__ __align__(256) float scratch[kStaticScratchFloats];
constexpr int kMaxDevices = 64;
static float* g_scratch_ptr[kMaxDevices] = {};
static std::mutex g_scratch_mu;

static varuna_status_t static_scratch(float** out) {
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(VARUNA_EUNSUPPORTED, "device index %d out of range", dev);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(VARUNA_EHIP, "hipGetSymbolAddress returned a null address");
    g_scratch_ptr[dev] = static_cast<float*>(p);
  }
  *out = g_scratch_ptr[dev];
  return VARUNA_OK;
}

size_t varuna_op_colsum_static_max_bytes(void) { return kStaticScratchFloats * sizeof(float); }

varuna_status_t varuna_op_colsum_static(int32_t dtype, int64_t rows, int64_t n, const void* a, float* out_f32, void* hip_stream) {
  if (rows < 1 || n < 1 || !a || !out_f32) return fail(VARUNA_EINVAL, "bad colsum arguments");
  if (dtype != VARUNA_F32 && dtype != VARUNA_BF16) return fail(VARUNA_EINVAL, "unknown dtype %d", dtype);
  const size_t need = varuna_op_colreduce_scratch_bytes(rows, n);
  if (rows > (1ll << 40) || n > (1ll << 40) || need > kStaticScratchFloats * sizeof(float))
    return fail(VARUNA_EUNSUPPORTED, "colsum of [%lld, %lld] needs %zu bytes of partial sums; the built-in scratch holds %zu",
                (long long)rows, (long long)n, need, kStaticScratchFloats * sizeof(float));
  float* partial = nullptr;
  varuna_status_t rc = static_scratch(&partial);
  if (rc) return rc;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipError_t e;
  // stage 1 overwrites every partial that stage 2 reads, so nothing has to be cleared
  if (dtype == VARUNA_F32) e = launch_colsum<float>(static_cast<const float*>(a), out_f32, partial, rows, n, s);
  else e = launch_colsum<bf16>(static_cast<const bf16*>(a), out_f32, partial, rows, n, s);
  return hip_result(e, "varuna_op_colsum_static");
}

varuna_status_t varuna_debug_set_gemm_kernels(int32_t fwd256, int32_t dgrad256, int32_t wgrad256, int32_t fwd128,
                                              int32_t dgrad128, int32_t wgrad128) {
  const int32_t v[6] = {fwd256, dgrad256, wgrad256, fwd128, dgrad128, wgrad128};
  GemmTile t;
  for (int i = 0; i < 6; ++i) {
    if (v[i] == 0) continue;
    if (!dg_variant_tile(v[i], &t) || t.bm != t.bn || t.bm != (i < 3 ? 256 : 128))
      return fail(VARUNA_EINVAL, "kernel configuration %d does not exist or has another tile size", v[i]);
  }
  const DgFlavours d;
  DgFlavours& f = dg_flavours();
  f.fwd256 = fwd256 ? fwd256 : d.fwd256; f.bwd256 = dgrad256 ? dgrad256 : d.bwd256; f.wgrad256 = wgrad256 ? wgrad256 : d.wgrad256;
  f.fwd128 = fwd128 ? fwd128 : d.fwd128; f.dgrad128 = dgrad128 ? dgrad128 : d.dgrad128; f.wgrad128 = wgrad128 ? wgrad128 : d.wgrad128;
  f.pair128 = fwd128 == 0 && dgrad128 == 0;   // naming a 128x128 configuration also turns the merging of tile pairs off
  return VARUNA_OK;
}

int32_t varuna_debug_gemm_choice(int32_t op, int64_t M, int64_t N, int64_t K) {
  if (op < GEMM_FWD || op > GEMM_WGRAD || M < 1 || N < 1 || K < 1) return -2;
  const int64_t lda = (op == GEMM_WGRAD) ? M : K, ldb = (op == GEMM_FWD) ? K : N;
  const int v = (N % 8 == 0) ? dg_pick(op, M, N, K, lda, ldb) : 0;
  return v == 0 ? -1 : v;
}

varuna_status_t varuna_probe_mfma_rate(const void* operands, int64_t n_elems, int32_t waves_per_simd, int32_t pattern,
                                       int32_t iters, float* sink, double* flops, void* hip_stream) {
  if (pattern < 0 || pattern > 7) return fail(VARUNA_EINVAL, "pattern must be in [0, 7]");
  if (!operands || !sink) return fail(VARUNA_EINVAL, "NULL pointer");
  if (n_elems < 8 || n_elems > (1ll << 31) || n_elems % 8 != 0) return fail(VARUNA_EINVAL, "n_elems must be a multiple of 8 in [8, 2^31]");
  if (reinterpret_cast<uintptr_t>(operands) % 16 != 0) return fail(VARUNA_EINVAL, "operands must be 16-byte aligned");
  if (waves_per_simd < 1 || waves_per_simd > 2) return fail(VARUNA_EINVAL, "waves_per_simd must be 1 or 2");
  if (iters < 4 || iters % 4 != 0 || iters > (1 << 24)) return fail(VARUNA_EINVAL, "iters must be a multiple of 4 in [4, 2^24]");
  int dev = 0, cus = 0;
  HIP_TRY(hipGetDevice(&dev));
  HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
  if (cus < 1 || cus > 1024) return fail(VARUNA_EHIP, "implausible compute-unit count %d", cus);
  const unsigned nwg = (unsigned)(cus * waves_per_simd);   // 4 waves per workgroup: one per SIMD
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const bf16x8* src = static_cast<const bf16x8*>(operands);
  const uint32_t nv = (uint32_t)(n_elems / 8);
  switch (pattern) {
    case 0: hipLaunchKernelGGL(mfma_rate_kernel<0>, dim3(nwg), dim3(256), 0, s, src, nv, sink, (int)iters); break;
    case 1: hipLaunchKernelGGL(mfma_rate_kernel<1>, dim3(nwg), dim3(256), 0, s, src, nv, sink, (int)iters); break;
    case 2: hipLaunchKernelGGL(mfma_rate_kernel<2>, dim3(nwg), dim3(256), 0, s, src, nv, sink, (int)iters); break;
    case 3: hipLaunchKernelGGL(mfma_rate_kernel<3>, dim3(nwg), dim3(256), 0, s, src, nv, sink, (int)iters); break;
    case 4: hipLaunchKernelGGL(mfma_rate_kernel<4>, dim3(nwg), dim3(256), 0, s, src, nv, sink, (int)iters); break;
    case 5: hipLaunchKernelGGL(mfma_rate_kernel<5>, dim3(nwg), dim3(256), 0, s, src, nv, sink, (int)iters); break;
    case 6: hipLaunchKernelGGL(mfma_rate_kernel<6>, dim3(nwg), dim3(256), 0, s, src, nv, sink, (int)iters); break;
    default: hipLaunchKernelGGL(mfma_rate_kernel<7>, dim3(nwg), dim3(256), 0, s, src, nv, sink, (int)iters); break;
  }
  if (flops) *flops = (double)nwg * 4.0 * (double)iters * 8.0 * (2.0 * 32 * 32 * 16);
  return hip_result(hipGetLastError(), "varuna_probe_mfma_rate");
}

static varuna_status_t check_attn(int32_t b, int32_t s, int32_t heads, int32_t d) {
  if (b < 1 || s < 1 || heads < 1 || d < 1) return fail(VARUNA_EINVAL, "non-positive attention dimension");
  if (s > ATS_MAX_S || d > ATS_MAX_D) return fail(VARUNA_EUNSUPPORTED, "attention shape exceeds supported maximum");
  if (b > 65535 || heads > 65535) return fail(VARUNA_EUNSUPPORTED, "too many batch elements or heads");
  return VARUNA_OK;
}

varuna_status_t varuna_op_attention_fwd(int32_t dtype, int32_t variant, int32_t b, int32_t s, int32_t heads, int32_t d,
                                        int32_t causal, const void* qkv, void* ctx, float* lse_f32, void* hip_stream) {
  varuna_status_t rc = check_attn(b, s, heads, d);
  if (rc) return rc;
  if (!qkv || !ctx) return fail(VARUNA_EINVAL, "NULL tensor pointer");
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  hipError_t e;
  if (dtype == VARUNA_F32) e = AttnDispatch<float>::fwd(variant, static_cast<const float*>(qkv), static_cast<float*>(ctx), lse_f32, b, s, heads, d, causal, DropArgs{}, st);
  else if (dtype == VARUNA_BF16) e = AttnDispatch<bf16>::fwd(variant, static_cast<const bf16*>(qkv), static_cast<bf16*>(ctx), lse_f32, b, s, heads, d, causal, DropArgs{}, st);
  else return fail(VARUNA_EINVAL, "unknown dtype %d", dtype);
  return hip_result(e, "varuna_op_attention_fwd");
}

varuna_status_t varuna_op_attention_bwd(int32_t dtype, int32_t variant, int32_t b, int32_t s, int32_t heads, int32_t d,
                                        int32_t causal, const void* qkv, const void* ctx, const float* lse_f32,
                                        const void* dctx, void* dqkv, float* delta_f32, void* hip_stream) {
  varuna_status_t rc = check_attn(b, s, heads, d);
  if (rc) return rc;
  if (!qkv || !ctx || !lse_f32 || !dctx || !dqkv || !delta_f32) return fail(VARUNA_EINVAL, "NULL tensor pointer");
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  hipError_t e;
  if (dtype == VARUNA_F32) e = AttnDispatch<float>::bwd(variant, static_cast<const float*>(qkv), static_cast<const float*>(ctx), lse_f32, static_cast<const float*>(dctx), static_cast<float*>(dqkv), delta_f32, b, s, heads, d, causal, DropArgs{}, st);
  else if (dtype == VARUNA_BF16) e = AttnDispatch<bf16>::bwd(variant, static_cast<const bf16*>(qkv), static_cast<const bf16*>(ctx), lse_f32, static_cast<const bf16*>(dctx), static_cast<bf16*>(dqkv), delta_f32, b, s, heads, d, causal, DropArgs{}, st);
  else return fail(VARUNA_EINVAL, "unknown dtype %d", dtype);
  return hip_result(e, "varuna_op_attention_bwd");
}

}  // extern "C"
