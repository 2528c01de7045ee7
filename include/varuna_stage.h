/*
 * varuna_stage.h -- C ABI of the MI355X (gfx950) pipeline-stage compute library.
 *
 * One pipeline stage's micro-batched training step for a GPT-style transformer:
 * forward for each micro-batch keeping only the stage-input ("boundary")
 * activation; backward first recomputes the stage's internal activations from
 * that stored tensor, then produces the input gradient and the parameter
 * gradients, which accumulate in fp32 over the micro-batches a GPU holds.
 * (Paper: Design Overview, "High-level architecture" -- stage k takes
 * activations from k-1 and gradients from k+1, and recomputes activations from
 * the stored input activation; Background, "Memory optimization" -- gradient
 * checkpointing, forward is about a third of the compute; Job Morphing,
 * "Correctness-preserving morphing" -- gradient accumulation within a GPU.)
 *
 * Conventions
 *   - Every pointer marked "device" is GPU memory owned by the caller (the
 *     caller allocates, e.g. through PyTorch); it must stay valid until
 *     varuna_stage_destroy and be 256-byte aligned.  The library allocates no
 *     device memory in any call.
 *   - hip_stream is a hipStream_t passed as void* (NULL = the default stream).
 *     Every compute call only enqueues work and returns; nothing synchronises
 *     with the host.  All results of a call are ordered on hip_stream.  The
 *     library creates no stream: if the caller hands over a second one with
 *     varuna_stage_set_side_stream, the backward calls run their bias-gradient
 *     reductions there, forked from and joined back into hip_stream with events
 *     inside the call.  One handle is used from one stream at a time.
 *   - Activations are row-major [T, h], T = micro_batch * seq_len, row index
 *     = batch_index * seq_len + position.  dtype F32: all tensors fp32.
 *     dtype BF16: activations, parameters and dX are bf16; all accumulators,
 *     LayerNorm statistics, log-sum-exp and every parameter gradient are fp32.
 *   - Parameter buffer layout: layers back to back; inside a layer, in this
 *     order, each matrix row-major [out, in]:
 *        ln1_g[h] ln1_b[h] Wqkv[3h,h] bqkv[3h] Wo[h,h] bo[h]
 *        ln2_g[h] ln2_b[h] W1[f,h] b1[f] W2[h,f] b2[h]
 *     Rows of Wqkv are [Q | K | V] blocks of h rows; head j owns rows
 *     j*d .. (j+1)*d-1 of each block (d = h / heads).  The gradient buffer has
 *     the same element order, always fp32.  varuna_stage_param_offset reports
 *     the element offsets.
 *   - Every call returns a varuna_status_t; on failure varuna_last_error()
 *     returns a message (thread-local storage, valid until the next failing
 *     call on that thread).  Argument checks never touch the GPU.
 */
#ifndef VARUNA_STAGE_H
#define VARUNA_STAGE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct varuna_stage varuna_stage_t; /* opaque, host memory owned by the library */

typedef enum {
  VARUNA_OK = 0,
  VARUNA_EINVAL = -1,       /* bad argument or configuration */
  VARUNA_ESTATE = -2,       /* call order violated (e.g. backward before forward of that slot) */
  VARUNA_ENOMEM = -3,       /* host allocation failed */
  VARUNA_EHIP = -4,         /* a HIP runtime call or kernel launch failed */
  VARUNA_EUNSUPPORTED = -5  /* valid but not implemented for this shape */
} varuna_status_t;

typedef enum { VARUNA_F32 = 0, VARUNA_BF16 = 1 } varuna_dtype_t;

/* Number of parameter tensors per layer and their indices in the layout above. */
#define VARUNA_PARAMS_PER_LAYER 12
enum {
  VARUNA_P_LN1_G = 0, VARUNA_P_LN1_B, VARUNA_P_WQKV, VARUNA_P_BQKV, VARUNA_P_WO, VARUNA_P_BO,
  VARUNA_P_LN2_G, VARUNA_P_LN2_B, VARUNA_P_W1, VARUNA_P_B1, VARUNA_P_W2, VARUNA_P_B2
};

/* Plain data; the library copies it. */
typedef struct {
  int32_t n_layers;        /* L >= 1: transformer layers in this stage */
  int32_t hidden;          /* h */
  int32_t n_heads;         /* a, must divide h */
  int32_t seq_len;         /* s */
  int32_t micro_batch;     /* b: examples per micro-batch (the paper's m) */
  int32_t n_micro_batches; /* M: number of boundary slots (the paper's N_m) */
  int32_t mlp_hidden;      /* f; 0 means 4*h */
  int32_t causal;          /* 1: key index <= query index only; 0: bidirectional */
  int32_t dtype;           /* varuna_dtype_t */
  float ln_eps;            /* 0 means 1e-5 */
  int32_t wgrad_group;     /* G: weight-gradient GEMMs are issued once per G micro-batches with
                              reduction length G*T (0 or 1: after every micro-batch); on the bf16 path
                              G * T * mlp_hidden * 2 bytes must stay below 4 GiB (VARUNA_EUNSUPPORTED) */
  float dropout_p;         /* dropout probability in [0,1), applied as round(256 p)/256; 0: none.
                              See varuna_stage_set_dropout_seed. */
} varuna_stage_config_t;

/* Byte sizes of the four caller-allocated device buffers for this configuration.
 * boundary_bytes = M * T * h * sizeof(activation): one stage-input tensor per
 * micro-batch is all that forward keeps (Design Overview: 3.75 MB per example
 * for h=1920, s=1024 in 16-bit).  Any output pointer may be NULL. */
varuna_status_t varuna_stage_query_sizes(const varuna_stage_config_t* cfg, size_t* param_bytes,
                                         size_t* grad_bytes, size_t* boundary_bytes,
                                         size_t* workspace_bytes);

/* Element offset (from the start of the parameter buffer, equally of the
 * gradient buffer) and element count of parameter tensor `which` of `layer`. */
varuna_status_t varuna_stage_param_offset(const varuna_stage_config_t* cfg, int32_t layer,
                                          int32_t which, size_t* offset_elems, size_t* n_elems);

/* Creates a stage over caller-owned device buffers of the sizes reported by
 * varuna_stage_query_sizes.  params: read-only; grads_f32: accumulators, not
 * cleared here (call varuna_stage_grad_accum_reset); boundary: M slots [T,h];
 * workspace: scratch, contents undefined between calls.  Validates the
 * configuration without touching the GPU. */
varuna_status_t varuna_stage_create(const varuna_stage_config_t* cfg, const void* params /*device*/,
                                    void* grads_f32 /*device*/, void* boundary /*device*/,
                                    void* workspace /*device*/, varuna_stage_t** out);

/* Stage forward for micro-batch slot mb (0 <= mb < M): copies x_in [T,h] into
 * boundary slot mb (skipped when x_in is that slot), runs the L layers, writes
 * the stage output y_out [T,h].  Nothing else is kept. */
varuna_status_t varuna_stage_forward(varuna_stage_t* st, int32_t mb, const void* x_in /*device*/,
                                     void* y_out /*device*/, void* hip_stream);

/* Recompute + backward for slot mb: re-derives all internal activations from
 * boundary slot mb (bit-identical to what forward computed), then from the
 * upstream gradient dy_in [T,h] writes the input gradient dx_out [T,h] and adds
 * this micro-batch's parameter gradients into grads_f32 (the four matrix gradients
 * per layer possibly deferred, see varuna_stage_grad_flush).  Requires a forward of
 * slot mb since that slot was last consumed (else VARUNA_ESTATE).  Calls for
 * different slots may be interleaved with forwards in any order. */
varuna_status_t varuna_stage_backward_recompute(varuna_stage_t* st, int32_t mb,
                                                const void* dy_in /*device*/,
                                                void* dx_out /*device*/, void* hip_stream);

/* Last-stage variant (Design Overview, "Tuning pipeline efficiency": in the paper's schedule
 * the last pipeline stage runs the backward of a micro-batch straight after its forward and
 * therefore never recomputes).  varuna_stage_forward_keep is varuna_stage_forward that also
 * leaves every layer's internal activations of micro-batch mb in the workspace, in exactly
 * the form the recompute pass would leave them (same kernels, same launch geometry);
 * varuna_stage_backward_stored then runs the backward pass of backward_recompute on them
 * without recomputing.  The workspace holds the internals of ONE micro-batch: the pair must
 * be adjacent for a given mb -- any other forward_keep, backward_recompute or
 * grad_accum_reset in between invalidates them (plain varuna_stage_forward calls of other
 * slots do not) and backward_stored then returns VARUNA_ESTATE.  Arguments, layouts, the
 * accumulation into grads_f32 and the wgrad_group deferral are those of the two calls above;
 * outputs and gradients are bit-identical to the forward / backward_recompute pair. */
varuna_status_t varuna_stage_forward_keep(varuna_stage_t* st, int32_t mb, const void* x_in /*device*/,
                                          void* y_out /*device*/, void* hip_stream);
varuna_status_t varuna_stage_backward_stored(varuna_stage_t* st, int32_t mb,
                                             const void* dy_in /*device*/,
                                             void* dx_out /*device*/, void* hip_stream);

/* Optional second stream, created and owned by the caller (default priority; it must outlive
 * the handle or be replaced by NULL first).  The bias-gradient column sums of the backward
 * calls depend on nothing downstream of them and are bound by HBM, not by the matrix cores:
 * given a side stream they overlap the GEMM chain; every backward call waits for them before
 * it returns control of hip_stream's order, so the caller never has to synchronise with the
 * side stream itself.  NULL (the state after create): everything runs on hip_stream.
 * Results are bit-identical either way. */
varuna_status_t varuna_stage_set_side_stream(varuna_stage_t* st, void* side_stream);

/* Dropout (config.dropout_p > 0) acts on the attention probabilities and on the two residual
 * branches (attention-output projection and MLP output, after their bias, before the add).
 * The paper's implementation saves and restores the random-number state so that the
 * recompute pass reproduces the forward pass (Implementation, list of library functions);
 * here every mask is a pure function of (seed, micro-batch slot mb, layer, site, element),
 * so forward, recompute and backward regenerate it and nothing is stored.  Generator:
 * Philox4x32-10, key = (seed mod 2^32, seed div 2^32), counter = (row div 4, column div 4,
 * site + 256*layer, mb); the byte of element (row, column) is byte (column mod 4), little end
 * first, of output word (row mod 4); the element is kept iff byte >= thr = round(256 p) and
 * kept values are multiplied by 256 / (256 - thr).  Sites: 0 = attention probabilities
 * (row = (batch*heads + head)*seq_len + query, column = key), 1 = projection branch,
 * 2 = MLP branch (row = token, column = hidden index).
 * The seed is 0 after create; set a new one per mini-batch.  It must not change between a
 * forward and the backward of the same slot (VARUNA_ESTATE while any slot is forwarded and
 * not yet consumed). */
varuna_status_t varuna_stage_set_dropout_seed(varuna_stage_t* st, uint64_t seed);

/* With wgrad_group G > 1 the operands of the weight-gradient products dW += dY^T X are kept
 * for up to G micro-batches (the workspace holds G slots of them, stacked along the token
 * dimension) and each dW receives ONE GEMM over G*T tokens and one fp32 read-modify-write:
 * gradient accumulation within a GPU (Job Morphing, "Correctness-preserving morphing") with
 * the accumulation partly folded into the GEMM's reduction.  The matrix gradients are then
 * complete only after every G-th backward_recompute call, or after this call, which issues
 * the GEMMs for whatever has been gathered (a no-op when nothing is pending or G <= 1).
 * Bias, gamma and beta gradients are always added per call.  Call it before reading
 * grads_f32 at the end of a mini-batch. */
varuna_status_t varuna_stage_grad_flush(varuna_stage_t* st, void* hip_stream);

/* Zero-fills grads_f32 (start of a mini-batch) and drops any gathered, unflushed operands. */
varuna_status_t varuna_stage_grad_accum_reset(varuna_stage_t* st, void* hip_stream);

/* ---- mini-batch tail: one GPU's share of the optimizer step ------------------------------
 * The paper keeps 16 bytes of state per parameter -- a 16-bit parameter and gradient plus
 * fp32 master weight, momentum and variance (Background, "Memory optimization") -- and
 * synchronises an overflow flag / gradient norm over the stages of a pipeline (Enabling Ease
 * of Programming, "Tracking cross-partition dependencies"; Implementation, "Synchronization
 * of shared state").  These two calls are the per-GPU part; the reduction across GPUs is the
 * caller's.  Both return VARUNA_ESTATE while deferred weight gradients are pending (call
 * varuna_stage_grad_flush first). */

/* out2 (device, 2 floats): [0] = sum of squares of the finite entries of grads_f32,
 * [1] = number of non-finite entries.  Deterministic (fixed reduction order). */
varuna_status_t varuna_stage_grad_stats(varuna_stage_t* st, float* out2 /*device*/, void* hip_stream);

typedef struct {
  float lr, beta1, beta2, eps;
  float weight_decay;  /* decoupled: w -= lr * weight_decay * w */
  float grad_scale;    /* multiplies every gradient first (1/loss scale, 1/M, clip factor) */
  int32_t step;        /* number of this update, >= 1 (bias correction) */
} varuna_adam_t;

/* One Adam update (Kingma & Ba, Algorithm 1, with decoupled weight decay) over all parameters
 * of the stage, element order = parameter layout:  g = grad_scale * grads_f32;
 * m = b1 m + (1-b1) g;  v = b2 v + (1-b2) g^2;
 * master -= lr * ((m / (1-b1^step)) / (sqrt(v / (1-b2^step)) + eps) + weight_decay * master);
 * params_out = master rounded to the stage's storage type (RNE).  master_f32, m_f32, v_f32:
 * caller-owned device buffers of grad_bytes each, 16-byte aligned; params_out: normally the
 * params buffer given to varuna_stage_create.  If skip_if_nonzero (device, may be NULL)
 * points to a non-zero value when the kernel runs, nothing is changed (an overflow anywhere
 * in the pipeline cancels the step). */
varuna_status_t varuna_stage_adam_step(varuna_stage_t* st, const varuna_adam_t* hp, void* params_out /*device*/,
                                       float* master_f32 /*device*/, float* m_f32 /*device*/,
                                       float* v_f32 /*device*/, const float* skip_if_nonzero /*device*/,
                                       void* hip_stream);

/* Releases the host-side handle.  Device buffers stay with the caller. */
varuna_status_t varuna_stage_destroy(varuna_stage_t* st);

const char* varuna_last_error(void);

/* ---- test hooks (not on the timed path) -------------------------------- */

/* Forward that also stores the internal activations of every layer in the
 * workspace, exactly as the recompute pass stores them, so a test can compare
 * the two bit for bit. */
varuna_status_t varuna_stage_debug_forward_save(varuna_stage_t* st, int32_t mb,
                                                const void* x_in /*device*/,
                                                void* y_out /*device*/, void* hip_stream);
/* Byte range of the workspace that holds those stored activations. */
varuna_status_t varuna_stage_debug_saved_region(const varuna_stage_t* st, size_t* offset_bytes,
                                                size_t* n_bytes);

/* Tuning aid: which bf16 MFMA GEMM kernel configuration (the `variant` numbers of varuna_op_gemm)
 * the stage calls use for forward / dgrad / wgrad products on 256x256 and on 128x128 tiles; 0
 * restores the library's choice.  Naming a 128x128 configuration for forward or dgrad also turns
 * off the library's merging of 128x128 tile pairs into one 128x256 / 256x128 tile (configurations
 * 15 / 16) for products of 257..512 such tiles.  Process-wide, not thread-safe, for same-process
 * A/B timing only: results of every configuration agree to rounding but not bit for bit. */
varuna_status_t varuna_debug_set_gemm_kernels(int32_t fwd256, int32_t dgrad256, int32_t wgrad256,
                                              int32_t fwd128, int32_t dgrad128, int32_t wgrad128);
/* Host only (no GPU call): the kernel configuration the library picks for a bf16 product of
 * contiguous, 16-byte aligned operands, op as in varuna_op_gemm (0 forward, 1 dgrad, 2 wgrad):
 * a `variant` number of varuna_op_gemm, -1 for the plain FMA kernel (shape not a multiple of
 * the MFMA tiles), -2 for an invalid argument. */
int32_t varuna_debug_gemm_choice(int32_t op, int64_t M, int64_t N, int64_t K);

/* ---- per-kernel timing (HIP events on the caller's stream) -------------- */

/* Kernel classes reported by the profiler. */
enum {
  VARUNA_K_GEMM_FWD = 0,  /* Y = X W^T (+bias, GeLU, residual) */
  VARUNA_K_GEMM_DGRAD,    /* dX = dY W (+GeLU') */
  VARUNA_K_GEMM_WGRAD,    /* dW += dY^T X */
  VARUNA_K_ATTN_FWD,
  VARUNA_K_ATTN_BWD,
  VARUNA_K_LN_FWD,
  VARUNA_K_LN_BWD,
  VARUNA_K_COLREDUCE,     /* bias / gamma / beta gradient reductions */
  VARUNA_K_OTHER,         /* copies, fills */
  VARUNA_K_COUNT
};
/* While enabled, each kernel launch is bracketed by HIP events on the stream it
 * runs on.  Events come from a fixed pool created here (no device memory). */
varuna_status_t varuna_stage_profile_enable(varuna_stage_t* st, int32_t on);
/* Synchronises the recorded events, adds their durations per class into
 * ms[VARUNA_K_COUNT], launches[...] and flops[...] (algorithmic FLOPs of the
 * launches, 0 for memory-bound classes) and bytes[...] (algorithmic HBM bytes),
 * then clears the record. */
varuna_status_t varuna_stage_profile_collect(varuna_stage_t* st, double* ms, int64_t* launches,
                                             double* flops, double* bytes);

/* ---- measurement hook: what the matrix cores sustain when fed from registers ----------
 * Launches compute_units * waves_per_simd workgroups of 4 waves (waves_per_simd = 1 or 2),
 * each wave issuing iters * 8 independent v_mfma_f32_32x32x16_bf16 products on operand
 * fragments it loaded once from `operands` (device, bf16, n_elems a multiple of 8, 16-byte
 * aligned; indices wrap) -- no LDS or memory traffic inside the loop.  pattern selects which
 * of its 4 + 4 fragments consecutive products read: 0 both operands change every product,
 * 1 the first is held for 8 products, 2 the first for 8 and the second for 2 (a 4x2 register
 * tile walked row by row), 3 both always the same, 4 / 5 as 0 with 4 / 2 consecutive products
 * adding to the same accumulator tile, 6 / 7 as 0 / 2 with two v_mfma_f32_16x16x32_bf16 in
 * place of every 32x32x16 product (the same operation count).  The caller times the
 * launch with events on hip_stream; *flops (host, may be NULL) receives the floating-point
 * operations of the launch.  sink: device, compute_units * waves_per_simd * 256 floats,
 * receives accumulator sums (so the products cannot be elided).  The rate depends on the
 * operand data (all-zero operands toggle no multiplier inputs and run at a higher clock
 * than normally distributed ones): it is the measured ceiling a GEMM on the same kind of
 * data sits under, reported beside the nominal peak. */
varuna_status_t varuna_probe_mfma_rate(const void* operands /*device*/, int64_t n_elems, int32_t waves_per_simd,
                                       int32_t pattern, int32_t iters, float* sink /*device*/,
                                       double* flops /*host*/, void* hip_stream);

/* ---- single-operation entry points (unit parity tests, kernel tuning) ---- */

/* C[M,N] = A * B^T style products on device buffers, dtype as varuna_dtype_t.
 * op: 0 forward  (a = X[M,K],  b = W[N,K],  out[M,N]  = X W^T + bias; epi selects
 *                 0 bias, 1 bias+GeLU (aux_out receives pre-GeLU u if not NULL),
 *                 2 bias+residual (aux_in = residual [M,N]))
 *     1 dgrad    (a = dY[M,K], b = W[K,N],  out[M,N]  = dY W; epi 0 plain,
 *                 3 multiply by GeLU'(aux_in[M,N]))
 *     2 wgrad    (a = dY[K,M], b = X[K,N],  out_f32[M,N] += dY^T X)
 * variant: 0 = library's choice; other values force one kernel configuration
 * (VARUNA_EUNSUPPORTED if it cannot run the shape). */
varuna_status_t varuna_op_gemm(int32_t dtype, int32_t op, int32_t epi, int32_t variant, int64_t M,
                               int64_t N, int64_t K, const void* a, const void* b,
                               const void* bias, const void* aux_in, void* out, void* aux_out,
                               void* hip_stream);

/* LayerNorm forward: y = gamma*(x-mean)*rstd+beta on [rows, h]; stats_f32
 * ([2*rows]: mean then rstd) may be NULL. */
varuna_status_t varuna_op_layernorm_fwd(int32_t dtype, int64_t rows, int64_t h, float eps,
                                        const void* x, const void* gamma, const void* beta,
                                        void* y, float* stats_f32, void* hip_stream);
/* LayerNorm backward: dx = res + LN'(dy); dgamma_f32, dbeta_f32 [h] are added to.
 * partial_f32 is scratch of at least varuna_op_colreduce_scratch_bytes(rows, 2*h). */
varuna_status_t varuna_op_layernorm_bwd(int32_t dtype, int64_t rows, int64_t h, const void* dy,
                                        const void* x, const float* stats_f32, const void* gamma,
                                        const void* res, void* dx, float* dgamma_f32,
                                        float* dbeta_f32, float* partial_f32, void* hip_stream);
/* out_f32[n] += sum over rows of a[rows, n]. */
varuna_status_t varuna_op_colsum(int32_t dtype, int64_t rows, int64_t n, const void* a,
                                 float* out_f32, float* partial_f32, void* hip_stream);
size_t varuna_op_colreduce_scratch_bytes(int64_t rows, int64_t n);

/* varuna_op_colsum for callers that cannot allocate device memory and have no workspace to
 * hand over (code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): the stage-1 partial sums go to a device array built into the library
 * (varuna_op_colsum_static_max_bytes() = 4 MiB per GPU, held until the process ends), so the
 * call takes inputs and outputs only and calls no allocating routine.  Same kernels, same
 * result bit for bit as varuna_op_colsum.  Shapes whose partial sums
 * (varuna_op_colreduce_scratch_bytes(rows, n)) exceed the built-in array are rejected with
 * VARUNA_EUNSUPPORTED before anything is enqueued.  All calls on one GPU share that array:
 * calls whose kernels may overlap on the GPU (different streams, no ordering between them)
 * race; calls ordered on one stream do not.  The array's address is looked up once per
 * device at the first call on that device (the current device when the call is made). */
varuna_status_t varuna_op_colsum_static(int32_t dtype, int64_t rows, int64_t n, const void* a /*device*/,
                                        float* out_f32 /*device*/, void* hip_stream);
size_t varuna_op_colsum_static_max_bytes(void);

/* Attention forward on qkv [b*s, 3h] -> ctx [b*s, h], lse_f32 [b, heads, s]. */
varuna_status_t varuna_op_attention_fwd(int32_t dtype, int32_t variant, int32_t b, int32_t s,
                                        int32_t heads, int32_t d, int32_t causal, const void* qkv,
                                        void* ctx, float* lse_f32, void* hip_stream);
/* Attention backward: dqkv [b*s, 3h] from dctx; delta_f32 [b, heads, s] scratch. */
varuna_status_t varuna_op_attention_bwd(int32_t dtype, int32_t variant, int32_t b, int32_t s,
                                        int32_t heads, int32_t d, int32_t causal, const void* qkv,
                                        const void* ctx, const float* lse_f32, const void* dctx,
                                        void* dqkv, float* delta_f32, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* VARUNA_STAGE_H */
