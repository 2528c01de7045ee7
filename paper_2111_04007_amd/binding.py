"""ctypes binding of the C ABI in include/varuna_stage.h.

Argument marshalling only: every step of the stage runs in the HIP library.
PyTorch tensors supply device memory and the stream.  There is no CPU
fallback: if the shared library is missing, load() raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

from .synth import StageConfig

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libvaruna_stage.so")

OK, EINVAL, ESTATE, ENOMEM, EHIP, EUNSUPPORTED = 0, -1, -2, -3, -4, -5
F32, BF16 = 0, 1
PARAM_NAMES = ("ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo", "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")
KERNEL_CLASSES = ("gemm_fwd", "gemm_dgrad", "gemm_wgrad", "attn_fwd", "attn_bwd", "ln_fwd", "ln_bwd",
                  "colreduce", "other")
OP_FWD, OP_DGRAD, OP_WGRAD = 0, 1, 2

EXPORTS = (
    "varuna_stage_query_sizes", "varuna_stage_param_offset", "varuna_stage_create",
    "varuna_stage_forward", "varuna_stage_backward_recompute", "varuna_stage_grad_accum_reset",
    "varuna_stage_forward_keep", "varuna_stage_backward_stored", "varuna_stage_grad_stats", "varuna_stage_adam_step", "varuna_stage_set_dropout_seed", "varuna_stage_set_side_stream",
    "varuna_stage_grad_flush", "varuna_stage_destroy", "varuna_last_error", "varuna_stage_debug_forward_save",
    "varuna_stage_debug_saved_region", "varuna_stage_profile_enable", "varuna_stage_profile_collect",
    "varuna_op_gemm", "varuna_op_layernorm_fwd", "varuna_op_layernorm_bwd", "varuna_op_colsum",
    "varuna_op_colreduce_scratch_bytes", "varuna_op_attention_fwd", "varuna_op_attention_bwd",
    "varuna_op_colsum_static", "varuna_op_colsum_static_max_bytes", "varuna_probe_mfma_rate",
    "varuna_debug_set_gemm_kernels",
    "varuna_debug_gemm_choice",
)


class VarunaError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"varuna status {code}: {msg}")
        self.code = code


class CAdam(C.Structure):
    _fields_ = [(n, C.c_float) for n in ("lr", "beta1", "beta2", "eps", "weight_decay", "grad_scale")] + [("step", C.c_int32)]


class CConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_layers", "hidden", "n_heads", "seq_len", "micro_batch", "n_micro_batches",
        "mlp_hidden", "causal", "dtype")] + [("ln_eps", C.c_float), ("wgrad_group", C.c_int32), ("dropout_p", C.c_float)]


def c_config(cfg: StageConfig) -> CConfig:
    return CConfig(cfg.n_layers, cfg.hidden, cfg.n_heads, cfg.seq_len, cfg.micro_batch,
                   cfg.n_micro_batches, cfg.mlp_hidden, int(cfg.causal),
                   F32 if cfg.dtype == "f32" else BF16, cfg.ln_eps, cfg.wgrad_group, cfg.dropout_p)


_lib = None


def load():
    """Loads libvaruna_stage.so (built by build.py). Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} not found: build it with `python -m paper_2111_04007_amd.build` "
            "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    psz = C.POINTER(C.c_size_t)
    pcfg = C.POINTER(CConfig)
    sig = {
        "varuna_stage_query_sizes": (i32, [pcfg, psz, psz, psz, psz]),
        "varuna_stage_param_offset": (i32, [pcfg, i32, i32, psz, psz]),
        "varuna_stage_create": (i32, [pcfg, vp, vp, vp, vp, C.POINTER(vp)]),
        "varuna_stage_forward": (i32, [vp, i32, vp, vp, vp]),
        "varuna_stage_backward_recompute": (i32, [vp, i32, vp, vp, vp]),
        "varuna_stage_forward_keep": (i32, [vp, i32, vp, vp, vp]),
        "varuna_stage_backward_stored": (i32, [vp, i32, vp, vp, vp]),
        "varuna_stage_grad_accum_reset": (i32, [vp, vp]),
        "varuna_stage_set_dropout_seed": (i32, [vp, C.c_uint64]),
        "varuna_stage_set_side_stream": (i32, [vp, vp]),
        "varuna_stage_grad_stats": (i32, [vp, vp, vp]),
        "varuna_stage_adam_step": (i32, [vp, C.POINTER(CAdam), vp, vp, vp, vp, vp, vp]),
        "varuna_stage_grad_flush": (i32, [vp, vp]),
        "varuna_stage_destroy": (i32, [vp]),
        "varuna_last_error": (C.c_char_p, []),
        "varuna_stage_debug_forward_save": (i32, [vp, i32, vp, vp, vp]),
        "varuna_stage_debug_saved_region": (i32, [vp, psz, psz]),
        "varuna_stage_profile_enable": (i32, [vp, i32]),
        "varuna_stage_profile_collect": (i32, [vp, C.POINTER(C.c_double), C.POINTER(i64),
                                               C.POINTER(C.c_double), C.POINTER(C.c_double)]),
        "varuna_op_gemm": (i32, [i32, i32, i32, i32, i64, i64, i64, vp, vp, vp, vp, vp, vp, vp]),
        "varuna_op_layernorm_fwd": (i32, [i32, i64, i64, C.c_float, vp, vp, vp, vp, vp, vp]),
        "varuna_op_layernorm_bwd": (i32, [i32, i64, i64, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]),
        "varuna_op_colsum": (i32, [i32, i64, i64, vp, vp, vp, vp]),
        "varuna_op_colreduce_scratch_bytes": (sz, [i64, i64]),
        "varuna_op_colsum_static": (i32, [i32, i64, i64, vp, vp, vp]),
        "varuna_op_colsum_static_max_bytes": (sz, []),
        "varuna_debug_set_gemm_kernels": (i32, [i32] * 6),
        "varuna_debug_gemm_choice": (i32, [i32, i64, i64, i64]),
        "varuna_probe_mfma_rate": (i32, [vp, i64, i32, i32, i32, vp, C.POINTER(C.c_double), vp]),
        "varuna_op_attention_fwd": (i32, [i32, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp]),
        "varuna_op_attention_bwd": (i32, [i32, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def _check(rc: int):
    if rc != OK:
        raise VarunaError(rc, load().varuna_last_error().decode())


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream_ptr(stream=None):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def query_sizes(cfg: StageConfig):
    """(param_bytes, grad_bytes, boundary_bytes, workspace_bytes); touches no GPU."""
    cc = c_config(cfg)
    vals = [C.c_size_t() for _ in range(4)]
    _check(load().varuna_stage_query_sizes(C.byref(cc), *[C.byref(v) for v in vals]))
    return tuple(v.value for v in vals)


def param_offset(cfg: StageConfig, layer: int, which: int):
    cc = c_config(cfg)
    off, n = C.c_size_t(), C.c_size_t()
    _check(load().varuna_stage_param_offset(C.byref(cc), layer, which, C.byref(off), C.byref(n)))
    return off.value, n.value


class Stage:
    """varuna_stage_* over torch-allocated device buffers."""

    def __init__(self, cfg: StageConfig, device="cuda:0", params_flat: Optional[torch.Tensor] = None):
        self.cfg = cfg
        self.lib = load()
        self.device = torch.device(device)
        pb, gb, bb, wb = query_sizes(cfg)
        self.act_dtype = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
        es = 4 if cfg.dtype == "f32" else 2
        if params_flat is None:
            params_flat = torch.zeros(pb // es, dtype=self.act_dtype, device=self.device)
        assert params_flat.numel() * es == pb and params_flat.dtype == self.act_dtype
        self.params = params_flat
        self.grads = torch.zeros(gb // 4, dtype=torch.float32, device=self.device)
        self.boundary = torch.empty(bb // es, dtype=self.act_dtype, device=self.device)
        self.workspace = torch.empty(wb, dtype=torch.uint8, device=self.device)
        self.handle = C.c_void_p()
        cc = c_config(cfg)
        _check(self.lib.varuna_stage_create(C.byref(cc), _ptr(self.params), _ptr(self.grads),
                                            _ptr(self.boundary), _ptr(self.workspace),
                                            C.byref(self.handle)))

    # -- parameters ---------------------------------------------------------
    def set_params(self, layers):
        """layers: list of dicts name -> CPU/GPU tensor in storage dtype."""
        for l, layer in enumerate(layers):
            for i, name in enumerate(PARAM_NAMES):
                off, n = param_offset(self.cfg, l, i)
                self.params[off:off + n].copy_(layer[name].reshape(-1).to(self.device))

    def grad_view(self, layer: int, name: str) -> torch.Tensor:
        off, n = param_offset(self.cfg, layer, PARAM_NAMES.index(name))
        return self.grads[off:off + n]

    def boundary_slot(self, mb: int) -> torch.Tensor:
        E = self.cfg.tokens * self.cfg.hidden
        return self.boundary[mb * E:(mb + 1) * E].view(self.cfg.tokens, self.cfg.hidden)

    # -- the four calls -----------------------------------------------------
    def forward(self, mb: int, x: torch.Tensor, y: torch.Tensor, stream=None):
        _check(self.lib.varuna_stage_forward(self.handle, mb, _ptr(x), _ptr(y), _stream_ptr(stream)))

    def backward_recompute(self, mb: int, dy: torch.Tensor, dx: torch.Tensor, stream=None):
        _check(self.lib.varuna_stage_backward_recompute(self.handle, mb, _ptr(dy), _ptr(dx), _stream_ptr(stream)))

    def forward_keep(self, mb: int, x: torch.Tensor, y: torch.Tensor, stream=None):
        _check(self.lib.varuna_stage_forward_keep(self.handle, mb, _ptr(x), _ptr(y), _stream_ptr(stream)))

    def backward_stored(self, mb: int, dy: torch.Tensor, dx: torch.Tensor, stream=None):
        _check(self.lib.varuna_stage_backward_stored(self.handle, mb, _ptr(dy), _ptr(dx), _stream_ptr(stream)))

    def set_side_stream(self, stream):
        """stream: a torch.cuda.Stream the caller keeps alive (held here too), or None."""
        self._side_stream = stream
        _check(self.lib.varuna_stage_set_side_stream(self.handle, None if stream is None else C.c_void_p(stream.cuda_stream)))

    def set_dropout_seed(self, seed: int):
        _check(self.lib.varuna_stage_set_dropout_seed(self.handle, seed))

    def grad_stats(self, out2: torch.Tensor, stream=None):
        _check(self.lib.varuna_stage_grad_stats(self.handle, _ptr(out2), _stream_ptr(stream)))

    def adam_step(self, master, m, v, step: int, lr: float, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0,
                  grad_scale=1.0, skip=None, params_out=None, stream=None):
        hp = CAdam(lr, beta1, beta2, eps, weight_decay, grad_scale, step)
        out = self.params if params_out is None else params_out
        _check(self.lib.varuna_stage_adam_step(self.handle, C.byref(hp), _ptr(out), _ptr(master), _ptr(m), _ptr(v),
                                               _ptr(skip), _stream_ptr(stream)))

    def grad_accum_reset(self, stream=None):
        _check(self.lib.varuna_stage_grad_accum_reset(self.handle, _stream_ptr(stream)))

    def grad_flush(self, stream=None):
        _check(self.lib.varuna_stage_grad_flush(self.handle, _stream_ptr(stream)))

    # -- hooks --------------------------------------------------------------
    def debug_forward_save(self, mb: int, x: torch.Tensor, y: torch.Tensor, stream=None):
        _check(self.lib.varuna_stage_debug_forward_save(self.handle, mb, _ptr(x), _ptr(y), _stream_ptr(stream)))

    def saved_region(self) -> torch.Tensor:
        off, n = C.c_size_t(), C.c_size_t()
        _check(self.lib.varuna_stage_debug_saved_region(self.handle, C.byref(off), C.byref(n)))
        return self.workspace[off.value:off.value + n.value]

    def profile_enable(self, on: bool):
        _check(self.lib.varuna_stage_profile_enable(self.handle, int(on)))

    def profile_collect(self):
        n = len(KERNEL_CLASSES)
        ms = (C.c_double * n)()
        cnt = (C.c_int64 * n)()
        fl = (C.c_double * n)()
        by = (C.c_double * n)()
        _check(self.lib.varuna_stage_profile_collect(self.handle, ms, cnt, fl, by))
        return {k: {"ms": ms[i], "launches": cnt[i], "flops": fl[i], "bytes": by[i]}
                for i, k in enumerate(KERNEL_CLASSES)}

    def close(self):
        if self.handle:
            torch.cuda.synchronize(self.device)
            _check(self.lib.varuna_stage_destroy(self.handle))
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# ---- single operations ------------------------------------------------------

def op_gemm(op: int, epi: int, a, b, out, bias=None, aux_in=None, aux_out=None, variant: int = 0,
            M: int = 0, N: int = 0, K: int = 0, stream=None):
    _check(load().varuna_op_gemm(dtype_code(a), op, epi, variant, M, N, K, _ptr(a), _ptr(b), _ptr(bias),
                                 _ptr(aux_in), _ptr(out), _ptr(aux_out), _stream_ptr(stream)))


def op_layernorm_fwd(x, gamma, beta, y, stats=None, eps=1e-5, stream=None):
    rows, h = x.shape
    _check(load().varuna_op_layernorm_fwd(dtype_code(x), rows, h, eps, _ptr(x), _ptr(gamma), _ptr(beta),
                                          _ptr(y), _ptr(stats), _stream_ptr(stream)))


def colreduce_scratch_bytes(rows: int, n: int) -> int:
    return load().varuna_op_colreduce_scratch_bytes(rows, n)


def op_layernorm_bwd(dy, x, stats, gamma, res, dx, dgamma, dbeta, partial, stream=None):
    rows, h = x.shape
    _check(load().varuna_op_layernorm_bwd(dtype_code(x), rows, h, _ptr(dy), _ptr(x), _ptr(stats), _ptr(gamma),
                                          _ptr(res), _ptr(dx), _ptr(dgamma), _ptr(dbeta), _ptr(partial),
                                          _stream_ptr(stream)))


def op_colsum(a, out, partial, stream=None):
    rows, n = a.shape
    _check(load().varuna_op_colsum(dtype_code(a), rows, n, _ptr(a), _ptr(out), _ptr(partial), _stream_ptr(stream)))


def op_colsum_static(a, out, stream=None):
    rows, n = a.shape
    _check(load().varuna_op_colsum_static(dtype_code(a), rows, n, _ptr(a), _ptr(out), _stream_ptr(stream)))


def colsum_static_max_bytes() -> int:
    return load().varuna_op_colsum_static_max_bytes()


def debug_set_gemm_kernels(fwd256=0, dgrad256=0, wgrad256=0, fwd128=0, dgrad128=0, wgrad128=0):
    _check(load().varuna_debug_set_gemm_kernels(fwd256, dgrad256, wgrad256, fwd128, dgrad128, wgrad128))


def debug_gemm_choice(op: int, M: int, N: int, K: int) -> int:
    """Host only: the bf16 GEMM kernel configuration the library picks for this product."""
    return int(load().varuna_debug_gemm_choice(op, M, N, K))


def probe_mfma_rate(operands, waves_per_simd: int, iters: int, sink, pattern: int = 0, stream=None) -> float:
    """Enqueues the register-only MFMA loop; returns the FLOPs of the launch."""
    fl = C.c_double()
    _check(load().varuna_probe_mfma_rate(_ptr(operands), operands.numel(), waves_per_simd, pattern, iters, _ptr(sink),
                                         C.byref(fl), _stream_ptr(stream)))
    return fl.value


def op_attention_fwd(qkv, ctx, lse, b, s, heads, d, causal, variant=0, stream=None):
    _check(load().varuna_op_attention_fwd(dtype_code(qkv), variant, b, s, heads, d, int(causal), _ptr(qkv),
                                          _ptr(ctx), _ptr(lse), _stream_ptr(stream)))


def op_attention_bwd(qkv, ctx, lse, dctx, dqkv, delta, b, s, heads, d, causal, variant=0, stream=None):
    _check(load().varuna_op_attention_bwd(dtype_code(qkv), variant, b, s, heads, d, int(causal), _ptr(qkv),
                                          _ptr(ctx), _ptr(lse), _ptr(dctx), _ptr(dqkv), _ptr(delta),
                                          _stream_ptr(stream)))
