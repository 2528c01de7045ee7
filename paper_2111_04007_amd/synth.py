"""Seeded synthetic stage inputs (weights, stage-input activations, upstream
gradients).  This module is data plumbing shared by the tests, the benchmark
and the oracle's callers; it contains none of the method's arithmetic.

Recipe (shapes follow the paper's workloads: BERT-large, GPT-2 2.5B / 8.3B and
a 200B-class GPT; Evaluation section; a middle stage only ever sees activation
tensors, which the paper's own calibration mocks with random values,
Scale-invariant Calibration):
  weights ~ N(0, w_std), LayerNorm gamma = 1, beta = 0, biases = 0,
  stage inputs ~ N(0, 1), upstream gradients ~ N(0, 1).
Values are drawn in float64 from numpy's Philox counter-based generator keyed
on (seed, tensor id), then rounded once to the storage dtype; the rounded
values are what both the GPU path and the oracle consume.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List

import numpy as np
import torch

PARAM_ORDER = (
    "ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo",
    "ln2_g", "ln2_b", "w1", "b1", "w2", "b2",
)


@dataclass(frozen=True)
class StageConfig:
    name: str
    n_layers: int
    hidden: int
    n_heads: int
    seq_len: int
    micro_batch: int
    n_micro_batches: int
    mlp_hidden: int
    causal: bool
    dtype: str            # "f32" or "bf16"
    w_std: float = 0.02
    ln_eps: float = 1e-5
    seed: int = 20211104
    wgrad_group: int = 1  # micro-batches per weight-gradient GEMM (library knob, not part of the workload)
    dropout_p: float = 0.0  # dropout probability (0: none; the paper's configs name none)

    @property
    def tokens(self) -> int:
        return self.micro_batch * self.seq_len

    @property
    def head_dim(self) -> int:
        return self.hidden // self.n_heads

    def replace(self, **kw) -> "StageConfig":
        d = dict(self.__dict__)
        d.update(kw)
        return StageConfig(**d)


# The five workloads (tiny fp32 stage; BERT-large-, GPT-2 2.5B-, 8.3B- and
# 200B-class-shaped bf16 stages).
CONFIGS: Dict[str, StageConfig] = {
    "C1": StageConfig("C1-tiny-fp32", 2, 128, 2, 64, 2, 4, 512, True, "f32", 0.02, seed=20211104),
    "C2": StageConfig("C2-bert-large-stage", 6, 1024, 16, 512, 8, 8, 4096, False, "bf16", 0.02, seed=20211105),
    "C3": StageConfig("C3-gpt2-2.5b-stage", 4, 1920, 20, 1024, 4, 16, 7680, True, "bf16", 0.02, seed=20211106),
    "C4": StageConfig("C4-gpt-8.3b-stage", 3, 3072, 32, 1024, 2, 16, 12288, True, "bf16", 0.02, seed=20211107),
    "C5": StageConfig("C5-gpt-200b-class-stage", 2, 8192, 64, 2048, 1, 32, 32768, True, "bf16", 0.01, seed=20211108),
}


def param_shapes(cfg: StageConfig):
    h, f = cfg.hidden, cfg.mlp_hidden
    return {
        "ln1_g": (h,), "ln1_b": (h,), "wqkv": (3 * h, h), "bqkv": (3 * h,),
        "wo": (h, h), "bo": (h,), "ln2_g": (h,), "ln2_b": (h,),
        "w1": (f, h), "b1": (f,), "w2": (h, f), "b2": (h,),
    }


def torch_dtype(cfg: StageConfig):
    return torch.float32 if cfg.dtype == "f32" else torch.bfloat16


def _normal(seed: int, tensor_id: int, shape, std: float) -> np.ndarray:
    rng = np.random.Generator(np.random.Philox(key=[seed, tensor_id]))
    return rng.standard_normal(size=shape) * std


def _round(a: np.ndarray, cfg: StageConfig) -> torch.Tensor:
    """Round a float64 array once to the storage dtype (RNE)."""
    return torch.from_numpy(np.ascontiguousarray(a)).to(torch_dtype(cfg))


def make_params(cfg: StageConfig, perturb: float = 0.0) -> List[Dict[str, torch.Tensor]]:
    """Per-layer parameter tensors in storage dtype (CPU).

    perturb > 0 adds N(0, perturb) noise to gamma/beta/biases so that tests
    can exercise every term; perturb = 0 is the configs' initialisation.
    """
    out = []
    for l in range(cfg.n_layers):
        layer = {}
        for i, (k, shp) in enumerate(param_shapes(cfg).items()):
            tid = 1000 * (l + 1) + i
            if k in ("wqkv", "wo", "w1", "w2"):
                a = _normal(cfg.seed, tid, shp, cfg.w_std)
            else:
                base = 1.0 if k.endswith("_g") else 0.0
                a = np.full(shp, base)
                if perturb > 0.0:
                    a = a + _normal(cfg.seed, tid, shp, perturb)
            layer[k] = _round(a, cfg)
        out.append(layer)
    return out


def make_activations(cfg: StageConfig, n_mb: int | None = None):
    """(xs, dys): lists of [T, h] CPU tensors in storage dtype."""
    n = cfg.n_micro_batches if n_mb is None else n_mb
    T, h = cfg.tokens, cfg.hidden
    xs = [_round(_normal(cfg.seed, 10_000_000 + 2 * m, (T, h), 1.0), cfg) for m in range(n)]
    dys = [_round(_normal(cfg.seed, 10_000_000 + 2 * m + 1, (T, h), 1.0), cfg) for m in range(n)]
    return xs, dys


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().to(torch.float64).numpy()


def params_to_f64(params):
    return [{k: to_f64(v) for k, v in layer.items()} for layer in params]


def device_random_stage(cfg: StageConfig, device, n_mb: int | None = None):
    """Same distributions drawn directly on the device with torch's seeded
    generator (for throughput runs at sizes where host generation would take
    minutes).  Returns (flat params tensor, xs [M,T,h], dys [M,T,h])."""
    g = torch.Generator(device=device)
    g.manual_seed(cfg.seed)
    dt = torch_dtype(cfg)
    chunks = []
    for _ in range(cfg.n_layers):
        for k, shp in param_shapes(cfg).items():
            n = int(np.prod(shp))
            if k in ("wqkv", "wo", "w1", "w2"):
                t = torch.empty(n, device=device, dtype=torch.float32)
                t.normal_(0.0, cfg.w_std, generator=g)
                chunks.append(t.to(dt))
            elif k.endswith("_g"):
                chunks.append(torch.ones(n, device=device, dtype=dt))
            else:
                chunks.append(torch.zeros(n, device=device, dtype=dt))
    flat = torch.cat(chunks)
    n = cfg.n_micro_batches if n_mb is None else n_mb
    xs = torch.empty((n, cfg.tokens, cfg.hidden), device=device, dtype=torch.float32).normal_(generator=g).to(dt)
    dys = torch.empty((n, cfg.tokens, cfg.hidden), device=device, dtype=torch.float32).normal_(generator=g).to(dt)
    return flat, xs, dys
