"""Cost model of the stage step (host logic, no GPU).

Per layer and micro-batch, forward: 24*T*h^2 GEMM FLOPs (for f = 4h; in general
2*T*h*(4h + 2f)) plus 4*T*s*h attention FLOPs (dense count; a causal mask does
half).  One step runs forward, recompute and backward (= 2 forwards) per
micro-batch: 4 forward units of hardware work, 3 of which are "useful" in the
paper's convention (Evaluation, Performance & Cost: the recompute share is
removed from reported TFLOP/s).
"""
from __future__ import annotations

from .synth import StageConfig

MI355X_BF16_DENSE_PEAK = 2.5e15   # FLOP/s, published dense bf16 MFMA peak
MI355X_HBM_PEAK = 8.0e12          # B/s


def forward_flops(cfg: StageConfig, causal_aware: bool = True) -> float:
    """FLOPs of one stage forward for one micro-batch."""
    T, h, f, s = cfg.tokens, cfg.hidden, cfg.mlp_hidden, cfg.seq_len
    gemm = 2.0 * T * h * (4 * h + 2 * f)
    attn = 4.0 * T * s * h
    if cfg.causal and causal_aware:
        attn *= 0.5
    return cfg.n_layers * (gemm + attn)


def step_flops_per_microbatch(cfg: StageConfig, causal_aware: bool = True) -> float:
    """Hardware FLOPs per micro-batch: forward + recompute + backward = 4 units."""
    return 4.0 * forward_flops(cfg, causal_aware)


def useful_flops_per_microbatch(cfg: StageConfig, causal_aware: bool = True) -> float:
    """The paper's convention: recompute excluded = 3 units."""
    return 3.0 * forward_flops(cfg, causal_aware)


def model_flops_per_example(n_layers: int, hidden: int, seq_len: int) -> float:
    """Useful FLOPs to train one example through n_layers (f = 4h, dense attention)."""
    return n_layers * seq_len * (72.0 * hidden ** 2 + 12.0 * seq_len * hidden)
