"""fp64 CPU oracle for one pipeline stage's micro-batched training step.

THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only tests, the smoke check
and the benchmark's cpu_baseline leg may import it.  It shares nothing with
the HIP path and imports nothing from the package.

What it computes (paper: Design Overview, "High-level architecture"; Background,
"Memory optimization"; Job Morphing, "Correctness-preserving morphing"):

  * a stage receives input activations, runs its layers, emits output
    activations (stage forward);
  * it receives output gradients, and produces parameter gradients and the
    input gradient for the previous stage (stage backward);
  * activation recomputation and gradient accumulation over the micro-batches
    held by one GPU change cost, not the result, so the oracle is the plain
    definition: forward storing every intermediate, analytic backward, plain
    sum of parameter gradients over micro-batches.

The paper does not define the transformer layer itself (it refers to GPT-2 /
BERT / Megatron).  The layer used here is the pre-LayerNorm GPT block:

    xn1 = LN(x; g1, b1)               qkv = xn1 Wqkv^T + bqkv
    ctx = softmax(mask(Q K^T / sqrt d)) V      (per batch element and head)
    x1  = x + ctx Wo^T + bo
    xn2 = LN(x1; g2, b2)              u = xn2 W1^T + b1m ;  g = GeLU_tanh(u)
    y   = x1 + g W2^T + b2m

Everything is float64; inputs are whatever the caller hands over (already
rounded to the storage dtype of the GPU path and widened).  No blocking,
fusion or reordering: each line below is one formula of the definition.
Library primitives used as steps: numpy matmul, exp, tanh, sqrt.

Optional dropout (attention probabilities and the two residual branches) takes its masks
from dropout_oracle.py; pins in tests/test_dropout_oracle_pins.py (the generator's published
known-answer vectors, mask statistics, finite differences and torch autograd with the same
masks, recompute regenerating the masks).

Pins (tests/test_oracle_pins.py): central finite differences of every
gradient, torch-autograd composition of library ops, softmax row sums,
causal-mask invariants, closed forms (zero query weights, s=1, zero output
weights), LayerNorm identities, brute-force loops for the linear pieces,
accumulation linearity.  No function here is "parity unpinned".
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Dict, List, Sequence, Tuple

import numpy as np

PARAM_NAMES = (
    "ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo",
    "ln2_g", "ln2_b", "w1", "b1", "w2", "b2",
)

_GELU_C = math.sqrt(2.0 / math.pi)
_GELU_A = 0.044715


@dataclass(frozen=True)
class StageShape:
    n_layers: int
    hidden: int
    n_heads: int
    seq_len: int
    micro_batch: int
    mlp_hidden: int
    causal: bool
    ln_eps: float = 1e-5

    @property
    def head_dim(self) -> int:
        return self.hidden // self.n_heads

    @property
    def tokens(self) -> int:
        return self.micro_batch * self.seq_len


def param_shapes(sh: StageShape) -> Dict[str, Tuple[int, ...]]:
    h, f = sh.hidden, sh.mlp_hidden
    return {
        "ln1_g": (h,), "ln1_b": (h,),
        "wqkv": (3 * h, h), "bqkv": (3 * h,),
        "wo": (h, h), "bo": (h,),
        "ln2_g": (h,), "ln2_b": (h,),
        "w1": (f, h), "b1": (f,),
        "w2": (h, f), "b2": (h,),
    }


# --------------------------------------------------------------------------
# elementary pieces
# --------------------------------------------------------------------------

def gelu_tanh(u: np.ndarray) -> np.ndarray:
    """GeLU, tanh form: 0.5 u (1 + tanh(sqrt(2/pi) (u + 0.044715 u^3)))."""
    return 0.5 * u * (1.0 + np.tanh(_GELU_C * (u + _GELU_A * u ** 3)))


def gelu_tanh_grad(u: np.ndarray) -> np.ndarray:
    """d/du of gelu_tanh."""
    t = np.tanh(_GELU_C * (u + _GELU_A * u ** 3))
    dinner = _GELU_C * (1.0 + 3.0 * _GELU_A * u ** 2)
    return 0.5 * (1.0 + t) + 0.5 * u * (1.0 - t * t) * dinner


def layernorm_forward(x, gamma, beta, eps):
    """Row-wise LayerNorm with biased variance. Returns (y, xhat, rstd)."""
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * rstd
    return gamma * xhat + beta, xhat, rstd


def layernorm_backward(dy, xhat, rstd, gamma):
    """Returns (dx, dgamma, dbeta) for y = gamma*xhat + beta."""
    dxhat = dy * gamma
    m1 = dxhat.mean(axis=-1, keepdims=True)
    m2 = (dxhat * xhat).mean(axis=-1, keepdims=True)
    dx = rstd * (dxhat - m1 - xhat * m2)
    return dx, (dy * xhat).sum(axis=0), dy.sum(axis=0)


def linear_forward(x, w, b):
    """y = x w^T + b with w stored [out, in]."""
    return x @ w.T + b


def linear_backward(dy, x, w):
    """Returns (dx, dw, db) of y = x w^T + b."""
    return dy @ w, dy.T @ x, dy.sum(axis=0)


def attention_forward(qkv, sh: StageShape, keep=None):
    """Softmax attention per (batch element, head).

    keep (optional): function (bi, j) -> [s, s] array of dropout factors (scale where the
    probability is kept, 0 where dropped), applied to the probabilities after the softmax.

    qkv is [T, 3h] with column blocks [Q | K | V]; head j owns columns
    j*d..(j+1)*d-1 of each block.  Scores are scaled by 1/sqrt(d) before the
    mask; masked scores (key index > query index when causal) are -inf, so
    their probabilities are exactly zero.  Returns (ctx [T,h], P list) where
    P[(bi, j)] is the [s, s] probability matrix.
    """
    h, d, s = sh.hidden, sh.head_dim, sh.seq_len
    ctx = np.zeros((sh.tokens, h))
    probs = {}
    scale = 1.0 / math.sqrt(d)
    for bi in range(sh.micro_batch):
        rows = slice(bi * s, (bi + 1) * s)
        for j in range(sh.n_heads):
            q = qkv[rows, j * d:(j + 1) * d]
            k = qkv[rows, h + j * d:h + (j + 1) * d]
            v = qkv[rows, 2 * h + j * d:2 * h + (j + 1) * d]
            sc = (q @ k.T) * scale
            if sh.causal:
                ii, kk = np.indices((s, s))
                sc = np.where(kk > ii, -np.inf, sc)
            e = np.exp(sc - sc.max(axis=1, keepdims=True))
            p = e / e.sum(axis=1, keepdims=True)
            probs[(bi, j)] = p
            ctx[rows, j * d:(j + 1) * d] = (p if keep is None else p * keep(bi, j)) @ v
    return ctx, probs


def attention_backward(dctx, qkv, probs, sh: StageShape, keep=None):
    """Gradient of attention_forward w.r.t. qkv (same dropout factors). Returns dqkv [T, 3h]."""
    h, d, s = sh.hidden, sh.head_dim, sh.seq_len
    dqkv = np.zeros_like(qkv)
    scale = 1.0 / math.sqrt(d)
    for bi in range(sh.micro_batch):
        rows = slice(bi * s, (bi + 1) * s)
        for j in range(sh.n_heads):
            q = qkv[rows, j * d:(j + 1) * d]
            k = qkv[rows, h + j * d:h + (j + 1) * d]
            v = qkv[rows, 2 * h + j * d:2 * h + (j + 1) * d]
            p = probs[(bi, j)]
            do = dctx[rows, j * d:(j + 1) * d]
            if keep is None:
                dv = p.T @ do
                dp = do @ v.T
            else:
                kp = keep(bi, j)
                dv = (p * kp).T @ do
                dp = (do @ v.T) * kp
            ds = p * (dp - (p * dp).sum(axis=1, keepdims=True))
            dqkv[rows, j * d:(j + 1) * d] = (ds @ k) * scale
            dqkv[rows, h + j * d:h + (j + 1) * d] = (ds.T @ q) * scale
            dqkv[rows, 2 * h + j * d:2 * h + (j + 1) * d] = dv
    return dqkv


# --------------------------------------------------------------------------
# one layer
# --------------------------------------------------------------------------

def _drop_factors(drop, sh: StageShape, layer: int, mb: int):
    """(keep(bi, j) for the attention probabilities, [T,h] factors of the projection branch,
    [T,h] factors of the MLP branch) for one layer of one micro-batch, or (None, 1, 1)."""
    if drop is None:
        return None, 1.0, 1.0
    s, a = sh.seq_len, sh.n_heads
    keep = lambda bi, j: drop.keep_scale(0, layer, mb, (bi * a + j) * s, s, s)
    return keep, drop.keep_scale(1, layer, mb, 0, sh.tokens, sh.hidden), drop.keep_scale(2, layer, mb, 0, sh.tokens, sh.hidden)


def layer_forward(x, p: Dict[str, np.ndarray], sh: StageShape, drop=None, layer: int = 0, mb: int = 0):
    """Forward of one pre-LN block. Returns (y, cache of every intermediate).  With drop (a
    dropout_oracle.Dropout) the attention probabilities and the two residual branches are
    multiplied by their dropout factors, which depend only on (seed, mb, layer, site, element)."""
    keep, k1, k2 = _drop_factors(drop, sh, layer, mb)
    c = {"x": x, "keep": keep, "k1": k1, "k2": k2}
    c["xn1"], c["xhat1"], c["rstd1"] = layernorm_forward(x, p["ln1_g"], p["ln1_b"], sh.ln_eps)
    c["qkv"] = linear_forward(c["xn1"], p["wqkv"], p["bqkv"])
    c["ctx"], c["probs"] = attention_forward(c["qkv"], sh, keep)
    c["x1"] = x + k1 * linear_forward(c["ctx"], p["wo"], p["bo"])
    c["xn2"], c["xhat2"], c["rstd2"] = layernorm_forward(c["x1"], p["ln2_g"], p["ln2_b"], sh.ln_eps)
    c["u"] = linear_forward(c["xn2"], p["w1"], p["b1"])
    c["g"] = gelu_tanh(c["u"])
    y = c["x1"] + k2 * linear_forward(c["g"], p["w2"], p["b2"])
    return y, c


def layer_backward(dy, p: Dict[str, np.ndarray], c, sh: StageShape):
    """Backward of one block. Returns (dx, dict of parameter gradients)."""
    gr = {}
    dg, gr["w2"], gr["b2"] = linear_backward(dy * c["k2"], c["g"], p["w2"])
    du = dg * gelu_tanh_grad(c["u"])
    dxn2, gr["w1"], gr["b1"] = linear_backward(du, c["xn2"], p["w1"])
    dln2, gr["ln2_g"], gr["ln2_b"] = layernorm_backward(dxn2, c["xhat2"], c["rstd2"], p["ln2_g"])
    dx1 = dy + dln2
    dctx, gr["wo"], gr["bo"] = linear_backward(dx1 * c["k1"], c["ctx"], p["wo"])
    dqkv = attention_backward(dctx, c["qkv"], c["probs"], sh, c["keep"])
    dxn1, gr["wqkv"], gr["bqkv"] = linear_backward(dqkv, c["xn1"], p["wqkv"])
    dln1, gr["ln1_g"], gr["ln1_b"] = layernorm_backward(dxn1, c["xhat1"], c["rstd1"], p["ln1_g"])
    return dx1 + dln1, gr


# --------------------------------------------------------------------------
# the stage
# --------------------------------------------------------------------------

def stage_forward(x, params: Sequence[Dict[str, np.ndarray]], sh: StageShape, drop=None, mb: int = 0):
    """Stage forward for one micro-batch (number mb).  x: [T, h].  Returns (y, caches).

    The caches are what a recompute pass re-derives from the stored stage
    input; the oracle simply keeps them.
    """
    caches = []
    for l, p in enumerate(params):
        x, c = layer_forward(x, p, sh, drop, l, mb)
        caches.append(c)
    return x, caches


def stage_backward(dy, params, caches, sh: StageShape):
    """Stage backward for one micro-batch. Returns (dX, per-layer grads)."""
    grads: List[Dict[str, np.ndarray]] = [None] * len(params)
    for l in range(len(params) - 1, -1, -1):
        dy, grads[l] = layer_backward(dy, params[l], caches[l], sh)
    return dy, grads


def stage_step(xs, dys, params, sh: StageShape, drop=None):
    """One mini-batch on the stage: all micro-batches, gradients summed.

    xs, dys: sequences of [T, h] arrays (stage inputs, upstream gradients).
    Returns (ys, dxs, accumulated per-layer grads).  Accumulation is a plain
    sum over micro-batches, no 1/M factor.
    """
    ys, dxs = [], []
    acc = [{k: np.zeros(v) for k, v in param_shapes(sh).items()} for _ in params]
    for mb, (x, dy) in enumerate(zip(xs, dys)):
        y, caches = stage_forward(x, params, sh, drop, mb)
        dx, gr = stage_backward(dy, params, caches, sh)
        ys.append(y)
        dxs.append(dx)
        for l in range(len(params)):
            for k in PARAM_NAMES:
                acc[l][k] += gr[l][k]
    return ys, dxs, acc


def stage_recompute(x_boundary, params, sh: StageShape, drop=None, mb: int = 0):
    """Recompute path: re-derive every intermediate from the stored boundary
    activation alone (Design Overview, High-level architecture).  Same
    arithmetic as stage_forward; kept as a separate entry so a test can
    state the equality."""
    return stage_forward(np.array(x_boundary, copy=True), params, sh, drop, mb)


def rel_l2(a, ref) -> float:
    """||a - ref||_2 / ||ref||_2 in float64 (the parity metric)."""
    a = np.asarray(a, dtype=np.float64).ravel()
    ref = np.asarray(ref, dtype=np.float64).ravel()
    den = float(np.linalg.norm(ref))
    num = float(np.linalg.norm(a - ref))
    if den == 0.0:
        return 0.0 if num == 0.0 else float("inf")
    return num / den
