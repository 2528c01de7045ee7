"""Helpers shared by the GPU parity tests: run the HIP stage through the C ABI,
run the oracle on the same seeded inputs, compare with the rel-L2 metric."""
from __future__ import annotations

import numpy as np
import torch

from oracle import stage_oracle as O
from paper_2111_04007_amd import binding as B, synth

TOL = {"f32": 1e-5, "bf16": 2e-2}


def oracle_shape(cfg: synth.StageConfig) -> O.StageShape:
    return O.StageShape(cfg.n_layers, cfg.hidden, cfg.n_heads, cfg.seq_len, cfg.micro_batch,
                        cfg.mlp_hidden, cfg.causal, cfg.ln_eps)


def gpu_stage_step(cfg, params, xs, dys, device="cuda:0", interleave=False, last_stage=False, seed=0, side_stream=True):
    """Runs reset, M forwards, M backward_recomputes (last_stage: M times forward_keep
    followed at once by backward_stored). Returns (stage, ys, dxs) with outputs as CPU
    tensors; the accumulated gradients stay in stage.grads."""
    st = B.Stage(cfg, device)
    st.set_params(params)
    if side_stream:   # the launch configuration bench.py times: bias-gradient sums beside the GEMM chain
        st.set_side_stream(torch.cuda.Stream(device))
    if cfg.dropout_p > 0:
        st.set_dropout_seed(seed)
    st.grad_accum_reset()
    n = len(xs)
    dx_ = [x.to(device) for x in xs]
    ddy = [d.to(device) for d in dys]
    ys = [torch.empty_like(dx_[0]) for _ in range(n)]
    dxs = [torch.empty_like(dx_[0]) for _ in range(n)]
    if last_stage:
        for m in range(n):
            st.forward_keep(m, dx_[m], ys[m])
            st.backward_stored(m, ddy[m], dxs[m])
    elif interleave:
        # a legal pipeline order: forward of m+1 issued between backward calls
        st.forward(0, dx_[0], ys[0])
        for m in range(n):
            if m + 1 < n:
                st.forward(m + 1, dx_[m + 1], ys[m + 1])
            st.backward_recompute(m, ddy[m], dxs[m])
    else:
        for m in range(n):
            st.forward(m, dx_[m], ys[m])
        for m in range(n):
            st.backward_recompute(m, ddy[m], dxs[m])
    st.grad_flush()   # issues a pending weight-gradient group (no-op when wgrad_group <= 1)
    torch.cuda.synchronize()
    return st, [y.cpu() for y in ys], [d.cpu() for d in dxs]


def oracle_stage_step(cfg, params, xs, dys, seed=0):
    sh = oracle_shape(cfg)
    p64 = synth.params_to_f64(params)
    drop = None
    if cfg.dropout_p > 0:
        from oracle.dropout_oracle import Dropout
        drop = Dropout(cfg.dropout_p, seed)
    return O.stage_step([synth.to_f64(x) for x in xs], [synth.to_f64(d) for d in dys], p64, sh, drop)


def block_rel_l2(got: np.ndarray, ref: np.ndarray, block: int = 128) -> float:
    """Worst rel-L2 over blocks of `block` consecutive rows and over blocks of `block`
    consecutive columns of a matrix (the last block of each kind may be ragged): an error
    confined to one tile edge cannot hide in the norm of the whole tensor.  A block whose
    reference values are (nearly) all zero -- the query/key rows of dWqkv at sequence length 1,
    say -- is measured against the tensor's mean square instead of its own."""
    worst = 0.0
    d2 = (got - ref) ** 2
    r2 = ref ** 2
    mean_sq = float(r2.mean())
    for axis in (0, 1):
        num = d2.sum(axis=1 - axis)
        den = r2.sum(axis=1 - axis)
        edges = np.arange(0, num.shape[0], block)
        nb = np.add.reduceat(num, edges)
        db = np.add.reduceat(den, edges)
        count = np.diff(np.append(edges, num.shape[0])) * d2.shape[1 - axis]
        db = np.maximum(db, mean_sq * count)
        with np.errstate(divide="ignore", invalid="ignore"):
            q = np.sqrt(np.where(db > 0, nb / db, np.where(nb > 0, np.inf, 0.0)))
        worst = max(worst, float(q.max()))
    return worst


def compare_step(cfg, st, ys, dxs, ref, tol=None, label=""):
    """Asserts rel-L2 <= tol for every micro-batch output, every dX, every accumulated
    gradient tensor and all gradient tensors of the stage concatenated; for every [T, h]
    output and every weight-gradient matrix additionally for each block of 128 rows and
    each block of 128 columns (keys ending in "/blk"), at the same tolerance."""
    tol = TOL[cfg.dtype] if tol is None else tol
    rys, rdxs, racc = ref
    report = {}
    for m in range(len(ys)):
        for key, got, want in ((f"y[{m}]", ys[m], rys[m]), (f"dx[{m}]", dxs[m], rdxs[m])):
            g = synth.to_f64(got).reshape(want.shape)
            report[key] = O.rel_l2(g, want)
            report[key + "/blk"] = block_rel_l2(g, want)
    num = den = 0.0
    for l in range(cfg.n_layers):
        for name in B.PARAM_NAMES:
            want = racc[l][name]
            g = st.grad_view(l, name).cpu().to(torch.float64).numpy().reshape(want.shape)
            report[f"grad[{l}].{name}"] = O.rel_l2(g, want)
            if want.ndim == 2:
                report[f"grad[{l}].{name}/blk"] = block_rel_l2(g, want)
            num += float(((g - want) ** 2).sum())
            den += float((want ** 2).sum())
    report["grad[all]"] = float(np.sqrt(num / den))
    bad = {k: v for k, v in report.items() if not (v <= tol)}
    assert not bad, f"{label} rel-L2 above {tol}: {bad}"
    return report
