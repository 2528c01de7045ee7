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


def gpu_stage_step(cfg, params, xs, dys, device="cuda:0", interleave=False, last_stage=False, seed=0):
    """Runs reset, M forwards, M backward_recomputes (last_stage: M times forward_keep
    followed at once by backward_stored). Returns (stage, ys, dxs) with outputs as CPU
    tensors; the accumulated gradients stay in stage.grads."""
    st = B.Stage(cfg, device)
    st.set_params(params)
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


def compare_step(cfg, st, ys, dxs, ref, tol=None, label=""):
    """Asserts rel-L2 <= tol for every micro-batch output, every dX and the
    accumulated gradients (each matrix, and all tensors of the stage concatenated;
    small-norm vectors are checked against the norm scale of their matrix)."""
    tol = TOL[cfg.dtype] if tol is None else tol
    rys, rdxs, racc = ref
    report = {}
    for m in range(len(ys)):
        report[f"y[{m}]"] = O.rel_l2(synth.to_f64(ys[m]), rys[m])
        report[f"dx[{m}]"] = O.rel_l2(synth.to_f64(dxs[m]), rdxs[m])
    got_all, ref_all = [], []
    for l in range(cfg.n_layers):
        for name in B.PARAM_NAMES:
            g = st.grad_view(l, name).cpu().to(torch.float64).numpy().reshape(racc[l][name].shape)
            report[f"grad[{l}].{name}"] = O.rel_l2(g, racc[l][name])
            got_all.append(g.ravel())
            ref_all.append(racc[l][name].ravel())
    report["grad[all]"] = O.rel_l2(np.concatenate(got_all), np.concatenate(ref_all))
    bad = {k: v for k, v in report.items() if not (v <= tol)}
    assert not bad, f"{label} rel-L2 above {tol}: {bad}"
    return report
