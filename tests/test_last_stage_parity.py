"""GPU parity of the last-stage variant (forward that keeps the internals, backward
without recompute) against the fp64 oracle and, bit for bit, against the
forward / backward_recompute pair, through the C ABI."""
import pytest
import torch

from paper_2111_04007_amd import CONFIGS, binding as B, synth
from tests import parity_util as U

pytestmark = pytest.mark.gpu


def _both(cfg, n_mb=None, perturb=0.05):
    params = synth.make_params(cfg, perturb=perturb)
    xs, dys = synth.make_activations(cfg, n_mb)
    st_l, ys_l, dxs_l = U.gpu_stage_step(cfg, params, xs, dys, last_stage=True)
    ref = U.oracle_stage_step(cfg, params, xs, dys)
    rep = U.compare_step(cfg, st_l, ys_l, dxs_l, ref, label=cfg.name + " last-stage")
    st_r, ys_r, dxs_r = U.gpu_stage_step(cfg, params, xs, dys)
    for m in range(len(xs)):
        assert torch.equal(ys_l[m], ys_r[m]), f"y[{m}] differs from the recompute path"
        assert torch.equal(dxs_l[m], dxs_r[m]), f"dx[{m}] differs from the recompute path"
    assert torch.equal(st_l.grads, st_r.grads), "accumulated gradients differ from the recompute path"
    worst = max(rep.items(), key=lambda kv: kv[1])
    print(f"\n{cfg.name} last-stage: worst rel-L2 {worst[1]:.3e} at {worst[0]}", flush=True)
    st_l.close()
    st_r.close()


def test_last_stage_c1_fp32():
    _both(CONFIGS["C1"])


def test_last_stage_fp32_ragged():
    _both(synth.StageConfig("ragged-f32-last", 2, 72, 3, 37, 3, 2, 200, False, "f32", 0.05, seed=17))


def test_last_stage_bf16_small():
    _both(synth.StageConfig("small-bf16-last", 2, 256, 4, 256, 2, 3, 1024, True, "bf16", 0.02, seed=18))


def test_last_stage_bf16_grouped_weight_gradients():
    cfg = synth.StageConfig("small-bf16-last-g2", 2, 256, 4, 256, 2, 3, 1024, True, "bf16", 0.02, seed=19, wgrad_group=2)
    _both(cfg)


def test_last_stage_c3_shape_one_microbatch():
    _both(CONFIGS["C3"], n_mb=1)


def test_backward_stored_needs_adjacent_forward_keep():
    cfg = CONFIGS["C1"]
    params = synth.make_params(cfg, perturb=0.05)
    xs, dys = synth.make_activations(cfg, 2)
    dev = "cuda:0"
    st = B.Stage(cfg, dev)
    st.set_params(params)
    st.grad_accum_reset()
    x = [t.to(dev) for t in xs]
    dy = [t.to(dev) for t in dys]
    y = torch.empty_like(x[0])
    dx = torch.empty_like(x[0])

    def expect_estate(mb):
        with pytest.raises(B.VarunaError) as ei:
            st.backward_stored(mb, dy[mb], dx)
        assert ei.value.code == B.ESTATE

    st.forward(0, x[0], y)
    expect_estate(0)                       # plain forward keeps nothing
    st.forward_keep(0, x[0], y)
    expect_estate(1)                       # other micro-batch
    st.forward(1, x[1], y)                 # a plain forward of another slot does not disturb
    st.backward_stored(0, dy[0], dx)
    expect_estate(0)                       # consumed
    st.forward_keep(0, x[0], y)
    st.backward_recompute(1, dy[1], dx)    # recompute overwrites the kept activations
    expect_estate(0)
    st.forward_keep(0, x[0], y)
    st.grad_accum_reset()
    expect_estate(0)
    torch.cuda.synchronize()
    st.close()
