"""GPU parity of the stage step with dropout (attention probabilities and both residual
branches, masks regenerated from counters in forward, recompute and backward) against the
fp64 oracle with the same masks, through the C ABI."""
import pytest
import torch

from paper_2111_04007_amd import CONFIGS, binding as B, synth
from tests import parity_util as U

pytestmark = pytest.mark.gpu

SEED = (0x1234 << 32) | 0x9abcdef1


def _run(cfg, n_mb=None, seed=SEED, **kw):
    params = synth.make_params(cfg, perturb=0.05)
    xs, dys = synth.make_activations(cfg, n_mb)
    st, ys, dxs = U.gpu_stage_step(cfg, params, xs, dys, seed=seed, **kw)
    ref = U.oracle_stage_step(cfg, params, xs, dys, seed=seed)
    rep = U.compare_step(cfg, st, ys, dxs, ref, label=cfg.name)
    worst = max(rep.items(), key=lambda kv: kv[1])
    print(f"\n{cfg.name}: worst rel-L2 {worst[1]:.3e} at {worst[0]}; grad[all] {rep['grad[all]']:.3e}", flush=True)
    return st, ys, dxs


def test_dropout_c1_fp32():
    st, _, _ = _run(CONFIGS["C1"].replace(name="C1-dropout", dropout_p=0.1))
    st.close()


def test_dropout_fp32_ragged_bidirectional_high_rate():
    cfg = synth.StageConfig("ragged-f32-dropout", 2, 72, 3, 37, 3, 2, 200, False, "f32", 0.05, seed=27, dropout_p=0.4)
    st, _, _ = _run(cfg)
    st.close()


@pytest.mark.parametrize("d,causal", [(64, True), (128, False), (96, True)])
def test_dropout_bf16_small(d, causal):
    heads = {64: 4, 128: 4, 96: 2}[d]
    cfg = synth.StageConfig(f"small-bf16-d{d}-dropout", 2, heads * d, heads, 256, 2, 2, 4 * heads * d, causal, "bf16",
                            0.02, seed=28 + d, dropout_p=0.1)
    st, _, _ = _run(cfg)
    st.close()


@pytest.mark.parametrize("d,causal", [(64, False), (64, True), (96, False), (96, True), (128, False), (128, True)])
def test_dropout_bf16_long_sequence_every_kernel_variant(d, causal):
    """Every (head dim, causal) instantiation of the dropout attention kernels at a sequence
    of 8 query / 16 key blocks (the small cases above have 2 / 4), one layer, one micro-batch."""
    heads = 4
    cfg = synth.StageConfig(f"long-bf16-d{d}-{'causal' if causal else 'bidir'}-dropout", 1, heads * d, heads, 1024, 1, 1,
                            4 * heads * d, causal, "bf16", 0.02, seed=40 + d + int(causal), dropout_p=0.15)
    st, _, _ = _run(cfg)
    st.close()


def test_dropout_bf16_grouped_weight_gradients_and_interleaved_order():
    cfg = synth.StageConfig("small-bf16-dropout-g2", 2, 256, 4, 256, 2, 3, 1024, True, "bf16", 0.02, seed=31,
                            wgrad_group=2, dropout_p=0.2)
    st, _, _ = _run(cfg, interleave=True)
    st.close()


def test_dropout_c3_shape_one_microbatch():
    st, _, _ = _run(CONFIGS["C3"].replace(name="C3-dropout", dropout_p=0.1), n_mb=1)
    st.close()


def test_dropout_recompute_last_stage_and_seed_semantics():
    """The recompute pass regenerates the forward masks: forward / backward_recompute and the
    keeping forward / stored backward give bit-identical results; another seed does not; the
    seed cannot change while a slot awaits its backward."""
    cfg = synth.StageConfig("small-bf16-dropout-seed", 2, 256, 4, 256, 2, 2, 1024, True, "bf16", 0.02, seed=33, dropout_p=0.1)
    params = synth.make_params(cfg, perturb=0.05)
    xs, dys = synth.make_activations(cfg)
    st_a, ys_a, dxs_a = U.gpu_stage_step(cfg, params, xs, dys, seed=SEED)
    st_b, ys_b, dxs_b = U.gpu_stage_step(cfg, params, xs, dys, seed=SEED, last_stage=True)
    st_c, ys_c, dxs_c = U.gpu_stage_step(cfg, params, xs, dys, seed=SEED + 1)
    for m in range(len(xs)):
        assert torch.equal(ys_a[m], ys_b[m]) and torch.equal(dxs_a[m], dxs_b[m])
        assert not torch.equal(ys_a[m], ys_c[m])
    assert torch.equal(st_a.grads, st_b.grads)
    assert not torch.equal(ys_a[0], ys_a[1]) or not torch.equal(xs[0], xs[1])
    # the stored internals of forward_keep equal those of the recompute pass, bit for bit
    x0 = xs[0].cuda()
    y = torch.empty_like(x0)
    st_a.debug_forward_save(0, x0, y)
    torch.cuda.synchronize()
    saved = st_a.saved_region().clone()
    st_a.saved_region().fill_(0xA5)
    st_a.backward_recompute(0, dys[0].cuda(), torch.empty_like(x0))
    torch.cuda.synchronize()
    n = saved.numel() - cfg.tokens * cfg.hidden * 2 - 256   # the last layer's output slot is not recomputed
    assert torch.equal(saved[:n], st_a.saved_region()[:n])
    # seed changes are refused between a forward and its backward
    st_a.forward(1, x0, y)
    with pytest.raises(B.VarunaError) as ei:
        st_a.set_dropout_seed(5)
    assert ei.value.code == B.ESTATE
    st_a.backward_recompute(1, dys[0].cuda(), torch.empty_like(x0))
    st_a.set_dropout_seed(5)
    torch.cuda.synchronize()
    for s in (st_a, st_b, st_c):
        s.close()


def test_dropout_probability_validation():
    bad = synth.StageConfig("bad-dropout", 1, 64, 1, 8, 1, 1, 256, True, "f32", 0.05, dropout_p=1.0)
    with pytest.raises(B.VarunaError) as ei:
        B.query_sizes(bad)
    assert ei.value.code == B.EINVAL
