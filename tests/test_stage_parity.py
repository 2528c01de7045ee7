"""GPU parity of the whole stage step (forward, recompute + backward, accumulation)
against the fp64 oracle, through the C ABI."""
import pytest
import torch

from paper_2111_04007_amd import CONFIGS, binding as B, synth
from tests import parity_util as U

pytestmark = pytest.mark.gpu


def _run(cfg, n_mb=None, perturb=0.05, interleave=False, tol=None):
    params = synth.make_params(cfg, perturb=perturb)
    xs, dys = synth.make_activations(cfg, n_mb)
    st, ys, dxs = U.gpu_stage_step(cfg, params, xs, dys, interleave=interleave)
    ref = U.oracle_stage_step(cfg, params, xs, dys)
    rep = U.compare_step(cfg, st, ys, dxs, ref, tol=tol, label=cfg.name)
    worst = max(rep.items(), key=lambda kv: kv[1])
    print(f"\n{cfg.name}: worst rel-L2 {worst[1]:.3e} at {worst[0]}; grad[all] {rep['grad[all]']:.3e}", flush=True)
    st.close()
    return rep


def test_c1_tiny_fp32_full():
    """Config 1 exactly as specified (gamma=1, beta=0, biases 0), all 4 micro-batches."""
    _run(CONFIGS["C1"], perturb=0.0)


def test_c1_tiny_fp32_perturbed_params_interleaved_order():
    """Non-trivial gamma/beta/biases and a pipeline-like call order."""
    _run(CONFIGS["C1"], perturb=0.05, interleave=True)


def test_fp32_bidirectional_ragged_shapes():
    """Sizes that are not multiples of any tile: h=72 (d=24), s=37, b=3, f=200."""
    cfg = synth.StageConfig("ragged-f32", 2, 72, 3, 37, 3, 2, 200, False, "f32", 0.05, seed=7)
    _run(cfg)


def test_fp32_degenerate_single_token_and_single_layer():
    cfg = synth.StageConfig("s1-f32", 1, 64, 1, 1, 1, 1, 256, True, "f32", 0.05, seed=8)
    _run(cfg)


def test_bf16_small_causal_d64():
    """bf16 storage with fp32 accumulation; several GEMM tiles (T=512, h=256)."""
    cfg = synth.StageConfig("small-bf16-d64", 2, 256, 4, 256, 2, 2, 1024, True, "bf16", 0.02, seed=9)
    _run(cfg)


def test_bf16_small_bidirectional_d128():
    cfg = synth.StageConfig("small-bf16-d128", 1, 512, 4, 256, 2, 2, 2048, False, "bf16", 0.02, seed=10)
    _run(cfg)


def test_bf16_small_causal_d96_ragged_gemm():
    """h=192 (d=96): N=192/576 are not multiples of the MFMA tiles => mixed kernels."""
    cfg = synth.StageConfig("small-bf16-d96", 2, 192, 2, 128, 2, 2, 768, True, "bf16", 0.02, seed=11)
    _run(cfg)


@pytest.mark.parametrize("group,n_mb", [(2, 3), (4, 4), (3, 2)])
def test_bf16_grouped_weight_gradients(group, n_mb):
    """wgrad_group G > 1: the matrix gradients come from one GEMM per G micro-batches (plus a
    flush for a partial group); results must match the oracle like the ungrouped path."""
    cfg = synth.StageConfig("grouped-bf16", 2, 256, 4, 256, 2, n_mb, 1024, True, "bf16", 0.02, seed=12,
                            wgrad_group=group)
    _run(cfg, interleave=(group == 2))


def test_fp32_grouped_weight_gradients():
    cfg = CONFIGS["C1"].replace(wgrad_group=3)
    _run(cfg)


def test_grouped_gradients_pending_until_flush_and_dropped_by_reset():
    cfg = synth.StageConfig("grouped-f32", 1, 64, 2, 16, 1, 2, 256, True, "f32", 0.05, seed=13, wgrad_group=4)
    params = synth.make_params(cfg, perturb=0.05)
    xs, dys = synth.make_activations(cfg, 1)
    st = B.Stage(cfg)
    st.set_params(params)
    st.grad_accum_reset()
    x, dy = xs[0].cuda(), dys[0].cuda()
    y, dx = torch.empty_like(x), torch.empty_like(x)
    st.forward(0, x, y)
    st.backward_recompute(0, dy, dx)
    torch.cuda.synchronize()
    assert float(st.grad_view(0, "w1").abs().max()) == 0.0      # matrix gradient still pending
    assert float(st.grad_view(0, "b1").abs().max()) > 0.0       # vector gradients are immediate
    st.grad_flush()
    torch.cuda.synchronize()
    w1 = st.grad_view(0, "w1").clone()
    assert float(w1.abs().max()) > 0.0
    st.grad_flush()                                              # nothing pending: no-op
    torch.cuda.synchronize()
    assert torch.equal(w1, st.grad_view(0, "w1"))
    st.forward(0, x, y)
    st.backward_recompute(0, dy, dx)
    st.grad_accum_reset()                                        # drops the pending group
    st.grad_flush()
    torch.cuda.synchronize()
    assert float(st.grads.abs().max()) == 0.0
    st.close()


def test_c2_bert_large_shaped_full_step():
    """Config 2 exactly as specified: full shape (6 layers, h=1024, s=512, b=8) and all M=8
    micro-batches of the mini-batch against the oracle."""
    _run(CONFIGS["C2"], perturb=0.0)


def test_c3_gpt2_2p5b_shaped_two_microbatches():
    """Config 3 at full shape (4 layers, h=1920, d=96, s=1024, b=4), M_parity = 2, with
    non-trivial LayerNorm gains/offsets and biases so that every term is exercised at a full
    shape (the named configuration itself has gamma=1, beta=0, biases 0: see C4)."""
    _run(CONFIGS["C3"].replace(n_micro_batches=2), n_mb=2, perturb=0.05)


def test_c4_gpt_8p3b_shaped_two_microbatches():
    """Config 4 at full shape (3 layers, h=3072, d=96, s=1024, b=2), M_parity = 2."""
    _run(CONFIGS["C4"].replace(n_micro_batches=2), n_mb=2, perturb=0.0)


_C5_REF = {}


def _c5_case():
    """Seeded C5 inputs (two micro-batches) and the oracle's result for each micro-batch on its
    own (about 21 TFLOP of fp64 work each), computed once for the two tests below."""
    if not _C5_REF:
        cfg = CONFIGS["C5"].replace(n_micro_batches=2)
        params = synth.make_params(cfg, perturb=0.0)
        xs, dys = synth.make_activations(cfg, 2)
        per_mb = [U.oracle_stage_step(cfg, params, [xs[m]], [dys[m]]) for m in range(2)]
        _C5_REF.update(params=params, xs=xs, dys=dys, per_mb=per_mb)
    return _C5_REF


def _c5_compare(cfg, ms):
    c = _c5_case()
    xs, dys = [c["xs"][m] for m in ms], [c["dys"][m] for m in ms]
    st, ys, dxs = U.gpu_stage_step(cfg, c["params"], xs, dys)
    refs = [c["per_mb"][m] for m in ms]
    acc = [{k: sum(r[2][l][k] for r in refs) for k in refs[0][2][l]} for l in range(cfg.n_layers)]  # plain sum over micro-batches
    rep = U.compare_step(cfg, st, ys, dxs, ([r[0][0] for r in refs], [r[1][0] for r in refs], acc), label=cfg.name)
    worst = max(rep.items(), key=lambda kv: kv[1])
    print(f"\n{cfg.name} G={cfg.wgrad_group}: worst rel-L2 {worst[1]:.3e} at {worst[0]}; grad[all] {rep['grad[all]']:.3e}", flush=True)
    st.close()


def test_c5_200b_class_two_microbatches_grouped_weight_gradients():
    """Config 5 (the benchmarked workload) at full shape (2 layers, h=8192, d=128, s=2048,
    b=1) in the launch configuration bench.py times: two micro-batches gathered into ONE
    weight-gradient GEMM per matrix over the stacked operand rings (reduction length 2 T,
    8192 x 32768 outputs), compared with the oracle."""
    _c5_compare(CONFIGS["C5"].replace(n_micro_batches=2, wgrad_group=2), [0, 1])


def test_c5_200b_class_one_microbatch_ungrouped():
    """Config 5 as specified (weight gradients accumulated after every micro-batch), one
    micro-batch against the oracle."""
    _c5_compare(CONFIGS["C5"].replace(n_micro_batches=1, wgrad_group=1), [1])
    _C5_REF.clear()   # several GB of fp64 reference values


def test_c5_accumulation_linearity_on_gpu():
    """fp32 accumulators at full C5 shape with bench.py's group of 8: gradients after 8
    distinct micro-batches (one weight-gradient GEMM of reduction length 8 T per matrix)
    equal the sum of eight single-micro-batch runs."""
    cfg = CONFIGS["C5"].replace(n_micro_batches=8, wgrad_group=8)
    params, xs, dys = synth.device_random_stage(cfg, "cuda:0", 8)
    st = B.Stage(cfg, "cuda:0", params_flat=params)
    y = torch.empty_like(xs[0])
    dx = torch.empty_like(xs[0])

    def run(ms):
        st.grad_accum_reset()
        for m in ms:
            st.forward(m, xs[m], y)
        for m in ms:
            st.backward_recompute(m, dys[m], dx)
        st.grad_flush()
        torch.cuda.synchronize()
        return st.grads.double()

    total = run(list(range(8)))
    parts = run([0])
    for m in range(1, 8):
        parts += run([m])
    err = float((total - parts).norm() / parts.norm())
    print(f"\nC5 accumulation linearity rel-L2 {err:.3e}", flush=True)
    assert err <= 1e-6   # one 8-micro-batch GEMM vs eight single ones summed in fp64: fp32 rounding of the sums only
    st.close()


def test_recompute_equals_stored_bitwise():
    """The activations re-derived by backward_recompute are bit-identical to those a
    storing forward produced (same kernels, same launch geometry)."""
    # (the third shape has products of 384 128x128 tiles, which run on merged 128x256 tiles)
    for cfg in (CONFIGS["C1"],
                synth.StageConfig("small-bf16", 2, 256, 4, 256, 2, 2, 1024, True, "bf16", 0.02, seed=9),
                synth.StageConfig("one-8.3b-layer", 1, 3072, 24, 1024, 2, 1, 12288, True, "bf16", 0.02, seed=10)):
        params = synth.make_params(cfg, perturb=0.05)
        xs, dys = synth.make_activations(cfg, 1)
        st = B.Stage(cfg)
        st.set_params(params)
        st.grad_accum_reset()
        x, dy = xs[0].cuda(), dys[0].cuda()
        y_plain, y_save, dx = torch.empty_like(x), torch.empty_like(x), torch.empty_like(x)
        st.forward(0, x, y_plain)
        st.debug_forward_save(0, x, y_save)
        torch.cuda.synchronize()
        stored = st.saved_region().clone()
        assert torch.equal(y_plain.view(torch.uint8), y_save.view(torch.uint8))
        st.saved_region().fill_(0xA5)
        st.backward_recompute(0, dy, dx)
        torch.cuda.synchronize()
        again = st.saved_region()
        # the last layer's output slot is not recomputed (backward does not need it)
        E = cfg.tokens * cfg.hidden * (4 if cfg.dtype == "f32" else 2)
        n = stored.numel() - E - 256
        assert torch.equal(stored[:n], again[:n])
        st.close()


def test_accumulation_reset_and_determinism():
    cfg = CONFIGS["C1"]
    params = synth.make_params(cfg, perturb=0.05)
    xs, dys = synth.make_activations(cfg, 2)
    st, _, dx_a = U.gpu_stage_step(cfg, params, xs, dys)
    g_a = st.grads.clone()
    st.grad_accum_reset()
    torch.cuda.synchronize()
    assert float(st.grads.abs().max()) == 0.0
    st.close()
    st2, _, dx_b = U.gpu_stage_step(cfg, params, xs, dys)
    assert torch.equal(g_a, st2.grads)                      # run-to-run bit-identical
    assert all(torch.equal(a, b) for a, b in zip(dx_a, dx_b))
    # same micro-batch twice doubles the gradients exactly (fp32 add of equal values)
    st3, _, _ = U.gpu_stage_step(cfg, params, [xs[0], xs[0]], [dys[0], dys[0]])
    st4, _, _ = U.gpu_stage_step(cfg, params, [xs[0]], [dys[0]])
    assert torch.equal(st3.grads, 2 * st4.grads)
    for s in (st2, st3, st4):
        s.close()


@pytest.mark.parametrize("name", ["C2", "C3", "C4"])
def test_bf16_run_to_run_determinism_at_full_shape(name):
    """The bf16 path (MFMA GEMMs with split-K weight gradients, MFMA attention, bias-gradient
    sums on the side stream, grouped weight-gradient GEMMs) gives bit-identical outputs, input
    gradients and accumulated gradients on two independent runs: nothing in it adds floats
    in an order that depends on timing."""
    cfg = CONFIGS[name].replace(n_micro_batches=2, wgrad_group=2)
    params, xs, dys = synth.device_random_stage(cfg, "cuda:0", 2)

    def run(side=True):
        st = B.Stage(cfg, "cuda:0", params_flat=params)
        if side:
            st.set_side_stream(torch.cuda.Stream("cuda:0"))
        ys = [torch.empty_like(xs[0]) for _ in range(2)]
        dxs = [torch.empty_like(xs[0]) for _ in range(2)]
        st.grad_accum_reset()
        for m in range(2):
            st.forward(m, xs[m], ys[m])
        for m in range(2):
            st.backward_recompute(m, dys[m], dxs[m])
        st.grad_flush()
        torch.cuda.synchronize()
        g = st.grads.clone()
        st.close()
        return ys, dxs, g

    ya, dxa, ga = run()
    yb, dxb, gb = run()
    assert torch.isfinite(ga).all()
    assert torch.equal(ga, gb)
    assert all(torch.equal(a, b) for a, b in zip(ya + dxa, yb + dxb))
    yc, dxc, gc = run(side=False)     # everything on the caller's stream: the same bits
    assert torch.equal(ga, gc)
    assert all(torch.equal(a, b) for a, b in zip(ya + dxa, yc + dxc))


def test_state_error_after_consumed_slot():
    cfg = CONFIGS["C1"]
    st = B.Stage(cfg)
    x = torch.zeros(cfg.tokens, cfg.hidden, device="cuda")
    y = torch.empty_like(x)
    st.forward(1, x, y)
    st.backward_recompute(1, x, y)
    with pytest.raises(B.VarunaError) as ei:
        st.backward_recompute(1, x, y)
    assert ei.value.code == B.ESTATE
    st.close()
