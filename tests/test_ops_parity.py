"""GPU parity of the individual kernels (GEMM variants and epilogues, LayerNorm,
column reductions, attention) against the fp64 oracle's pieces."""
import numpy as np
import pytest
import torch

from oracle import stage_oracle as O
from paper_2111_04007_amd import binding as B
from paper_2111_04007_amd.synth import to_f64

pytestmark = pytest.mark.gpu

DT = {"f32": torch.float32, "bf16": torch.bfloat16}
TOL = {"f32": 1e-5, "bf16": 2e-2}


def rnd(shape, dtype, seed, scale=1.0):
    g = np.random.Generator(np.random.Philox(key=[seed, 99]))
    return torch.from_numpy(g.standard_normal(shape) * scale).to(DT[dtype]).cuda()


def run_gemm_case(dtype, M, N, K, variant, seed=1):
    """All six op/epilogue combinations for one shape and kernel configuration."""
    x = rnd((M, K), dtype, seed)                # forward input / dgrad dY has shape [M,K]
    w = rnd((N, K), dtype, seed + 1, 0.05)      # forward weight [N,K]
    bias = rnd((N,), dtype, seed + 2, 0.5)
    res = rnd((M, N), dtype, seed + 3)
    x64, w64, b64, r64 = map(to_f64, (x, w, bias, res))
    tol = TOL[dtype]
    out = torch.empty((M, N), dtype=DT[dtype], device="cuda")
    aux = torch.empty_like(out)
    # forward, bias
    B.op_gemm(B.OP_FWD, 0, x, w, out, bias=bias, variant=variant, M=M, N=N, K=K)
    assert O.rel_l2(to_f64(out), O.linear_forward(x64, w64, b64)) <= tol
    # forward, bias + GeLU, also storing u
    B.op_gemm(B.OP_FWD, 1, x, w, out, bias=bias, aux_out=aux, variant=variant, M=M, N=N, K=K)
    u64 = O.linear_forward(x64, w64, b64)
    assert O.rel_l2(to_f64(aux), u64) <= tol
    assert O.rel_l2(to_f64(out), O.gelu_tanh(u64)) <= tol
    # forward, bias + residual
    B.op_gemm(B.OP_FWD, 2, x, w, out, bias=bias, aux_in=res, variant=variant, M=M, N=N, K=K)
    assert O.rel_l2(to_f64(out), r64 + O.linear_forward(x64, w64, b64)) <= tol
    # dgrad: dX[M,N] = dY[M,K] W[K,N]
    wd = rnd((K, N), dtype, seed + 4, 0.05)
    B.op_gemm(B.OP_DGRAD, 0, x, wd, out, variant=variant, M=M, N=N, K=K)
    ref = x64 @ to_f64(wd)
    assert O.rel_l2(to_f64(out), ref) <= tol
    B.op_gemm(B.OP_DGRAD, 3, x, wd, out, aux_in=res, variant=variant, M=M, N=N, K=K)
    assert O.rel_l2(to_f64(out), ref * O.gelu_tanh_grad(r64)) <= tol
    # wgrad: dW[M,N] += dY[K,M]^T X[K,N], twice to see the accumulation
    dy = rnd((K, M), dtype, seed + 5)
    xx = rnd((K, N), dtype, seed + 6)
    acc = torch.full((M, N), 0.5, dtype=torch.float32, device="cuda")
    for _ in range(2):
        B.op_gemm(B.OP_WGRAD, 0, dy, xx, acc, variant=variant, M=M, N=N, K=K)
    _, dw, _ = O.linear_backward(to_f64(dy), to_f64(xx), np.zeros((M, N)))
    assert O.rel_l2(to_f64(acc), 0.5 + 2 * dw) <= tol
    torch.cuda.synchronize()


@pytest.mark.parametrize("shape", [(128, 384, 128), (70, 45, 33), (1, 1, 1), (65, 64, 17)])
def test_gemm_fp32(shape):
    run_gemm_case("f32", *shape, variant=0)


@pytest.mark.parametrize("shape", [(96, 200, 72), (64, 8, 40)])
def test_gemm_bf16_simple_kernel(shape):
    run_gemm_case("bf16", *shape, variant=-1)


@pytest.mark.parametrize("variant,shape", [
    (5, (512, 768, 256)), (6, (512, 768, 256)), (7, (384, 640, 320)), (8, (512, 384, 192)),
    (5, (256, 256, 64)), (7, (128, 128, 64)), (7, (256, 128, 128)), (6, (256, 512, 192)),
    (9, (512, 768, 256)), (9, (256, 256, 64)), (9, (256, 512, 128)), (9, (512, 256, 448)),
    (10, (384, 640, 320)), (10, (128, 128, 64)), (10, (256, 128, 192)),
    (11, (512, 768, 256)), (11, (256, 256, 64)),
    (12, (512, 768, 256)), (12, (256, 256, 64)), (12, (256, 512, 128)), (12, (512, 256, 448)),
    (13, (512, 768, 256)), (13, (256, 256, 64)), (13, (256, 512, 192)),
    (14, (384, 640, 320)), (14, (128, 128, 64)), (14, (256, 128, 192)),
    (15, (384, 768, 320)), (15, (128, 256, 64)), (15, (256, 512, 192)),
    (16, (768, 384, 320)), (16, (256, 128, 64)), (16, (512, 256, 192)),
    (17, (512, 768, 256)), (17, (256, 256, 64)), (17, (256, 512, 448)), (17, (256, 256, 832)),
    (18, (512, 768, 256)), (18, (256, 256, 64)), (18, (256, 512, 448)), (18, (256, 256, 832)),
    (19, (384, 640, 320)), (19, (128, 128, 64)), (19, (256, 128, 448)), (19, (128, 256, 832)),
    (20, (384, 768, 320)), (20, (128, 256, 64)), (20, (256, 512, 448)),
    (21, (768, 384, 320)), (21, (256, 128, 64)), (21, (512, 256, 448)),
])
def test_gemm_bf16_mfma_variants(variant, shape):
    """Each MFMA tile configuration on several tiles, k-steps and a single-k-step case."""
    run_gemm_case("bf16", *shape, variant=variant, seed=variant)


def test_gemm_bf16_auto_choice_and_unsupported_variant():
    run_gemm_case("bf16", 512, 1024, 512, variant=0)
    a = rnd((100, 64), "bf16", 1)
    w = rnd((128, 64), "bf16", 2)
    out = torch.empty((100, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(B.VarunaError) as ei:
        B.op_gemm(B.OP_FWD, 0, a, w, out, bias=w[0].contiguous(), variant=7, M=100, N=128, K=64)
    assert ei.value.code == B.EUNSUPPORTED


@pytest.mark.parametrize("dtype,rows,h", [("f32", 130, 128), ("f32", 5, 37), ("bf16", 257, 1024), ("bf16", 9, 100)])
def test_layernorm_fwd_bwd(dtype, rows, h):
    x = rnd((rows, h), dtype, 3, 2.0) + 0.5
    gamma = (rnd((h,), dtype, 4, 0.2) + 1.0).to(DT[dtype])
    beta = rnd((h,), dtype, 5, 0.2)
    y = torch.empty_like(x)
    stats = torch.empty(2 * rows, dtype=torch.float32, device="cuda")
    B.op_layernorm_fwd(x, gamma, beta, y, stats)
    y64, xhat, rstd = O.layernorm_forward(to_f64(x), to_f64(gamma), to_f64(beta), 1e-5)
    tol = TOL[dtype]
    assert O.rel_l2(to_f64(y), y64) <= tol
    assert O.rel_l2(to_f64(stats[:rows]), to_f64(x).mean(axis=1)) <= 1e-5
    assert O.rel_l2(to_f64(stats[rows:]), rstd[:, 0]) <= 1e-5
    dy = rnd((rows, h), dtype, 6)
    res = rnd((rows, h), dtype, 7)
    dx = torch.empty_like(x)
    dg = torch.full((h,), 0.25, dtype=torch.float32, device="cuda")
    db = torch.full((h,), -0.25, dtype=torch.float32, device="cuda")
    partial = torch.empty(B.colreduce_scratch_bytes(rows, 2 * h) // 4, dtype=torch.float32, device="cuda")
    B.op_layernorm_bwd(dy, x, stats, gamma, res, dx, dg, db, partial)
    dx64, dg64, db64 = O.layernorm_backward(to_f64(dy), xhat, rstd, to_f64(gamma))
    assert O.rel_l2(to_f64(dx), to_f64(res) + dx64) <= tol
    assert O.rel_l2(to_f64(dg), 0.25 + dg64) <= max(tol, 1e-5) * (1 if dtype == "f32" else 0.1)
    assert O.rel_l2(to_f64(db), -0.25 + db64) <= max(tol, 1e-5) * (1 if dtype == "f32" else 0.1)


@pytest.mark.parametrize("dtype,rows,n", [("f32", 300, 70), ("bf16", 1025, 384), ("bf16", 3, 8)])
def test_colsum(dtype, rows, n):
    a = rnd((rows, n), dtype, 8)
    out = torch.full((n,), 1.0, dtype=torch.float32, device="cuda")
    partial = torch.empty(B.colreduce_scratch_bytes(rows, n) // 4, dtype=torch.float32, device="cuda")
    B.op_colsum(a, out, partial)
    assert O.rel_l2(to_f64(out), 1.0 + to_f64(a).sum(axis=0)) <= 1e-5


def run_attention_case(dtype, b, s, heads, d, causal, variant, seed=20, key_ramp=None):
    h = heads * d
    sh = O.StageShape(1, h, heads, s, b, 4 * h, bool(causal))
    qkv = rnd((b * s, 3 * h), dtype, seed, 1.0)
    if key_ramp is not None:   # keys grow along the sequence: row maxima keep rising from key block to key block
        pos = torch.arange(b * s, device="cuda") % s
        ramp = key_ramp[0] + (key_ramp[1] - key_ramp[0]) * pos.to(torch.float32) / max(1, s - 1)
        qkv[:, h:2 * h] = (qkv[:, h:2 * h].float() * ramp[:, None]).to(qkv.dtype)
    dctx = rnd((b * s, h), dtype, seed + 1)
    ctx = torch.empty((b * s, h), dtype=DT[dtype], device="cuda")
    lse = torch.empty(b * heads * s, dtype=torch.float32, device="cuda")
    B.op_attention_fwd(qkv, ctx, lse, b, s, heads, d, causal, variant=variant)
    ctx64, probs = O.attention_forward(to_f64(qkv), sh)
    tol = TOL[dtype]
    assert O.rel_l2(to_f64(ctx), ctx64) <= tol
    # log-sum-exp of the scaled, masked scores (natural log)
    q64 = to_f64(qkv)
    want = np.empty((b, heads, s))
    for bi in range(b):
        for j in range(heads):
            q = q64[bi * s:(bi + 1) * s, j * d:(j + 1) * d]
            k = q64[bi * s:(bi + 1) * s, h + j * d:h + (j + 1) * d]
            sc = q @ k.T / np.sqrt(d)
            if causal:
                sc = np.where(np.triu(np.ones((s, s), bool), 1), -np.inf, sc)
            mx = sc.max(axis=1)
            want[bi, j] = mx + np.log(np.exp(sc - mx[:, None]).sum(axis=1))
    assert np.abs(to_f64(lse).reshape(b, heads, s) - want).max() <= (1e-4 if dtype == "f32" else 2e-2)
    dqkv = torch.empty_like(qkv)
    delta = torch.empty_like(lse)
    B.op_attention_bwd(qkv, ctx, lse, dctx, dqkv, delta, b, s, heads, d, causal, variant=variant)
    ref = O.attention_backward(to_f64(dctx), q64, probs, sh)
    got = to_f64(dqkv)
    for part, name in ((slice(0, h), "dq"), (slice(h, 2 * h), "dk"), (slice(2 * h, 3 * h), "dv")):
        if np.linalg.norm(ref[:, part]) > 0:
            assert O.rel_l2(got[:, part], ref[:, part]) <= tol, name
        else:   # s = 1: dQ and dK are exactly zero; measure against the scale of the whole gradient
            assert np.linalg.norm(got[:, part]) <= tol * np.linalg.norm(ref), name
    torch.cuda.synchronize()


@pytest.mark.parametrize("b,s,heads,d,causal", [(2, 64, 2, 64, 1), (3, 37, 3, 24, 0), (1, 1, 1, 8, 1), (1, 130, 2, 96, 1)])
def test_attention_fp32(b, s, heads, d, causal):
    run_attention_case("f32", b, s, heads, d, causal, variant=0)


@pytest.mark.parametrize("b,s,heads,d,causal", [(2, 128, 2, 64, 1), (1, 200, 2, 96, 0), (1, 256, 1, 128, 1)])
def test_attention_bf16_simple(b, s, heads, d, causal):
    run_attention_case("bf16", b, s, heads, d, causal, variant=-1)


@pytest.mark.parametrize("b,s,heads,d,causal", [
    (2, 128, 2, 64, 1), (1, 256, 2, 64, 0), (1, 384, 1, 96, 1), (2, 256, 1, 96, 0),
    (1, 256, 2, 128, 1), (1, 128, 1, 128, 0), (1, 512, 1, 128, 1),
])
def test_attention_bf16_mfma(b, s, heads, d, causal):
    """MFMA kernels: every head dim, causal and bidirectional, 1 to 4 query/key blocks."""
    run_attention_case("bf16", b, s, heads, d, causal, variant=1, seed=30 + d)


@pytest.mark.parametrize("b,s,heads,d,causal", [(1, 512, 2, 64, 0), (1, 512, 1, 128, 1), (1, 384, 1, 96, 0)])
def test_attention_bf16_mfma_rising_row_maxima(b, s, heads, d, causal):
    """Keys whose norm grows 8x along the sequence: the scores of later key blocks exceed the
    earlier maxima by more than 2^8 for many rows and by less for others, so both branches of
    the forward kernel's thresholded online-softmax rescale run after the first block."""
    run_attention_case("bf16", b, s, heads, d, causal, variant=1, seed=70 + d, key_ramp=(0.5, 4.0))


def test_attention_mfma_rejects_unsupported_shape():
    qkv = rnd((100, 3 * 64), "bf16", 1)
    ctx = torch.empty((100, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(B.VarunaError) as ei:
        B.op_attention_fwd(qkv, ctx, None, 1, 100, 1, 64, 1, variant=1)
    assert ei.value.code == B.EUNSUPPORTED


@pytest.mark.parametrize("variant", [12, 13, 14, 9, 15, 16, 17, 18, 19, 20, 21])
def test_gemm_bit_stable_under_memory_contention(variant):
    """The kernels that keep loads in flight across a barrier must not let a k-tile be read
    before it has landed when memory latency rises (a wait that counted loads past the end of
    the reduction as outstanding once let the last k-tiles through early; the whole-step
    determinism tests are what caught it).  The same product is repeated while a second stream
    keeps HBM busy with copies; every repetition must be bit-identical to the first, for
    reductions of 1, 2, 3 and many k-tiles and all three operand layouts."""
    side = torch.cuda.Stream()
    big = torch.empty(1 << 28, dtype=torch.uint8, device="cuda")
    big2 = torch.empty_like(big)
    M, N = 1024, 1536
    for K in (64, 128, 192, 1024):
        x = rnd((M, K), "bf16", 40 + K)
        w = rnd((N, K), "bf16", 41 + K, 0.05)
        wd = rnd((K, N), "bf16", 42 + K, 0.05)
        dy = rnd((K, M), "bf16", 43 + K)
        xx = rnd((K, N), "bf16", 44 + K)
        bias = rnd((N,), "bf16", 45 + K, 0.5)
        torch.cuda.synchronize()

        def products():
            o1 = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
            o2 = torch.empty_like(o1)
            o3 = torch.zeros((M, N), dtype=torch.float32, device="cuda")
            B.op_gemm(B.OP_FWD, 0, x, w, o1, bias=bias, variant=variant, M=M, N=N, K=K)
            B.op_gemm(B.OP_DGRAD, 0, x, wd, o2, variant=variant, M=M, N=N, K=K)
            B.op_gemm(B.OP_WGRAD, 0, dy, xx, o3, variant=variant, M=M, N=N, K=K)
            return o1, o2, o3

        ref = products()
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            for _ in range(12):
                big2.copy_(big, non_blocking=True)
        outs = [products() for _ in range(8)]
        torch.cuda.synchronize()
        for o in outs:
            for got, want in zip(o, ref):
                assert torch.equal(got, want), (variant, K)


@pytest.mark.parametrize("variant", [5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15, 16, 17, 18, 19, 20, 21])
def test_gemm_bf16_variants_to_rounding_accuracy(variant):
    """The whole-stage tolerance (2e-2) would hide a k-tile read before it landed or dropped from
    a long reduction.  Here every kernel configuration is held to what its arithmetic allows: the
    fp32 weight-gradient accumulator to 1e-5, bf16 outputs to the rounding of the output itself
    (rel-L2 about 2^-9 / sqrt(3) = 1.1e-3), for reductions of 1 to 16 k-tiles."""
    M, N = 512, 768
    for K in (64, 128, 192, 256, 320, 384, 448, 1024):
        x = rnd((M, K), "bf16", 60 + K)
        w = rnd((N, K), "bf16", 61 + K, 0.05)
        wd = rnd((K, N), "bf16", 62 + K, 0.05)
        dy = rnd((K, M), "bf16", 63 + K)
        xx = rnd((K, N), "bf16", 64 + K)
        bias = rnd((N,), "bf16", 65 + K, 0.5)
        out = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        B.op_gemm(B.OP_FWD, 0, x, w, out, bias=bias, variant=variant, M=M, N=N, K=K)
        assert O.rel_l2(to_f64(out), O.linear_forward(to_f64(x), to_f64(w), to_f64(bias))) <= 2.5e-3, K
        B.op_gemm(B.OP_DGRAD, 0, x, wd, out, variant=variant, M=M, N=N, K=K)
        assert O.rel_l2(to_f64(out), to_f64(x) @ to_f64(wd)) <= 2.5e-3, K
        acc = torch.zeros((M, N), dtype=torch.float32, device="cuda")
        B.op_gemm(B.OP_WGRAD, 0, dy, xx, acc, variant=variant, M=M, N=N, K=K)
        assert O.rel_l2(to_f64(acc), to_f64(dy).T @ to_f64(xx)) <= 1e-5, K
