"""Pins for the fp64 oracle: each check ties it to something other than itself
(finite differences, library routines, closed forms, invariants, brute force)."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import stage_oracle as O


def tiny_shape(causal=True, L=2, h=8, a=2, s=5, b=2, f=16):
    return O.StageShape(L, h, a, s, b, f, causal, 1e-5)


def rand_params(sh, rng, scale=0.3):
    ps = []
    for _ in range(sh.n_layers):
        p = {}
        for k, shp in O.param_shapes(sh).items():
            p[k] = rng.standard_normal(shp) * scale
            if k.endswith("_g"):
                p[k] = 1.0 + p[k]
        ps.append(p)
    return ps


# ---------------------------------------------------------------- gradients
@pytest.mark.parametrize("causal", [True, False])
def test_finite_difference_all_gradients(causal):
    """Central differences on a tiny 2-layer stage: every parameter gradient
    entry and every dX entry (scalar loss = sum(y * R), so dy = R)."""
    rng = np.random.default_rng(7)
    sh = tiny_shape(causal)
    ps = rand_params(sh, rng)
    x = rng.standard_normal((sh.tokens, sh.hidden))
    R = rng.standard_normal((sh.tokens, sh.hidden))

    def loss(xv, pv):
        y, _ = O.stage_forward(xv, pv, sh)
        return float((y * R).sum())

    y, caches = O.stage_forward(x, ps, sh)
    dx, grads = O.stage_backward(R, ps, caches, sh)

    def fd(arr, idx):
        old = arr[idx]
        step = 1e-6 * max(1.0, abs(old))
        arr[idx] = old + step
        lp = loss(x, ps)
        arr[idx] = old - step
        lm = loss(x, ps)
        arr[idx] = old
        return (lp - lm) / (2 * step)

    for l in range(sh.n_layers):
        for k in O.PARAM_NAMES:
            num = np.zeros_like(ps[l][k])
            for idx in np.ndindex(*ps[l][k].shape):
                num[idx] = fd(ps[l][k], idx)
            err = np.linalg.norm(num - grads[l][k]) / max(np.linalg.norm(num), 1e-12)
            assert err < 1e-6, (l, k, err)
    num = np.zeros_like(x)
    for idx in np.ndindex(*x.shape):
        num[idx] = fd(x, idx)
    assert np.linalg.norm(num - dx) / np.linalg.norm(num) < 1e-6


def _torch_layer(x, p, sh):
    """The same block composed from torch library routines (fp64, autograd)."""
    h, a, d, s, b = sh.hidden, sh.n_heads, sh.head_dim, sh.seq_len, sh.micro_batch
    xn1 = F.layer_norm(x, (h,), p["ln1_g"], p["ln1_b"], sh.ln_eps)
    qkv = F.linear(xn1, p["wqkv"], p["bqkv"])
    q, k, v = qkv.split(h, dim=1)
    sp = lambda t: t.reshape(b, s, a, d).permute(0, 2, 1, 3)
    ctx = F.scaled_dot_product_attention(sp(q), sp(k), sp(v), is_causal=sh.causal)
    ctx = ctx.permute(0, 2, 1, 3).reshape(b * s, h)
    x1 = x + F.linear(ctx, p["wo"], p["bo"])
    xn2 = F.layer_norm(x1, (h,), p["ln2_g"], p["ln2_b"], sh.ln_eps)
    g = F.gelu(F.linear(xn2, p["w1"], p["b1"]), approximate="tanh")
    return x1 + F.linear(g, p["w2"], p["b2"])


@pytest.mark.parametrize("causal", [True, False])
def test_against_torch_library_autograd(causal):
    """Whole stage step (2 micro-batches) vs torch's own layer_norm / linear /
    scaled_dot_product_attention / gelu with autograd, all in fp64."""
    rng = np.random.default_rng(11)
    sh = O.StageShape(2, 32, 4, 12, 2, 64, causal, 1e-5)
    ps = rand_params(sh, rng, 0.2)
    xs = [rng.standard_normal((sh.tokens, sh.hidden)) for _ in range(2)]
    dys = [rng.standard_normal((sh.tokens, sh.hidden)) for _ in range(2)]
    ys, dxs, acc = O.stage_step(xs, dys, ps, sh)

    tps = [{k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in p.items()} for p in ps]
    for m in range(2):
        xt = torch.tensor(xs[m], dtype=torch.float64, requires_grad=True)
        yt = xt
        for p in tps:
            yt = _torch_layer(yt, p, sh)
        yt.backward(torch.tensor(dys[m]))
        assert O.rel_l2(ys[m], yt.detach().numpy()) < 1e-12
        assert O.rel_l2(dxs[m], xt.grad.numpy()) < 1e-11
    for l in range(sh.n_layers):
        for k in O.PARAM_NAMES:
            assert O.rel_l2(acc[l][k], tps[l][k].grad.numpy()) < 1e-11, (l, k)


# ------------------------------------------------------------------ softmax
@pytest.mark.parametrize("causal", [True, False])
def test_softmax_rows_sum_to_one_and_mask(causal):
    rng = np.random.default_rng(3)
    sh = tiny_shape(causal, s=9)
    qkv = rng.standard_normal((sh.tokens, 3 * sh.hidden)) * 3
    _, probs = O.attention_forward(qkv, sh)
    assert len(probs) == sh.micro_batch * sh.n_heads
    for p in probs.values():
        assert np.all(p >= 0)
        assert np.abs(p.sum(axis=1) - 1).max() < 1e-14
        if causal:
            assert np.all(np.triu(p, 1) == 0.0)
            assert np.all(np.diag(p) > 0)
        else:
            assert np.all(p > 0)


def test_causal_forward_future_independence():
    """Perturbing token t' leaves stage outputs at tokens < t' bit-identical."""
    rng = np.random.default_rng(5)
    sh = tiny_shape(True, s=7)
    ps = rand_params(sh, rng)
    x = rng.standard_normal((sh.tokens, sh.hidden))
    y0, _ = O.stage_forward(x, ps, sh)
    tp = 4
    x2 = x.copy()
    x2[tp] += 1.0           # batch element 0, position 4
    y1, _ = O.stage_forward(x2, ps, sh)
    assert np.array_equal(y0[:tp], y1[:tp])
    assert not np.array_equal(y0[tp:sh.seq_len], y1[tp:sh.seq_len])
    assert np.array_equal(y0[sh.seq_len:], y1[sh.seq_len:])   # other batch element


@pytest.mark.parametrize("causal", [True, False])
def test_gradient_into_future_tokens(causal):
    """dy non-zero only at position t: causal => dX at positions > t is exactly
    zero; bidirectional => non-zero."""
    rng = np.random.default_rng(6)
    sh = tiny_shape(causal, s=7)
    ps = rand_params(sh, rng)
    x = rng.standard_normal((sh.tokens, sh.hidden))
    _, caches = O.stage_forward(x, ps, sh)
    t = 3
    dy = np.zeros((sh.tokens, sh.hidden))
    dy[t] = rng.standard_normal(sh.hidden)
    dx, _ = O.stage_backward(dy, ps, caches, sh)
    fut = dx[t + 1:sh.seq_len]
    if causal:
        assert np.all(fut == 0.0)
    else:
        assert np.abs(fut).min() > 0
    assert np.all(dx[sh.seq_len:] == 0.0)      # other batch element untouched
    assert np.abs(dx[:t + 1]).max() > 0


# -------------------------------------------------------------- closed forms
@pytest.mark.parametrize("causal", [True, False])
def test_zero_query_gives_mean_of_values(causal):
    rng = np.random.default_rng(8)
    sh = tiny_shape(causal, s=6)
    h, s = sh.hidden, sh.seq_len
    qkv = rng.standard_normal((sh.tokens, 3 * h))
    qkv[:, :h] = 0.0
    ctx, _ = O.attention_forward(qkv, sh)
    v = qkv[:, 2 * h:]
    for bi in range(sh.micro_batch):
        vb = v[bi * s:(bi + 1) * s]
        for i in range(s):
            want = vb[:i + 1].mean(axis=0) if causal else vb.mean(axis=0)
            assert np.allclose(ctx[bi * s + i], want, atol=1e-14)


def test_attention_seq_len_one_returns_v():
    rng = np.random.default_rng(9)
    sh = O.StageShape(1, 8, 2, 1, 3, 16, True)
    qkv = rng.standard_normal((sh.tokens, 24))
    ctx, _ = O.attention_forward(qkv, sh)
    assert np.allclose(ctx, qkv[:, 16:], atol=0)


def test_attention_brute_force_loops():
    """Scalar triple loops of the definition, heads and batch laid out by hand:
    catches a wrong head/column slice or a transposed operand."""
    rng = np.random.default_rng(10)
    sh = O.StageShape(1, 6, 3, 4, 2, 8, True)
    h, d, s = 6, 2, 4
    qkv = rng.standard_normal((sh.tokens, 18))
    dctx = rng.standard_normal((sh.tokens, h))
    ctx, probs = O.attention_forward(qkv, sh)
    dqkv = O.attention_backward(dctx, qkv, probs, sh)
    want = np.zeros_like(ctx)
    P = np.zeros((2, 3, s, s))
    for b in range(2):
        for j in range(3):
            for i in range(s):
                sc = [sum(qkv[b * s + i, j * d + e] * qkv[b * s + k, h + j * d + e] for e in range(d)) / math.sqrt(d)
                      for k in range(i + 1)]
                mx = max(sc)
                ex = [math.exp(v - mx) for v in sc]
                z = sum(ex)
                for k in range(i + 1):
                    P[b, j, i, k] = ex[k] / z
                    for e in range(d):
                        want[b * s + i, j * d + e] += P[b, j, i, k] * qkv[b * s + k, 2 * h + j * d + e]
    assert np.allclose(ctx, want, atol=1e-14)
    wd = np.zeros_like(qkv)
    for b in range(2):
        for j in range(3):
            for i in range(s):
                dp = [sum(dctx[b * s + i, j * d + e] * qkv[b * s + k, 2 * h + j * d + e] for e in range(d)) for k in range(s)]
                dot = sum(P[b, j, i, k] * dp[k] for k in range(s))
                for k in range(s):
                    ds = P[b, j, i, k] * (dp[k] - dot)
                    for e in range(d):
                        wd[b * s + i, j * d + e] += ds * qkv[b * s + k, h + j * d + e] / math.sqrt(d)
                        wd[b * s + k, h + j * d + e] += ds * qkv[b * s + i, j * d + e] / math.sqrt(d)
                        wd[b * s + k, 2 * h + j * d + e] += P[b, j, i, k] * dctx[b * s + i, j * d + e]
    assert np.allclose(dqkv, wd, atol=1e-13)


def test_head_and_batch_permutation_equivariance():
    rng = np.random.default_rng(12)
    sh = tiny_shape(True, h=12, a=3, s=5, b=2)
    h, d, s = sh.hidden, sh.head_dim, sh.seq_len
    qkv = rng.standard_normal((sh.tokens, 3 * h))
    ctx, _ = O.attention_forward(qkv, sh)
    perm = [2, 0, 1]
    cols = np.concatenate([np.arange(j * d, (j + 1) * d) for j in perm])
    qkv_p = np.concatenate([qkv[:, cols], qkv[:, h + cols], qkv[:, 2 * h + cols]], axis=1)
    ctx_p, _ = O.attention_forward(qkv_p, sh)
    assert np.array_equal(ctx_p, ctx[:, cols])
    swap = np.concatenate([np.arange(s, 2 * s), np.arange(0, s)])
    ctx_s, _ = O.attention_forward(qkv[swap], sh)
    assert np.array_equal(ctx_s, ctx[swap])


def test_zero_output_weights_make_identity():
    """Wo = bo = W2 = b2 = 0  =>  y = x and dX = dy exactly."""
    rng = np.random.default_rng(13)
    sh = tiny_shape(True)
    ps = rand_params(sh, rng)
    for p in ps:
        for k in ("wo", "bo", "w2", "b2"):
            p[k][...] = 0.0
    x = rng.standard_normal((sh.tokens, sh.hidden))
    dy = rng.standard_normal((sh.tokens, sh.hidden))
    y, c = O.stage_forward(x, ps, sh)
    dx, _ = O.stage_backward(dy, ps, c, sh)
    assert np.array_equal(y, x)
    assert np.array_equal(dx, dy)


# ---------------------------------------------------------------- LayerNorm
def test_layernorm_identities():
    rng = np.random.default_rng(14)
    x = rng.standard_normal((6, 10)) * 2 + 1
    g = rng.standard_normal(10)
    b = rng.standard_normal(10)
    eps = 1e-5
    y, xhat, rstd = O.layernorm_forward(x, g, b, eps)
    assert np.abs(xhat.sum(axis=1)).max() < 1e-13
    var = x.var(axis=1)
    assert np.allclose((xhat ** 2).mean(axis=1), var / (var + eps), rtol=1e-13)
    yc, xc, _ = O.layernorm_forward(np.full((2, 10), 2.5), g, b, eps)
    assert np.all(xc == 0) and np.array_equal(yc, np.tile(b, (2, 1)))
    dy = rng.standard_normal((6, 10))
    dx, dg, db = O.layernorm_backward(dy, xhat, rstd, g)
    assert np.abs(dx.sum(axis=1)).max() < 1e-12
    # dx is orthogonal to xhat up to the eps term: sum_j dx*xhat = h * m2 * eps * rstd^3
    m2 = (dy * g * xhat).mean(axis=1)
    assert np.allclose((dx * xhat).sum(axis=1), 10 * m2 * eps * rstd[:, 0] ** 3, rtol=1e-9, atol=1e-15)
    assert np.allclose(db, dy.sum(axis=0)) and np.allclose(dg, (dy * xhat).sum(axis=0))
    want = F.layer_norm(torch.tensor(x), (10,), torch.tensor(g), torch.tensor(b), eps).numpy()
    assert np.allclose(y, want, atol=1e-13)


# --------------------------------------------------------------------- GEMM
def test_linear_pieces_brute_force():
    rng = np.random.default_rng(15)
    x = rng.standard_normal((3, 4))
    w = rng.standard_normal((5, 4))
    b = rng.standard_normal(5)
    dy = rng.standard_normal((3, 5))
    y = O.linear_forward(x, w, b)
    dx, dw, db = O.linear_backward(dy, x, w)
    for t in range(3):
        for o in range(5):
            assert abs(y[t, o] - (sum(x[t, i] * w[o, i] for i in range(4)) + b[o])) < 1e-14
    for t in range(3):
        for i in range(4):
            assert abs(dx[t, i] - sum(dy[t, o] * w[o, i] for o in range(5))) < 1e-14
    for o in range(5):
        assert abs(db[o] - sum(dy[t, o] for t in range(3))) < 1e-14
        for i in range(4):
            assert abs(dw[o, i] - sum(dy[t, o] * x[t, i] for t in range(3))) < 1e-14


# --------------------------------------------------------------------- GeLU
def test_gelu_values():
    from scipy.special import erf
    assert O.gelu_tanh(np.array([0.0]))[0] == 0.0
    assert O.gelu_tanh_grad(np.array([0.0]))[0] == 0.5
    assert abs(O.gelu_tanh(np.array([12.0]))[0] - 12.0) < 1e-12
    assert abs(O.gelu_tanh(np.array([-12.0]))[0]) < 1e-12
    u = np.linspace(-6, 6, 2001)
    exact = 0.5 * u * (1 + erf(u / math.sqrt(2)))
    assert np.abs(O.gelu_tanh(u) - exact).max() < 1e-3
    want = F.gelu(torch.tensor(u), approximate="tanh").numpy()
    assert np.abs(O.gelu_tanh(u) - want).max() < 1e-14
    hstep = 1e-6
    num = (O.gelu_tanh(u + hstep) - O.gelu_tanh(u - hstep)) / (2 * hstep)
    assert np.abs(num - O.gelu_tanh_grad(u)).max() < 1e-8


# -------------------------------------------------------------- accumulation
def test_accumulation_is_plain_sum():
    rng = np.random.default_rng(16)
    sh = tiny_shape(True, L=1)
    ps = rand_params(sh, rng)
    x = rng.standard_normal((sh.tokens, sh.hidden))
    dy = rng.standard_normal((sh.tokens, sh.hidden))
    x2 = rng.standard_normal((sh.tokens, sh.hidden))
    dy2 = rng.standard_normal((sh.tokens, sh.hidden))
    _, _, one = O.stage_step([x], [dy], ps, sh)
    _, _, three = O.stage_step([x] * 3, [dy] * 3, ps, sh)
    _, _, ab = O.stage_step([x, x2], [dy, dy2], ps, sh)
    _, _, ba = O.stage_step([x2, x], [dy2, dy], ps, sh)
    for k in O.PARAM_NAMES:
        assert np.allclose(three[0][k], 3 * one[0][k], rtol=1e-13, atol=1e-13)
        assert np.allclose(ab[0][k], ba[0][k], rtol=1e-13, atol=1e-13)


def test_recompute_equals_stored():
    """Re-deriving the intermediates from the stored boundary activation gives
    bit-identical values to the ones a storing forward kept."""
    rng = np.random.default_rng(17)
    sh = tiny_shape(True)
    ps = rand_params(sh, rng)
    x = rng.standard_normal((sh.tokens, sh.hidden))
    y, stored = O.stage_forward(x, ps, sh)
    y2, again = O.stage_recompute(x, ps, sh)
    assert np.array_equal(y, y2)
    for c0, c1 in zip(stored, again):
        for k in c0:
            if k == "probs":
                for key in c0[k]:
                    assert np.array_equal(c0[k][key], c1[k][key])
            else:
                assert np.array_equal(c0[k], c1[k]), k


def test_rel_l2_metric():
    assert O.rel_l2([3.0, 4.0], [3.0, 4.0]) == 0.0
    assert abs(O.rel_l2([3.0, 4.0 + 5e-3], [3.0, 4.0]) - 1e-3) < 1e-15
    assert O.rel_l2([0.0], [0.0]) == 0.0
