"""Pins for the dropout part of the oracle (CPU): the generator against its published
known-answer vectors, the mask statistics, finite differences and torch autograd with the
same masks, and the recompute property."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import dropout_oracle as D
from oracle import stage_oracle as O
from tests.test_oracle_pins import rand_params, tiny_shape


def test_philox4x32_10_known_answers():
    """Known-answer vectors distributed with the generator's reference implementation
    (Random123, kat_vectors: philox4x32 with 10 rounds)."""
    kat = [
        ((0, 0, 0, 0), (0, 0), (0x6627e8d5, 0xe169c58d, 0xbc57ac4c, 0x9b00dbd8)),
        ((0xffffffff,) * 4, (0xffffffff,) * 2, (0x408f276d, 0x41c83b0e, 0xa20bc7c6, 0x6d5451fd)),
        ((0x243f6a88, 0x85a308d3, 0x13198a2e, 0x03707344), (0xa4093822, 0x299f31d0),
         (0xd16cfe09, 0x94fdcceb, 0x5001e420, 0x24126ea1)),
    ]
    for ctr, key, want in kat:
        got = tuple(int(w) for w in D.philox4x32_10(ctr, key))
        assert got == want
    # vectorised call == element-wise calls
    c0 = np.arange(5, dtype=np.uint64)
    vec = D.philox4x32_10((c0, 7, 9, 11), (3, 4))
    for i in range(5):
        one = D.philox4x32_10((i, 7, 9, 11), (3, 4))
        assert [int(w[i]) for w in vec] == [int(w) for w in one]


def test_byte_layout_one_call_per_4x4_patch():
    d = D.Dropout(0.1, seed=(5 << 32) | 77)
    b = d.bytes(D.SITE_PROJ, 3, 2, row0=0, n_rows=8, n_cols=12)
    words = D.philox4x32_10((1, 2, D.SITE_PROJ + 256 * 3, 2), (77, 5))      # patch rows 4..7, cols 8..11
    for r in range(4):
        for c in range(4):
            assert b[4 + r, 8 + c] == (int(words[r]) >> (8 * c)) & 0xFF
    # a row offset only shifts the rows
    assert np.array_equal(d.bytes(D.SITE_PROJ, 3, 2, row0=5, n_rows=3, n_cols=12), b[5:8])
    # every coordinate of the counter and the seed matter
    base = d.bytes(0, 0, 0, 0, 64, 64)
    for other in (d.bytes(1, 0, 0, 0, 64, 64), d.bytes(0, 1, 0, 0, 64, 64), d.bytes(0, 0, 1, 0, 64, 64),
                  D.Dropout(0.1, seed=78).bytes(0, 0, 0, 0, 64, 64), d.bytes(0, 0, 0, 64, 64, 64)):
        assert np.mean(other == base) < 0.02


@pytest.mark.parametrize("p", [0.1, 0.25, 0.5])
def test_mask_statistics(p):
    d = D.Dropout(p, seed=1234567891011)
    ks = d.keep_scale(D.SITE_ATTN, 1, 3, 0, 1024, 1024)
    n = ks.size
    drop_rate = np.mean(ks == 0.0)
    q = d.thr / 256.0
    assert abs(q - p) <= 1.0 / 512
    assert abs(drop_rate - q) < 5.0 * np.sqrt(q * (1 - q) / n)
    assert set(np.unique(ks)) == {0.0, d.scale}
    assert abs(ks.mean() - 1.0) < 5.0 * d.scale * np.sqrt(q * (1 - q) / n)     # unbiased
    # bytes are uniform: chi-square over 256 bins
    b = d.bytes(D.SITE_ATTN, 1, 3, 0, 1024, 1024).ravel()
    cnt = np.bincount(b, minlength=256)
    chi2 = ((cnt - n / 256.0) ** 2 / (n / 256.0)).sum()
    assert chi2 < 255 + 6 * np.sqrt(2 * 255)
    # neighbouring rows / columns are uncorrelated
    x = (ks != 0).astype(np.float64) - (1 - q)
    assert abs((x[:, 1:] * x[:, :-1]).mean()) < 5 * q * (1 - q) / np.sqrt(n)
    assert abs((x[1:] * x[:-1]).mean()) < 5 * q * (1 - q) / np.sqrt(n)


def test_zero_probability_is_the_plain_stage():
    rng = np.random.default_rng(3)
    sh = tiny_shape()
    ps = rand_params(sh, rng)
    x = rng.standard_normal((sh.tokens, sh.hidden))
    dy = rng.standard_normal((sh.tokens, sh.hidden))
    y0, c0 = O.stage_forward(x, ps, sh)
    y1, c1 = O.stage_forward(x, ps, sh, D.Dropout(0.0, 5), mb=2)
    assert np.array_equal(y0, y1)
    dx0, g0 = O.stage_backward(dy, ps, c0, sh)
    dx1, g1 = O.stage_backward(dy, ps, c1, sh)
    assert np.array_equal(dx0, dx1)
    assert all(np.array_equal(g0[l][k], g1[l][k]) for l in range(sh.n_layers) for k in O.PARAM_NAMES)


@pytest.mark.parametrize("causal", [True, False])
def test_finite_difference_with_dropout(causal):
    """The masks are constants of the function, so central differences apply unchanged."""
    rng = np.random.default_rng(11)
    sh = tiny_shape(causal, s=6)
    ps = rand_params(sh, rng)
    x = rng.standard_normal((sh.tokens, sh.hidden))
    R = rng.standard_normal((sh.tokens, sh.hidden))
    drop = D.Dropout(0.3, seed=99)
    y, caches = O.stage_forward(x, ps, sh, drop, mb=1)
    dx, grads = O.stage_backward(R, ps, caches, sh)
    assert np.linalg.norm(y - O.stage_forward(x, ps, sh)[0]) > 1e-3      # dropout did change the output

    def loss():
        return float((O.stage_forward(x, ps, sh, drop, mb=1)[0] * R).sum())

    def fd(arr, idx):
        old = arr[idx]
        step = 1e-6 * max(1.0, abs(old))
        arr[idx] = old + step
        lp = loss()
        arr[idx] = old - step
        lm = loss()
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


def test_against_torch_autograd_with_the_same_masks():
    """One layer composed from torch library ops, the oracle's masks multiplied in at the three sites."""
    rng = np.random.default_rng(13)
    sh = tiny_shape(True, L=1, s=7)
    ps = rand_params(sh, rng)
    x = rng.standard_normal((sh.tokens, sh.hidden))
    R = rng.standard_normal((sh.tokens, sh.hidden))
    drop = D.Dropout(0.25, seed=4242)
    y, caches = O.stage_forward(x, ps, sh, drop, mb=3)
    dx, grads = O.stage_backward(R, ps, caches, sh)

    h, a, d, s, b = sh.hidden, sh.n_heads, sh.head_dim, sh.seq_len, sh.micro_batch
    tp = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in ps[0].items()}
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    k1 = torch.tensor(drop.keep_scale(D.SITE_PROJ, 0, 3, 0, sh.tokens, h))
    k2 = torch.tensor(drop.keep_scale(D.SITE_MLP, 0, 3, 0, sh.tokens, h))
    xn1 = F.layer_norm(tx, (h,), tp["ln1_g"], tp["ln1_b"], sh.ln_eps)
    qkv = F.linear(xn1, tp["wqkv"], tp["bqkv"])
    ctx = torch.zeros(sh.tokens, h, dtype=torch.float64)
    parts = []
    for bi in range(b):
        row = []
        for j in range(a):
            q = qkv[bi * s:(bi + 1) * s, j * d:(j + 1) * d]
            k = qkv[bi * s:(bi + 1) * s, h + j * d:h + (j + 1) * d]
            v = qkv[bi * s:(bi + 1) * s, 2 * h + j * d:2 * h + (j + 1) * d]
            sc = (q @ k.T) / d ** 0.5
            sc = sc.masked_fill(torch.triu(torch.ones(s, s, dtype=torch.bool), 1), float("-inf"))
            pm = F.softmax(sc, dim=1) * torch.tensor(drop.keep_scale(D.SITE_ATTN, 0, 3, (bi * a + j) * s, s, s))
            row.append(pm @ v)
        parts.append(torch.cat(row, dim=1))
    ctx = torch.cat(parts, dim=0)
    x1 = tx + k1 * F.linear(ctx, tp["wo"], tp["bo"])
    xn2 = F.layer_norm(x1, (h,), tp["ln2_g"], tp["ln2_b"], sh.ln_eps)
    g = F.gelu(F.linear(xn2, tp["w1"], tp["b1"]), approximate="tanh")
    ty = x1 + k2 * F.linear(g, tp["w2"], tp["b2"])
    (ty * torch.tensor(R)).sum().backward()
    np.testing.assert_allclose(y, ty.detach().numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dx, tx.grad.numpy(), rtol=1e-9, atol=1e-11)
    for k in O.PARAM_NAMES:
        np.testing.assert_allclose(grads[0][k], tp[k].grad.numpy(), rtol=1e-9, atol=1e-11)


def test_recompute_regenerates_the_masks_and_micro_batches_differ():
    rng = np.random.default_rng(17)
    sh = tiny_shape()
    ps = rand_params(sh, rng)
    x = rng.standard_normal((sh.tokens, sh.hidden))
    drop = D.Dropout(0.2, seed=31337)
    y_a, c_a = O.stage_forward(x, ps, sh, drop, mb=2)
    y_b, c_b = O.stage_recompute(x, ps, sh, drop, mb=2)
    assert np.array_equal(y_a, y_b)
    for ca, cb in zip(c_a, c_b):
        for k in ("xn1", "qkv", "ctx", "x1", "xn2", "u", "g"):
            assert np.array_equal(ca[k], cb[k])
    y_c, _ = O.stage_forward(x, ps, sh, drop, mb=3)
    assert not np.array_equal(y_a, y_c)
