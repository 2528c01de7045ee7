"""Pins for oracle/tail_oracle.py (CPU): closed forms and torch's library optimizers."""
import numpy as np
import torch

from oracle import tail_oracle as T


def test_grad_stats_closed_forms_and_nonfinite_count():
    a = np.arange(1, 11, dtype=np.float64)           # 1^2+...+10^2 = 385
    b = np.array([3.0, -4.0])                        # 25
    s, bad = T.grad_stats([a, b.reshape(2, 1)])
    assert s == 410.0 and bad == 0
    c = np.array([1.0, np.inf, -np.inf, np.nan, 2.0])
    s, bad = T.grad_stats([c])
    assert s == 5.0 and bad == 3
    assert T.grad_stats([]) == (0.0, 0)


def test_first_step_is_lr_times_sign_of_gradient():
    """With m = v = 0 the bias-corrected first step is g/(|g| + eps): lr * sign(g) for |g| >> eps."""
    g = np.array([0.5, -2.0, 1e-3, -7.0])
    w0 = np.array([1.0, 1.0, 1.0, 1.0])
    w, m, v = T.adam_step(w0, np.zeros(4), np.zeros(4), g, step=1, lr=0.01, eps=1e-12)
    np.testing.assert_allclose(w, w0 - 0.01 * g / (np.abs(g) + 1e-12), rtol=0, atol=1e-15)
    np.testing.assert_allclose(w, w0 - 0.01 * np.sign(g), rtol=0, atol=1e-10)
    np.testing.assert_allclose(m, 0.1 * g, rtol=1e-15)
    np.testing.assert_allclose(v, 0.001 * g * g, rtol=1e-12)


def test_constant_gradient_keeps_unit_steps_and_zero_gradient_only_decays():
    """A constant gradient gives mhat = g and vhat = g^2 at every step (geometric sums cancel
    the bias corrections), so every step moves by lr * sign(g); g = 0 leaves w to the decay."""
    g = np.array([0.3, -0.3])
    w, m, v = np.zeros(2), np.zeros(2), np.zeros(2)
    for t in range(1, 6):
        w, m, v = T.adam_step(w, m, v, g, step=t, lr=0.1, eps=0.0)
        np.testing.assert_allclose(w, -0.1 * t * np.sign(g), rtol=1e-12)
    w, m, v = T.adam_step(np.array([2.0]), np.zeros(1), np.zeros(1), np.zeros(1), step=1, lr=0.1,
                          eps=1e-8, weight_decay=0.5)
    np.testing.assert_allclose(w, [2.0 * (1 - 0.1 * 0.5)], rtol=1e-15)
    assert m[0] == 0.0 and v[0] == 0.0


def test_grad_scale_is_applied_before_the_moments():
    g = np.array([4.0, -8.0])
    a = T.adam_step(np.ones(2), np.zeros(2), np.zeros(2), g, 1, 0.01, grad_scale=0.25)
    b = T.adam_step(np.ones(2), np.zeros(2), np.zeros(2), 0.25 * g, 1, 0.01)
    for x, y in zip(a, b):
        np.testing.assert_allclose(x, y, rtol=1e-15)


def _torch_run(opt_cls, w0, grads, **kw):
    p = torch.nn.Parameter(torch.tensor(w0, dtype=torch.float64))
    opt = opt_cls([p], **kw)
    for g in grads:
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
    return p.detach().numpy()


def test_matches_torch_adam_and_adamw_over_several_steps():
    rng = np.random.default_rng(5)
    w0 = rng.standard_normal(64)
    grads = [rng.standard_normal(64) * (0.1 + i) for i in range(6)]
    # plain Adam (no decay)
    w, m, v = w0.copy(), np.zeros(64), np.zeros(64)
    for t, g in enumerate(grads, 1):
        w, m, v = T.adam_step(w, m, v, g, t, lr=3e-3, beta1=0.8, beta2=0.95, eps=1e-6)
    ref = _torch_run(torch.optim.Adam, w0, grads, lr=3e-3, betas=(0.8, 0.95), eps=1e-6)
    np.testing.assert_allclose(w, ref, rtol=1e-10, atol=1e-12)
    # decoupled weight decay == torch's AdamW
    w, m, v = w0.copy(), np.zeros(64), np.zeros(64)
    for t, g in enumerate(grads, 1):
        w, m, v = T.adam_step(w, m, v, g, t, lr=3e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.1)
    ref = _torch_run(torch.optim.AdamW, w0, grads, lr=3e-3, betas=(0.9, 0.999), eps=1e-8, weight_decay=0.1)
    np.testing.assert_allclose(w, ref, rtol=1e-10, atol=1e-12)
