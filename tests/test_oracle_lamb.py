"""Pins for the LAMB oracle (oracle/lamb.py).  CPU only.

Independent references: torch.optim.Adam (moments and bias-corrected direction: LAMB without weight decay is
Adam's step rescaled to length lr * ||w||) and closed forms.
"""
import numpy as np
import torch

from oracle.lamb import lamb_step


def _state(n=257, seed=0):
    rng = np.random.default_rng(seed)
    return rng.standard_normal(n) * 0.05, [rng.standard_normal(n) * 1e-3 for _ in range(4)]


def test_moments_and_direction_against_torch_adam():
    w0, grads = _state()
    lr, b1, b2, eps = 1e-3, 0.9, 0.95, 1e-6
    p = torch.nn.Parameter(torch.tensor(w0))
    opt = torch.optim.Adam([p], lr=lr, betas=(b1, b2), eps=eps)
    w, m, v = w0.copy(), np.zeros_like(w0), np.zeros_like(w0)
    for t, g in enumerate(grads, start=1):
        before = p.detach().numpy().copy()
        p.grad = torch.tensor(g)
        opt.step()
        adam_dw = p.detach().numpy() - before                 # = -lr * r with torch's own bias correction
        w_new, m, v, ratio = lamb_step(before, g, m, v, t, lr, b1, b2, eps, weight_decay=0.0)
        st = opt.state[p]
        assert np.allclose(m, st["exp_avg"].numpy(), rtol=1e-12, atol=0)
        assert np.allclose(v, st["exp_avg_sq"].numpy(), rtol=1e-12, atol=0)
        # same direction, length rescaled by ||w|| / ||r||
        r = -adam_dw / lr
        assert np.allclose(w_new - before, adam_dw * np.linalg.norm(before) / np.linalg.norm(r), rtol=1e-9, atol=1e-15)
        assert abs(ratio - np.linalg.norm(before) / np.linalg.norm(r)) < 1e-9 * ratio


def test_closed_forms():
    w0, grads = _state(seed=1)
    z = np.zeros_like(w0)
    # without weight decay the step has length lr * ||w|| whatever the gradient
    w1, _, _, _ = lamb_step(w0, grads[0], z, z, 1, lr=2e-3, weight_decay=0.0)
    assert abs(np.linalg.norm(w1 - w0) - 2e-3 * np.linalg.norm(w0)) < 1e-12
    # zero gradient: u = wd * w, ratio = 1 / wd, so w shrinks by exactly lr
    w1, m1, v1, ratio = lamb_step(w0, z, z, z, 1, lr=1e-3, weight_decay=0.01)
    assert np.allclose(w1, (1 - 1e-3) * w0, rtol=1e-13, atol=0) and abs(ratio - 100.0) < 1e-9
    assert not m1.any() and not v1.any()
    # zero weights: ratio 1, plain bias-corrected sign-like step r = g / (|g| + eps) on the first step
    g = grads[1]
    w1, _, _, ratio = lamb_step(z, g, z, z, 1, lr=1e-3, eps=1e-6, weight_decay=0.01)
    assert ratio == 1.0 and np.allclose(w1, -1e-3 * g / (np.abs(g) + 1e-6), rtol=1e-12, atol=0)
    # grad_scale trades against the gradient's own scale
    a = lamb_step(w0, grads[2] * 8.0, z, z, 3, grad_scale=0.125)
    b = lamb_step(w0, grads[2], z, z, 3, grad_scale=1.0)
    for x, y in zip(a[:3], b[:3]):
        assert np.allclose(x, y, rtol=1e-13, atol=0)
    # inputs are left alone
    keep = w0.copy()
    lamb_step(w0, grads[0], z, z, 1)
    assert np.array_equal(w0, keep)
