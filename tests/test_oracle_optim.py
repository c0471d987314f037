"""Pins for oracle/optim_oracle.py (AdamW step and learning-rate schedule, App. C)."""
import math

import numpy as np

from oracle import optim_oracle as OO


def test_first_step_closed_form():
    rng = np.random.default_rng(0)
    p, g = rng.standard_normal(50), rng.standard_normal(50)
    lr, wd, eps = 1e-3, 0.01, 1e-8
    q, m, v = OO.adamw_step(p, g, np.zeros(50), np.zeros(50), lr, 0.9, 0.999, eps, wd, 1)
    # with zero state the bias-corrected moments are g and g^2 exactly
    assert np.allclose(q, p - lr * wd * p - lr * g / (np.abs(g) + eps), rtol=1e-12, atol=1e-15)
    assert np.allclose(m, 0.1 * g) and np.allclose(v, 0.001 * g * g)


def test_constant_gradient_keeps_the_same_step():
    p = np.array([1.0, -2.0])
    g = np.array([0.3, -0.7])
    m = np.zeros(2)
    v = np.zeros(2)
    for t in range(1, 30):
        q, m, v = OO.adamw_step(p, g, m, v, 1e-2, 0.9, 0.999, 1e-8, 0.0, t)
        assert np.allclose(q - p, -1e-2 * np.sign(g), rtol=1e-6)   # mhat = g, sqrt(vhat) = |g| at every step
        p = q


def test_against_torch_adamw():
    import torch
    rng = np.random.default_rng(1)
    p0 = rng.standard_normal((7, 5))
    tp = torch.tensor(p0.copy(), dtype=torch.float64, requires_grad=True)
    opt = torch.optim.AdamW([tp], lr=3e-3, betas=(0.9, 0.999), eps=1e-8, weight_decay=0.01)
    p, m, v = p0.copy(), np.zeros_like(p0), np.zeros_like(p0)
    for t in range(1, 6):
        g = rng.standard_normal((7, 5))
        tp.grad = torch.tensor(g)
        opt.step()
        p, m, v = OO.adamw_step(p, g, m, v, 3e-3, 0.9, 0.999, 1e-8, 0.01, t)
        assert np.allclose(tp.detach().numpy(), p, rtol=1e-12, atol=1e-14)


def test_schedule_shape():
    N, lr = 1000, 5e-5
    w = 100
    assert math.isclose(OO.cosine_lr(0, N, lr), lr / w)
    assert math.isclose(OO.cosine_lr(w - 1, N, lr), lr)          # warm-up ends at the maximum
    assert math.isclose(OO.cosine_lr(w, N, lr), lr)              # cosine starts there
    assert math.isclose(OO.cosine_lr((N + w) // 2, N, lr), lr / 2, rel_tol=1e-9)
    assert OO.cosine_lr(N, N, lr) == 0.0 and OO.cosine_lr(N - 1, N, lr) < 1e-3 * lr
    vals = [OO.cosine_lr(t, N, lr) for t in range(N)]
    assert all(a <= b for a, b in zip(vals[:w - 1], vals[1:w])) and all(a >= b for a, b in zip(vals[w:-1], vals[w + 1:]))
