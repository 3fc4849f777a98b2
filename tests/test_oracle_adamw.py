"""Pins of the AdamW oracle (Experiments: the optimiser named there; algorithm of the work it cites)."""
import numpy as np

from oracle.adamw_oracle import adamw_step


def test_first_step_closed_form():
    # from a zero state mhat = g and vhat = g^2 exactly, so the step is lr * g / (|g| + eps)
    rng = np.random.default_rng(1)
    th = rng.normal(size=1000)
    g = rng.normal(size=1000) * 10.0 ** rng.integers(-6, 3, size=1000)
    lr, eps = 3e-4, 1e-8
    th1, m1, v1 = adamw_step(th, g, np.zeros_like(th), np.zeros_like(th), 1, lr, 0.9, 0.999, eps, 0.0)
    assert np.allclose(th1, th - lr * g / (np.abs(g) + eps), rtol=1e-12, atol=0)
    assert np.allclose(m1, 0.1 * g, rtol=1e-12) and np.allclose(v1, 0.001 * g * g, rtol=1e-12)


def test_constant_gradient_closed_form():
    # with the same gradient at every step the corrected moments stay g and g^2: t equal steps
    rng = np.random.default_rng(2)
    th0 = rng.normal(size=64)
    g = rng.normal(size=64)
    lr, eps, T = 1e-3, 1e-8, 25
    th, m, v = th0, np.zeros(64), np.zeros(64)
    for t in range(1, T + 1):
        th, m, v = adamw_step(th, g, m, v, t, lr, 0.9, 0.999, eps, 0.0)
    assert np.allclose(th, th0 - T * lr * g / (np.abs(g) + eps), rtol=1e-10)


def test_zero_gradient_is_geometric_decay():
    th0 = np.linspace(-2.0, 2.0, 33)
    lr, wd, T = 1e-2, 0.1, 40
    th, m, v = th0, np.zeros(33), np.zeros(33)
    for t in range(1, T + 1):
        th, m, v = adamw_step(th, np.zeros(33), m, v, t, lr, 0.9, 0.999, 1e-8, wd)
    assert np.allclose(th, th0 * (1.0 - lr * wd) ** T, rtol=1e-12)
    assert not m.any() and not v.any()


def test_decay_is_decoupled_from_the_moments():
    # the decay term never enters m or v (the difference to Adam with an L2 penalty)
    rng = np.random.default_rng(3)
    th, g = rng.normal(size=50), rng.normal(size=50)
    _, m_a, v_a = adamw_step(th, g, np.zeros(50), np.zeros(50), 1, 1e-3, weight_decay=0.0)
    _, m_b, v_b = adamw_step(th, g, np.zeros(50), np.zeros(50), 1, 1e-3, weight_decay=0.5)
    assert np.array_equal(m_a, m_b) and np.array_equal(v_a, v_b)


def test_against_library_optimiser():
    import torch
    rng = np.random.default_rng(4)
    n, T = 513, 7
    th0 = rng.normal(size=n)
    gs = rng.normal(size=(T, n)) * 10.0 ** rng.integers(-4, 2, size=(T, n))
    lr, b1, b2, eps, wd = 5e-5 * 40, 0.9, 0.999, 1e-8, 0.01
    p = torch.nn.Parameter(torch.tensor(th0, dtype=torch.float64))
    opt = torch.optim.AdamW([p], lr=lr, betas=(b1, b2), eps=eps, weight_decay=wd)
    th, m, v = th0, np.zeros(n), np.zeros(n)
    for t in range(1, T + 1):
        p.grad = torch.tensor(gs[t - 1], dtype=torch.float64)
        opt.step()
        th, m, v = adamw_step(th, gs[t - 1], m, v, t, lr, b1, b2, eps, wd)
        assert np.allclose(th, p.detach().numpy(), rtol=1e-9, atol=1e-13), t
