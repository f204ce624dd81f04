"""Pins of the AdamW oracle against things other than itself (no GPU)."""
import numpy as np
import pytest

from oracle.optim import adamw_step


def _rand(n, seed):
    rng = np.random.default_rng(seed)
    return rng.standard_normal(n), rng.standard_normal(n) * 0.1


def test_matches_the_library_optimizer_over_several_steps():
    torch = pytest.importorskip("torch")
    n = 257
    w0, _ = _rand(n, 0)
    p = torch.tensor(w0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.AdamW([p], lr=3e-3, betas=(0.8, 0.95), eps=1e-7, weight_decay=0.05)
    w, m, v = w0.copy(), np.zeros(n), np.zeros(n)
    for t in range(1, 8):
        g = np.random.default_rng(100 + t).standard_normal(n) * (0.5 ** t)
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        w, m, v = adamw_step(w, g, m, v, t, lr=3e-3, beta1=0.8, beta2=0.95, eps=1e-7, weight_decay=0.05)
        assert np.allclose(w, p.detach().numpy(), rtol=1e-12, atol=1e-14), t


def test_first_step_from_zero_moments_has_a_closed_form():
    # mhat = g and vhat = g^2 at t = 1, whatever the betas
    w0, g = _rand(64, 1)
    lr, eps, wd = 1e-3, 1e-8, 0.01
    w1, m1, v1 = adamw_step(w0, g, np.zeros(64), np.zeros(64), 1, lr=lr, beta1=0.7, beta2=0.9, eps=eps, weight_decay=wd)
    assert np.allclose(w1, w0 - lr * (g / (np.abs(g) + eps) + wd * w0), rtol=1e-13, atol=0)
    assert np.allclose(m1, 0.3 * g) and np.allclose(v1, 0.1 * g * g)
    # without decay the first step moves every weight by lr against the sign of its gradient
    w1, _, _ = adamw_step(w0, g, np.zeros(64), np.zeros(64), 1, lr=lr, eps=0.0, weight_decay=0.0)
    assert np.allclose(w1 - w0, -lr * np.sign(g), rtol=1e-12)


def test_zero_gradients_leave_pure_decay():
    w0, _ = _rand(32, 2)
    w, m, v = w0.copy(), np.zeros(32), np.zeros(32)
    for t in range(1, 6):
        w, m, v = adamw_step(w, np.zeros(32), m, v, t, lr=1e-2, weight_decay=0.1)
    assert np.allclose(w, w0 * (1 - 1e-2 * 0.1) ** 5, rtol=1e-13)
    assert not m.any() and not v.any()


def test_update_does_not_depend_on_the_gradient_scale():
    # Adam normalises by the second moment: scaling every gradient by c changes the step only through eps
    w0, _ = _rand(48, 3)
    outs = []
    for c in (1.0, 1e3):
        w, m, v = w0.copy(), np.zeros(48), np.zeros(48)
        for t in range(1, 5):
            g = np.random.default_rng(7 + t).standard_normal(48) + 0.5
            w, m, v = adamw_step(w, c * g, m, v, t, eps=0.0, weight_decay=0.0)
        outs.append(w)
    assert np.allclose(outs[0], outs[1], rtol=1e-10)


def test_moments_are_exponential_averages_of_what_they_should_be():
    # constant gradient: the bias-corrected moments equal g and g^2 at every step, so every step is the first step
    g = np.array([0.3, -2.0, 1e-3])
    w, m, v = np.zeros(3), np.zeros(3), np.zeros(3)
    for t in range(1, 10):
        w_prev = w
        w, m, v = adamw_step(w, g, m, v, t, lr=1e-3, eps=0.0, weight_decay=0.0)
        assert np.allclose(m / (1 - 0.9 ** t), g) and np.allclose(v / (1 - 0.999 ** t), g * g)
        assert np.allclose(w - w_prev, -1e-3 * np.sign(g), rtol=1e-10)
