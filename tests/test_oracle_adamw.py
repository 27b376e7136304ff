"""Pins for oracle/adamw.py: the library optimizer as the textbook form (with bias
correction), closed forms for a constant gradient, and sign / scale special cases."""
import numpy as np
import torch

from oracle import adamw


def test_matches_library_adamw_over_several_steps():
    r = np.random.default_rng(1)
    theta0 = r.standard_normal((7, 5))
    p = torch.nn.Parameter(torch.tensor(theta0, dtype=torch.float64))
    opt = torch.optim.AdamW([p], lr=3e-3, betas=(0.9, 0.95), eps=1e-8, weight_decay=0.1)
    th, m, v = theta0.copy(), np.zeros_like(theta0), np.zeros_like(theta0)
    for t in range(1, 9):
        g = r.standard_normal((7, 5)) * 0.1
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        th, m, v = adamw.adamw_step(th, m, v, g, lr=3e-3, beta1=0.9, beta2=0.95, eps=1e-8,
                                    weight_decay=0.1, step=t, bias_correction=True)
        assert np.max(np.abs(p.detach().numpy() - th)) < 1e-14
    st = opt.state[p]
    assert np.max(np.abs(st["exp_avg"].numpy() - m)) < 1e-16
    assert np.max(np.abs(st["exp_avg_sq"].numpy() - v)) < 1e-16


def test_constant_gradient_closed_form_without_bias_correction():
    # m_t = (1 - b1^t) g, v_t = (1 - b2^t) g^2: the step is lr * (1-b1^t) g / (sqrt(1-b2^t)|g| + eps)
    g = np.array([[0.5, -2.0, 1e-3]])
    th, m, v = np.zeros((1, 3)), np.zeros((1, 3)), np.zeros((1, 3))
    b1, b2, lr, eps = 0.9, 0.99, 0.01, 1e-8
    total = np.zeros((1, 3))
    for t in range(1, 6):
        th, m, v = adamw.adamw_step(th, m, v, g, lr=lr, beta1=b1, beta2=b2, eps=eps, weight_decay=0.0, step=t)
        assert np.allclose(m, (1 - b1 ** t) * g, rtol=1e-14) and np.allclose(v, (1 - b2 ** t) * g * g, rtol=1e-14)
        total -= lr * (1 - b1 ** t) * g / (np.sqrt(1 - b2 ** t) * np.abs(g) + eps)
        assert np.allclose(th, total, rtol=1e-13)
    # with bias correction every step is lr * sign(g) (up to eps)
    th, m, v = np.zeros((1, 3)), np.zeros((1, 3)), np.zeros((1, 3))
    for t in range(1, 4):
        prev = th
        th, m, v = adamw.adamw_step(th, m, v, g, lr=lr, beta1=b1, beta2=b2, eps=eps, weight_decay=0.0,
                                    step=t, bias_correction=True)
        assert np.allclose(th - prev, -lr * np.sign(g), rtol=1e-4)


def test_zero_gradient_is_pure_decoupled_decay():
    th0 = np.array([[1.0, -3.0]])
    th, m, v = adamw.adamw_step(th0, np.zeros((1, 2)), np.zeros((1, 2)), np.zeros((1, 2)), lr=0.1, beta1=0.9,
                                beta2=0.99, eps=1e-8, weight_decay=0.5, step=1)
    assert np.allclose(th, th0 * (1 - 0.1 * 0.5)) and not m.any() and not v.any()
