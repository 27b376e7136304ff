"""Pins for oracle/muon.py (CPU only).

The paper prints no worked example, so the oracle is pinned by what the mathematics
fixes: the iteration acts on singular values only (closed form on constructed spectra),
the textbook cubic Newton-Schulz coefficients converge to the SVD polar factor, the
tuned quintic lands every singular value in the band its critical points imply, the
left and right Gram forms agree, and the momentum/Nesterov rule equals the library's
SGD-with-Nesterov on a problem both can run.
"""
import os

import numpy as np
import pytest
import torch

from oracle import muon

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden_coeffs():
    vals = {}
    for line in open(os.path.join(GOLDEN, "ns_coefficients.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, v = line.split()
        vals[k] = float(v)
    return vals


def _haar(n, rng):
    q, r = np.linalg.qr(rng.standard_normal((n, n)))
    return q * np.sign(np.diag(r))


def _phi(sig, k, coeffs):
    a, b, c = coeffs
    sig = np.array(sig, dtype=np.float64)
    for _ in range(k):
        sig = a * sig + b * sig ** 3 + c * sig ** 5
    return sig


def test_coefficients_are_the_papers():
    g = _golden_coeffs()
    assert muon.NS_COEFFS == (g["a"], g["b"], g["c"])
    assert g["iterations"] == 5


@pytest.mark.parametrize("m,n", [(6, 6), (5, 11), (12, 4)])
@pytest.mark.parametrize("k", [0, 1, 2, 5, 8])
def test_closed_form_on_constructed_spectra(m, n, k):
    """X = P diag(s) Q^T  =>  NS_k(X) = P diag(phi^k(s / ||s||)) Q^T, wide and tall."""
    rng = np.random.default_rng(m * 100 + n)
    r = min(m, n)
    P, Q = _haar(m, rng), _haar(n, rng)
    sig = np.sort(rng.uniform(0.05, 1.0, r))[::-1]
    S = np.zeros((m, n))
    S[:r, :r] = np.diag(sig)
    X = 3.7 * (P @ S @ Q.T)                       # arbitrary positive scale
    out = muon.newton_schulz(X, iters=k, eps=0.0)
    want_sig = _phi(sig / np.linalg.norm(sig), k, muon.NS_COEFFS)
    Sw = np.zeros((m, n))
    Sw[:r, :r] = np.diag(want_sig)
    want = P @ Sw @ Q.T
    assert np.max(np.abs(out - want)) <= 1e-10 * max(1.0, np.max(np.abs(want)))


def test_cubic_newton_schulz_converges_to_svd_polar_factor():
    """(a,b,c) = (1.5,-0.5,0) is the classical iteration; its limit is U V^T."""
    rng = np.random.default_rng(1)
    for (m, n) in [(4, 4), (8, 16), (16, 8)]:
        X = rng.standard_normal((m, n))
        U, s, Vt = np.linalg.svd(X, full_matrices=False)
        polar = U @ Vt
        errs = [np.linalg.norm(muon.newton_schulz(X, k, (1.5, -0.5, 0.0)) - polar, 2)
                for k in (5, 20, 60)]
        assert errs[0] > errs[1] > errs[2] or errs[1] < 1e-12
        assert errs[2] < 1e-12


def test_quintic_band_and_distance_to_polar_factor():
    """With the tuned coefficients every singular value that starts in [2e-3, 1] ends in
    [phi(local min), phi(local max)] = [0.6818, 1.2024] after >= 5 iterations, so the
    output is within 0.3182 (spectral norm) of the polar factor but does not reach it."""
    a, b, c = muon.NS_COEFFS
    # critical points of phi from phi'(x) = a + 3b x^2 + 5c x^4 = 0 (quadratic in x^2)
    disc = np.sqrt(9 * b * b - 20 * a * c)
    x_lo, x_hi = np.sqrt((-3 * b - disc) / (10 * c)), np.sqrt((-3 * b + disc) / (10 * c))
    top = _phi([x_lo], 1, muon.NS_COEFFS)[0]
    bot = _phi([x_hi], 1, muon.NS_COEFFS)[0]
    assert abs(top - 1.202369) < 1e-5 and abs(bot - 0.681831) < 1e-5
    rng = np.random.default_rng(2)
    for (m, n) in [(4, 4), (8, 16), (24, 8)]:
        r = min(m, n)
        P, Q = _haar(m, rng), _haar(n, rng)
        sig = np.geomspace(1.0, 0.05, r)
        S = np.zeros((m, n)); S[:r, :r] = np.diag(sig)
        X = P @ S @ Q.T
        polar = P[:, :r] @ Q[:, :r].T
        for k in (5, 6, 9):
            O = muon.newton_schulz(X, k)
            sv = np.linalg.svd(O, compute_uv=False)
            assert sv.min() >= bot - 1e-9 and sv.max() <= top + 1e-9
            assert np.linalg.norm(O - polar, 2) <= max(1 - bot, top - 1) + 1e-9
            # orthonormal-step facts (paper Sec. 4.3): ||O||_F ~ sqrt(r), <X0,O> ~ ||X0||_*
            assert bot * np.sqrt(r) - 1e-9 <= np.linalg.norm(O) <= top * np.sqrt(r) + 1e-9
            X0 = muon.frobenius_normalise(X)
            nuc = np.linalg.svd(X0, compute_uv=False).sum()
            assert bot * nuc - 1e-9 <= np.sum(X0 * O) <= top * nuc + 1e-9


def test_left_and_right_forms_and_symmetries():
    rng = np.random.default_rng(3)
    for (m, n) in [(7, 7), (5, 13), (13, 5)]:
        X = rng.standard_normal((m, n)) * 1e-3
        L = muon.newton_schulz(X)
        R = muon.newton_schulz_right(X)
        assert np.max(np.abs(L - R)) < 1e-12
        assert np.max(np.abs(muon.newton_schulz(X.T).T - L)) < 1e-12
        Rm, Sn = _haar(m, rng), _haar(n, rng)
        assert np.max(np.abs(muon.newton_schulz(Rm @ X @ Sn) - Rm @ L @ Sn)) < 1e-11
        assert np.max(np.abs(muon.newton_schulz(1e4 * X, eps=0.0) - muon.newton_schulz(X, eps=0.0))) < 1e-11


def test_zero_matrix_and_zero_iterations():
    Z = np.zeros((4, 6))
    assert np.array_equal(muon.newton_schulz(Z), Z)
    X = np.arange(12, dtype=np.float64).reshape(3, 4)
    out = muon.newton_schulz(X, iters=0, eps=1e-7)
    assert np.allclose(out, X / (np.linalg.norm(X) + 1e-7), rtol=0, atol=1e-15)


def test_momentum_closed_form():
    rng = np.random.default_rng(4)
    gs = [rng.standard_normal((3, 5)) for _ in range(6)]
    beta = 0.95
    m = np.zeros((3, 5))
    for g in gs:
        m = muon.momentum_update(m, g, beta)
    want = sum(beta ** (len(gs) - 1 - i) * g for i, g in enumerate(gs))
    assert np.max(np.abs(m - want)) < 1e-14
    # constant gradient: geometric series, no (1 - beta) damping
    m = np.zeros(1)
    for _ in range(10):
        m = muon.momentum_update(m, np.ones(1), 0.9)
    assert abs(m[0] - (1 - 0.9 ** 10) / (1 - 0.9)) < 1e-13


def test_momentum_and_nesterov_match_library_sgd():
    """theta -= lr * U with the oracle's (m, U) must equal torch.optim.SGD with
    momentum, dampening 0, with and without nesterov, on a quadratic."""
    for nesterov in (True, False):
        torch.manual_seed(0)
        theta0 = torch.randn(4, 3, dtype=torch.float64)
        Hdiag = torch.rand(4, 3, dtype=torch.float64) + 0.5
        p = torch.nn.Parameter(theta0.clone())
        opt = torch.optim.SGD([p], lr=0.1, momentum=0.9, nesterov=nesterov)
        th = theta0.numpy().copy()
        m = np.zeros_like(th)
        for _ in range(7):
            opt.zero_grad()
            (0.5 * (Hdiag * p * p).sum()).backward()
            opt.step()
            g = Hdiag.numpy() * th
            m = muon.momentum_update(m, g, 0.9)
            th = th - 0.1 * muon.update_direction(m, g, 0.9, nesterov)
        assert np.max(np.abs(th - p.detach().numpy())) < 1e-14
    g = np.ones((2, 2))
    assert np.array_equal(muon.update_direction(muon.momentum_update(0 * g, g, 0.0), g, 0.0, True), g)


def test_parameter_update_and_step_norm():
    rng = np.random.default_rng(5)
    W = rng.standard_normal((6, 10)) * 0.02
    O = rng.standard_normal((6, 10))
    eta, lam, s = 0.05, 0.01, 2.0
    out = muon.parameter_update(W, O, eta, lam, s)
    # element-wise brute force of the printed rule
    for i in range(6):
        for j in range(10):
            assert abs(out[i, j] - (W[i, j] - eta * s * O[i, j] - eta * lam * W[i, j])) < 1e-16
    # lambda = 0: the step has norm eta * lr_scale * ||O||_F, inside the band times sqrt(r)
    g = rng.standard_normal((6, 10)) * 1e-3
    W1, m1, O1 = muon.inner_step(W, np.zeros_like(W), g, eta=eta, weight_decay=0.0, beta=0.95,
                                 lr_scale=s)
    step = np.linalg.norm(W1 - W)
    assert abs(step - eta * s * np.linalg.norm(O1)) < 1e-14
    assert 0.6818 * np.sqrt(6) * eta * s <= step <= 1.2024 * np.sqrt(6) * eta * s
    # decay aligned with the step direction enlarges it (the paper's remark on step norms)
    Wal = 0.02 * O1
    n0 = np.linalg.norm(muon.parameter_update(Wal, O1, eta, 0.0, s) - Wal)
    n1 = np.linalg.norm(muon.parameter_update(Wal, O1, eta, 0.1, s) - Wal)
    assert n1 > n0
    assert np.array_equal(m1, g)


def test_inner_step_composition_beta_zero():
    rng = np.random.default_rng(6)
    W = rng.standard_normal((5, 5)) * 0.02
    g = rng.standard_normal((5, 5)) * 1e-3
    for nesterov in (True, False):
        W1, m1, O1 = muon.inner_step(W, rng.standard_normal((5, 5)), g, eta=0.1, weight_decay=0.0,
                                     beta=0.0, nesterov=nesterov)
        assert np.max(np.abs(O1 - muon.newton_schulz(g))) < 1e-15
