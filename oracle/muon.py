"""fp64 oracle of the Muon inner step (test infrastructure only).

Follows the paper's Sec. 2 "Muon" paragraph (momentum accumulator, five Newton-Schulz
iterations with the tuned coefficients, decoupled weight decay) and Sec. 5 "MuLoCo"
(learning-rate rescale by sqrt(n/m) for an m x n matrix).  Readings where the paper is
silent or garbled:

* The printed iteration applies p to X X^T; taken literally that is not the quintic the
  text names.  The quintic reading is used: p acts on singular values,
  X <- a X + b (X X^T) X + c (X X^T)^2 X.
* Nesterov look-ahead is not in the paper's Muon equations; the workload descriptions
  ask for it.  U = g + beta * m_t with the updated accumulator; nesterov=False gives
  the paper's literal U = m_t.
* The iteration needs sigma_max <= 1.26 to stay bounded, so the input is divided by
  (||U||_F + eps) first; eps is added to the norm, not under the root.
* Only the orthogonalised term is multiplied by the per-shape rescale; the decay term
  uses eta * lambda as in the printed update rule.
"""
import numpy as np

NS_COEFFS = (3.4445, -4.7750, 2.0315)   # Sec. 2 "Muon": (a, b, c)


def momentum_update(m_prev, g, beta):
    """m_t = beta * m_{t-1} + g_t  (no (1 - beta) damping)."""
    return beta * np.asarray(m_prev, np.float64) + np.asarray(g, np.float64)


def update_direction(m_t, g, beta, nesterov):
    """Matrix handed to Newton-Schulz: m_t, or the look-ahead g + beta * m_t."""
    m_t = np.asarray(m_t, np.float64)
    if nesterov:
        return np.asarray(g, np.float64) + beta * m_t
    return m_t


def frobenius_normalise(U, eps=1e-7):
    U = np.asarray(U, np.float64)
    return U / (np.sqrt(np.sum(U * U)) + eps)


def newton_schulz(U, iters=5, coeffs=NS_COEFFS, eps=1e-7):
    """`iters` quintic Newton-Schulz iterations on U / (||U||_F + eps).

    Always the left (m x m Gram) form, for tall and wide matrices alike."""
    a, b, c = coeffs
    X = frobenius_normalise(U, eps)
    for _ in range(int(iters)):
        A = X @ X.T
        B = b * A + c * (A @ A)
        X = a * X + B @ X
    return X


def newton_schulz_right(U, iters=5, coeffs=NS_COEFFS, eps=1e-7):
    """Same iteration written with the n x n Gram matrix X^T X (algebraically equal)."""
    a, b, c = coeffs
    X = frobenius_normalise(U, eps)
    for _ in range(int(iters)):
        A = X.T @ X
        B = b * A + c * (A @ A)
        X = a * X + X @ B
    return X


def parameter_update(W, O, eta, weight_decay, lr_scale):
    """W_t = W_{t-1} - eta * lr_scale * O_t - eta * lambda * W_{t-1}."""
    W = np.asarray(W, np.float64)
    return W - eta * lr_scale * np.asarray(O, np.float64) - eta * weight_decay * W


def inner_step(W, m_prev, g, *, eta, weight_decay, beta, nesterov=True, ns_iters=5,
               coeffs=NS_COEFFS, eps=1e-7, lr_scale=1.0):
    """One Muon step on one matrix.  Returns (W_t, m_t, O_t), all float64."""
    m_t = momentum_update(m_prev, g, beta)
    U = update_direction(m_t, g, beta, nesterov)
    O = newton_schulz(U, ns_iters, coeffs, eps)
    return parameter_update(W, O, eta, weight_decay, lr_scale), m_t, O
