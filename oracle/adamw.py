"""fp64 oracle of the AdamW step used for the parameters that Muon does not cover
(embeddings, norms, biases) (test infrastructure only).

Follows Sec. 4 "AdamW inner updates and induced pseudogradient": exponential moving averages
of the gradient and of its square, the step alpha * m / (sqrt(v) + eps), and decoupled
weight decay lambda * alpha * theta.  Reading: the printed equations carry no bias
correction; it is an option here (bias_correction=True divides m by 1 - beta1^t and v by
1 - beta2^t, t counted from 1, which is the usual form of the optimizer).
"""
import numpy as np


def adamw_step(theta, m_prev, v_prev, g, *, lr, beta1, beta2, eps, weight_decay, step,
               bias_correction=False):
    """One step.  Returns (theta, m, v)."""
    theta = np.asarray(theta, np.float64)
    g = np.asarray(g, np.float64)
    m = beta1 * np.asarray(m_prev, np.float64) + (1.0 - beta1) * g
    v = beta2 * np.asarray(v_prev, np.float64) + (1.0 - beta2) * g * g
    m_hat, v_hat = m, v
    if bias_correction:
        assert step >= 1
        m_hat = m / (1.0 - beta1 ** step)
        v_hat = v / (1.0 - beta2 ** step)
    new = theta - lr * (m_hat / (np.sqrt(v_hat) + eps)) - weight_decay * lr * theta
    return new, m, v
