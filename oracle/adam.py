"""fp64 oracle of the Adam update with loss-scale removal.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

The paper makes the optimizer part of the compiled training graph (Section 3,
graph-generation phase) and evaluates with Adam (Section 5.1); the rule is
Kingma & Ba's: bias-corrected first and second moments, epsilon added outside
the square root, optional L2 weight decay folded into the
gradient, step count t starting at 1.
"""
import numpy as np


def adam_step(w, g, m, v, t, lr, beta1, beta2, eps, weight_decay=0.0, inv_loss_scale=1.0):
    """Returns (w_new, m_new, v_new); all fp64, no in-place mutation."""
    w = np.asarray(w, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64) * inv_loss_scale
    m = np.asarray(m, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    if weight_decay != 0.0:
        g = g + weight_decay * w
    m_new = beta1 * m + (1.0 - beta1) * g
    v_new = beta2 * v + (1.0 - beta2) * g * g
    m_hat = m_new / (1.0 - beta1 ** t)
    v_hat = v_new / (1.0 - beta2 ** t)
    w_new = w - lr * m_hat / (np.sqrt(v_hat) + eps)
    return w_new, m_new, v_new
