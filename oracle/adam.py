"""Adam update, NumPy float64.

Test infrastructure (see the package docstring).  For the translation experiments (Section 4) the paper
adopts the training recipe of Ott et al., whose optimiser is Adam (Kingma & Ba, Algorithm 1 there) with
beta = (0.9, 0.98) and eps = 1e-8; the paper itself prints no update rule for it.  The reading taken is the
original algorithm with the same coupled L2 term as the momentum-SGD update:

    g <- g + weight_decay * w
    m <- beta1 * m + (1 - beta1) * g              (m, v start at 0; t counts updates from 1)
    v <- beta2 * v + (1 - beta2) * g * g
    w <- w - lr * (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps)
"""
import numpy as np


def adam_step(w, m, v, g, lr, t, beta1=0.9, beta2=0.98, eps=1e-8, weight_decay=0.0):
    """Return (w_new, m_new, v_new) after update number t >= 1; inputs are not modified."""
    w = np.asarray(w, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64) + weight_decay * w
    m_new = beta1 * np.asarray(m, dtype=np.float64) + (1.0 - beta1) * g
    v_new = beta2 * np.asarray(v, dtype=np.float64) + (1.0 - beta2) * g * g
    m_hat = m_new / (1.0 - beta1 ** t)
    v_hat = v_new / (1.0 - beta2 ** t)
    return w - lr * m_hat / (np.sqrt(v_hat) + eps), m_new, v_new
