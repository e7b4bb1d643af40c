"""Momentum-SGD update, NumPy float64.

Test infrastructure (see the package docstring).  The paper's Algorithm 1 writes
the update as theta <- theta - eta * gradient and defers the optimiser details
to the large-minibatch ImageNet recipe it follows (Section 4.1); the word
"momentum" does not occur in it.  The reading taken: heavy-ball momentum in the
form used by that recipe's common implementation,

    g <- g + weight_decay * w        (coupled L2)
    v <- momentum * v + g            (dampening 0; v starts at 0)
    w <- w - lr * v                  (Nesterov: w <- w - lr * (g + momentum * v))
"""
import numpy as np


def sgd_step(w, v, g, lr, momentum, weight_decay=0.0, nesterov=False):
    """Return (w_new, v_new); inputs are not modified."""
    w = np.asarray(w, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64) + weight_decay * w
    v_new = momentum * v + g
    step = g + momentum * v_new if nesterov else v_new
    return w - lr * step, v_new
