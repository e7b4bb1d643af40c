"""CPU float64 oracle of one codistillation training step.

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain definition that the
GPU library is checked against; it is imported by the tests, by the smoke check
and by the benchmark's CPU-baseline leg, never by the product path.  It shares
no code with the HIP implementation and imports nothing from it.

What it computes (paper, Algorithm 1, the per-model update; Section 3, the
checkpoint-exchange implementation; appendix "Implementation Details" for the
choice of the distillation term):

    z   = f_theta(x)                  training-mode forward of the local model
    z'  = f_theta'(x)                 forward of the (stale) peer, a constant
    l   = L(y, z) + alpha * 1/(n-1) * sum_j D(z, z'_j)
    g   = d l / d theta               backward through the local model only
    theta <- momentum-SGD(theta, g)

Everything is NumPy float64.  Parity status: every function here is pinned by
the CPU tests (closed forms, invariants, brute force, finite differences and a
library autograd cross-check); the accuracy / loss / BLEU figures printed in
the paper need its datasets and full training runs and are "parity unpinned".
"""
from . import loss, layers, nets, sgd, step, driver  # noqa: F401
