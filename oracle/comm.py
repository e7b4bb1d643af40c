"""Bits each device communicates per iteration (Section 3 of the paper), plain Python.

Test infrastructure (see the package docstring).  b_model: bits of the parameters; b_pred: bits of one sample's
predictions; B: per-device batch; n models codistil, exchanging every T iterations.
"""


def allreduce_bits(b_model):
    """Ring or tree all-reduce: 2 b_model per iteration."""
    return 2.0 * b_model


def checkpoint_bits(b_model, n, T):
    """Codistillation exchanging checkpoints every T iterations: (n - 1) b_model / T on average."""
    return (n - 1) * b_model / T


def prediction_bits(b_pred, B, n, T):
    """Codistillation exchanging predictions every T iterations: (n - 1) b_pred B / T on average."""
    return (n - 1) * b_pred * B / T
