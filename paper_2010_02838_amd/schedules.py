"""Host-side schedules of the scalars a codistillation step takes (learning rate, L2 coefficient, alpha, label
smoothing), as functions of the update index k, in the forms the paper describes (Section 4.1 and the appendix on
experimental details).  Plain Python: the step itself receives the numbers.

The constants the paper prints are in PAPER; where the main text and the appendix disagree (the initial L2
coefficient) both are kept.
"""
import math

PAPER = {
    "lr_decay_factor": 0.1,                       # three step-wise decreases
    "lr_milestone_epochs_allreduce": (15, 30, 40),
    "lr_milestone_epochs_codistillation": (18, 38, 44),   # moved later: the training loss saturates more slowly
    "l2_initial_main_text": 5e-4,
    "l2_initial_appendix": 1e-4,
    "l2_after_first_lr_decay": 1e-5,
    "l2_after_second_lr_decay": 0.0,
    "alpha_growth_per_epoch_translation": 1.1,
    "tokens_per_gpu_translation": 3854,
    "per_gpu_batch_imagenet": 32,
}


def linear_scaled_lr(total_batch, base_lr=0.1, base_batch=256):
    """Peak learning rate proportional to the total minibatch size (the large-minibatch recipe the paper adopts)."""
    return base_lr * total_batch / base_batch


def warmup_step_lr(peak, warmup_iters, milestones, factor=0.1, start=None):
    """Linear warm-up from `start` (default peak / 10) to `peak` over warmup_iters updates, then the rate is multiplied
    by `factor` at every milestone (update indices)."""
    start = peak * 0.1 if start is None else start

    def lr(k):
        if k < warmup_iters:
            return start + (peak - start) * k / warmup_iters
        return peak * factor ** sum(1 for m in milestones if k >= m)
    return lr


def half_cosine_lr(peak, warmup_iters, total_iters, start=0.0):
    """Linear warm-up, then half a cosine period from `peak` down to zero at total_iters."""
    def lr(k):
        if k < warmup_iters:
            return start + (peak - start) * k / warmup_iters
        t = min(1.0, (k - warmup_iters) / max(1, total_iters - warmup_iters))
        return 0.5 * peak * (1.0 + math.cos(math.pi * t))
    return lr


def stepped_l2(initial, milestones, later=(PAPER["l2_after_first_lr_decay"], PAPER["l2_after_second_lr_decay"])):
    """The L2 coefficient that codistillation needs: `initial` until the first learning-rate decay, then later[0], then
    later[1] from the second decay on (milestones: the update indices of those decays)."""
    def wd(k):
        passed = sum(1 for m in milestones[:len(later)] if k >= m)
        return initial if passed == 0 else later[passed - 1]
    return wd


def geometric(value0, growth, iters_per_epoch):
    """value0 * growth^epoch: alpha grown by 1.1 per epoch in the translation runs; with growth < 1, a decaying
    label smoothing."""
    return lambda k: value0 * growth ** (k // iters_per_epoch)
