"""Several codistillation steps of n models in the checkpoint-exchange form, NumPy float64.

Test infrastructure (see the package docstring).  Paper, Algorithm 1 (all models take a step per
iteration, each against the others' predictions) in the implementation of Section 3: every model
keeps a copy of each peer's parameters that is refreshed only every T updates, and between refreshes
distils against the predictions of those stale copies on its own minibatch.  Schedules (learning
rate, alpha, weight decay) are plain functions of the update index; the paper's experiments grow alpha
and decay the L2 term over training (Section 4), here they are whatever the caller passes.
"""
import numpy as np

from .step import codistill_step


def codistill_train(arch, thetas, batches, steps, exchange_every, alpha, lr, momentum,
                    weight_decay=0.0, label_smoothing=0.0, dist="mse", exchange="checkpoints"):
    """thetas: list of n flat parameter vectors (one per model).
    batches(k, i) -> (x, y): the minibatch of model i at update k.
    alpha, lr, weight_decay, label_smoothing: numbers or functions of the update index k (Section 4 grows alpha and
    decays the L2 term or, for translation, the label smoothing over training).
    exchange: "checkpoints" (above), or "predictions", the other implementation of Section 3: all models process
    the same minibatch batches(k, 0) (coordinated sampling); on every T-th update each model distils against the
    predictions its peers make with their current parameters, on the other updates the distillation term is left out.
    Returns dict(theta=[...], v=[...], loss=[steps][n][3], refreshed=[update indices of exchanges])."""
    if exchange not in ("checkpoints", "predictions"):
        raise ValueError(exchange)
    n = len(thetas)
    sched = lambda s, k: s(k) if callable(s) else s
    theta = [np.asarray(t, dtype=np.float64).copy() for t in thetas]
    first = [t.copy() for t in theta]
    distance = []                                # per update and model: the L2 distance of the parameters from their
                                                 # initial values (the diagnostic of the appendix on regularisation)
    v = [np.zeros_like(t) for t in theta]
    stale = [t.copy() for t in theta]
    losses, refreshed = [], []
    for k in range(steps):
        if k % exchange_every == 0:              # checkpoint exchange: everybody's copies are refreshed
            stale = [t.copy() for t in theta]
            refreshed.append(k)
        row, new_theta, new_v = [], [], []
        for i in range(n):                       # all models step from the same (old) state
            if exchange == "predictions":
                x, y = batches(k, 0)
                peers = [theta[j] for j in range(n) if j != i] if k % exchange_every == 0 else []
            else:
                x, y = batches(k, i)
                peers = [stale[j] for j in range(n) if j != i]
            out = codistill_step(arch, theta[i], peers, x, y, sched(alpha, k), sched(lr, k), momentum, v=v[i],
                                 weight_decay=sched(weight_decay, k), label_smoothing=sched(label_smoothing, k), dist=dist)
            row.append(out["loss"])
            new_theta.append(out["theta"])
            new_v.append(out["v"])
        theta, v = new_theta, new_v
        losses.append(row)
        distance.append([float(np.linalg.norm(theta[i] - first[i])) for i in range(n)])
    return dict(theta=theta, v=v, loss=np.asarray(losses, dtype=np.float64), refreshed=refreshed,
                distance_from_init=np.asarray(distance))
