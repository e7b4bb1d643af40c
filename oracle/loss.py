"""Codistillation loss and its gradient with respect to the local logits.

Test infrastructure (see the package docstring).  NumPy float64.

Follows the paper's Algorithm 1 (the objective inside the gradient of the
per-model update): supervised loss L plus alpha times the distillation term D
averaged over the n-1 peers.  L is cross-entropy (Section 2 names cross-entropy
or MSE; every experiment is classification or translation).  D is, by default,
the mean squared error between the raw, uncentred logits of the two models
(appendix, "Implementation Details"); the KL divergence that prior work used
(Section 2) is the second mode, and the centred variant of the squared error
that the same appendix reports trying (with similar results) the third.
Gradients flow only into the local logits (Section 3: the backward pass is
taken with respect to the local parameters only), so the peer logits are
constants.

Readings where the paper is silent:
  * cross-entropy is averaged over the N valid rows (target != ignore_index);
    ignored rows contribute nothing to L or D and get a zero gradient;
  * label smoothing eps mixes the one-hot target with the uniform distribution
    over all C classes, q = (1-eps) onehot + eps/C;
  * "mean squared error" is the mean over all N*C elements ("mean_all"); the
    per-row sum averaged over rows ("mean_rows") is offered as well;
  * KL is KL(p' || p) with the peer as target, mean over rows.  The paper uses no
    temperature; the optional one here is the usual form of distillation (Hinton
    et al.): both logit rows are divided by tau before the softmax and the term is
    multiplied by tau^2 (so that its gradient keeps its scale); tau = 1 is the
    paper's term;
  * "centring" the logits subtracts from each model's logit row its own mean
    over the classes before the squared error is taken ("mse_centered"); the
    normalisers are those of the uncentred term.
"""
import numpy as np


def log_softmax(z):
    """Row-wise log-softmax, log p = z - logsumexp(z)."""
    z = np.asarray(z, dtype=np.float64)
    m = z.max(axis=1, keepdims=True)
    lse = m + np.log(np.exp(z - m).sum(axis=1, keepdims=True))
    return z - lse


def codistill_loss_grad(z, z_peers, targets, alpha, label_smoothing=0.0,
                        dist="mse", mse_reduction="mean_all", ignore_index=-1, temperature=1.0):
    """Return ((total, task, distill), dz).

    z        [rows, cols] local logits
    z_peers  list of [rows, cols] peer logits (may be empty or None: plain
             supervised loss, as on iterations without exchanged predictions,
             Section 3)
    targets  [rows] integer class ids, ignore_index marks a row to skip
    """
    z = np.asarray(z, dtype=np.float64)
    targets = np.asarray(targets).astype(np.int64)
    rows, cols = z.shape
    valid = targets != ignore_index
    n_valid = int(valid.sum())
    if n_valid == 0:
        return (0.0, 0.0, 0.0), np.zeros_like(z)
    vmask = valid[:, None].astype(np.float64)

    # supervised term: cross-entropy against the (smoothed) target distribution
    logp = log_softmax(z)
    p = np.exp(logp)
    q = np.full((rows, cols), label_smoothing / cols)
    safe_t = np.where(valid, targets, 0)
    q[np.arange(rows), safe_t] += 1.0 - label_smoothing
    task = float(-(q * logp * vmask).sum() / n_valid)
    dz = (p - q) * vmask / n_valid

    # distillation term, averaged over the n-1 peers (Algorithm 1)
    distill = 0.0
    peers = [] if z_peers is None else list(z_peers)
    if len(peers) > 0:
        w = 1.0 / len(peers)
        for zp in peers:
            zp = np.asarray(zp, dtype=np.float64)
            if dist in ("mse", "mse_centered"):
                if dist == "mse_centered":
                    zc = z - z.mean(axis=1, keepdims=True)
                    zpc = zp - zp.mean(axis=1, keepdims=True)
                    diff = (zc - zpc) * vmask
                else:
                    diff = (z - zp) * vmask
                if mse_reduction == "mean_all":
                    denom = n_valid * cols
                elif mse_reduction == "mean_rows":
                    denom = n_valid
                else:
                    raise ValueError(mse_reduction)
                distill += w * float((diff ** 2).sum() / denom)
                # d/dz of the centred term: the centring projector I - 11^T/C is applied to a
                # difference whose rows already sum to zero, which leaves it unchanged
                dz += alpha * w * 2.0 * diff / denom
            elif dist == "kl":
                tau = float(temperature)
                logpt = log_softmax(z / tau)
                logpp = log_softmax(zp / tau)
                pp = np.exp(logpp)
                distill += w * tau * tau * float((pp * (logpp - logpt) * vmask).sum() / n_valid)
                # d/dz of tau^2 KL(softmax(z'/tau) || softmax(z/tau)) = tau (p_tau - p'_tau)
                dz += alpha * w * tau * (np.exp(logpt) - pp) * vmask / n_valid
            else:
                raise ValueError(dist)
    total = task + alpha * distill
    return (total, task, distill), dz
