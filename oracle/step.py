"""One codistillation training step of one model, NumPy float64.

Test infrastructure (see the package docstring).  Follows the paper's
Algorithm 1 (the per-model update) in the checkpoint-exchange implementation of
Section 3: the device runs the forward pass of its own model and of a stale
copy of each peer on the same minibatch, takes the backward pass with respect
to its own parameters only, and updates them.
"""
import numpy as np
from . import nets, sgd
from .loss import codistill_loss_grad


def unflatten(arch, flat):
    """Split a flat parameter vector (declaration order) into a dict of float64 arrays."""
    out, off = {}, 0
    flat = np.asarray(flat)
    for name, shape, _, _ in arch.params:
        n = int(np.prod(shape))
        out[name] = flat[off:off + n].astype(np.float64).reshape(shape)
        off += n
    assert off == flat.size
    return out


def flatten(arch, d):
    return np.concatenate([np.asarray(d[name], dtype=np.float64).ravel() for name, _, _, _ in arch.params])


def codistill_step(arch, theta, theta_peers, x, y, alpha, lr, momentum, v=None,
                   weight_decay=0.0, label_smoothing=0.0, dist="mse",
                   mse_reduction="mean_all", ignore_index=-1, nesterov=False,
                   peer_archs=None, perturb=None, perturb_peers=None):
    """theta, theta_peers[j], v: flat vectors.  Returns a dict with logits, peer
    logits, losses, dlogits, flat gradient, updated flat parameters and momentum.
    perturb, perturb_peers[j]: see nets.forward (None = the plain float64 step)."""
    p_local = unflatten(arch, theta)
    z, tape = nets.forward(arch, p_local, x, perturb=perturb)                # local forward
    z_peers = []
    for j, th in enumerate(theta_peers):                           # peer forwards: constants
        pa = arch if peer_archs is None else peer_archs[j]
        zp, _ = nets.forward(pa, unflatten(pa, th), x,
                             perturb=None if perturb_peers is None else perturb_peers[j])
        z_peers.append(zp)
    losses, dz = codistill_loss_grad(z, z_peers, y, alpha, label_smoothing, dist,
                                     mse_reduction, ignore_index)
    grads = nets.backward(arch, p_local, tape, dz)                 # local backward only
    g = flatten(arch, grads)
    v0 = np.zeros_like(g) if v is None else np.asarray(v, dtype=np.float64)
    w_new, v_new = sgd.sgd_step(np.asarray(theta, dtype=np.float64), v0, g, lr, momentum,
                                weight_decay, nesterov)
    if arch.frozen:                                                # frozen parameters are left out of the update
        off = 0
        for name, shape, _, _ in arch.params:
            n = int(np.prod(shape))
            if name in arch.frozen:
                w_new[off:off + n] = np.asarray(theta, dtype=np.float64)[off:off + n]
                v_new[off:off + n] = v0[off:off + n]
            off += n
    return dict(logits=z, peer_logits=z_peers, loss=losses, dlogits=dz, grad=g,
                grads=grads, theta=w_new, v=v_new)
