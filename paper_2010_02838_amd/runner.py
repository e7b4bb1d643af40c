"""Buffer management around the four C-ABI calls of one codistillation step.

Plumbing only: allocates the device tensors (PyTorch), moves host arrays in and
out, and calls the entry points in the order of the paper's Algorithm 1 / the
checkpoint-exchange implementation of Section 3.  No arithmetic of the step
lives here.
"""
import numpy as np
import torch

from . import binding as B
from . import synth


def pack_flat(model, dense):
    """Dense concatenation of the parameter tensors -> the library's flat layout (8-element aligned)."""
    out = np.zeros(model.n_elements, dtype=np.float32)
    off = 0
    for p in model.params:
        out[p["offset"]:p["offset"] + p["size"]] = dense[off:off + p["size"]]
        off += p["size"]
    assert off == len(dense)
    return out


def unpack_flat(model, flat):
    return np.concatenate([np.asarray(flat[p["offset"]:p["offset"] + p["size"]]) for p in model.params])


def to_device(arr, torch_dtype, device="cuda:0"):
    """float32 host array -> device tensor of the model's storage type (bf16: round-to-nearest-even bits)."""
    arr = np.ascontiguousarray(arr, dtype=np.float32)
    if torch_dtype == torch.bfloat16:
        bits = torch.from_numpy(synth.bf16_bits(arr).view(np.int16).reshape(arr.shape))
        return bits.to(device).view(torch.bfloat16)
    return torch.from_numpy(arr).to(device)


class StepRunner:
    """One model's training state plus the stale peer copies it distils against."""

    def __init__(self, model, peer_models, batch, device="cuda:0", overlap_peers=True):
        self.model, self.peers, self.batch, self.dev = model, list(peer_models), batch, device
        # The peer forwards depend on nothing but the minibatch: they run on a second stream (default
        # priority) beside the local forward, so that one model's memory-bound kernels and partly
        # filled launches share the chip with the other's.
        self.overlap_peers = overlap_peers
        self.side = torch.cuda.Stream(device=device) if overlap_peers else None
        n, C = model.n_elements, model.classes
        f32 = dict(dtype=torch.float32, device=device)
        self.master = torch.zeros(n, **f32)
        self.momentum = torch.zeros(n, **f32)
        self.second_moment = None   # Adam's second buffer, allocated on the first step_adam
        self.updates = 0            # Adam's update counter
        self.grads = torch.empty(n, **f32)
        self.lowp = torch.zeros(n, dtype=torch.bfloat16, device=device) if model.dtype == B.CD_BF16 else None
        self.ws = torch.empty(model.workspace_bytes(batch, True), dtype=torch.uint8, device=device)
        self.peer_params = [torch.zeros(pm.n_elements, dtype=pm.torch_dtype, device=device) for pm in self.peers]
        wsp = max([pm.workspace_bytes(batch, False) for pm in self.peers] + [256])
        self.ws_peer = torch.empty(wsp, dtype=torch.uint8, device=device)
        rows = batch * model.rows_per_sample
        self.logits = torch.empty(rows, C, **f32)
        self.peer_logits = [torch.empty(rows, C, **f32) for _ in self.peers]
        self.dz = torch.empty(rows, C, **f32)
        self.loss = torch.zeros(4, **f32)
        self.scratch = torch.empty(B.loss_scratch_bytes(rows, C), dtype=torch.uint8, device=device)

    def params(self):
        return self.lowp if self.lowp is not None else self.master

    def load(self, theta, theta_peers, v=None):
        """theta, theta_peers[j], v: float32 host arrays in the library's flat layout."""
        self.master.copy_(torch.from_numpy(np.ascontiguousarray(theta, dtype=np.float32)))
        if self.lowp is not None:
            self.lowp.copy_(to_device(theta, torch.bfloat16, self.dev))
        for t, pm, th in zip(self.peer_params, self.peers, theta_peers):
            t.copy_(to_device(th, pm.torch_dtype, self.dev))
        if v is None:
            self.momentum.zero_()
        else:
            self.momentum.copy_(torch.from_numpy(np.ascontiguousarray(v, dtype=np.float32)))

    def forward_local(self, x):
        """The local model's forward pass alone (logits in self.logits, activations kept for the backward pass)."""
        B.codistill_forward(self.model, self.params(), x, self.ws, self.logits, True)

    def finish(self, x, y, peer_logits, alpha, lr, momentum, weight_decay=0.0, label_smoothing=0.0,
               dist_kind=B.CD_DIST_MSE_LOGITS, mse_reduction=B.CD_MEAN_ALL, ignore_index=-1, nesterov=False, adam=None,
               temperature=1.0):
        """Loss against the given peer logits (a list of [rows, classes] fp32 device tensors, possibly empty: the
        predictions other models sent, or none on an iteration without exchange), backward pass, update."""
        B.codistill_loss_grad(self.logits, peer_logits, y, self.loss, self.dz, self.scratch, alpha,
                              label_smoothing, dist_kind, mse_reduction, ignore_index, temperature)
        B.codistill_backward(self.model, self.params(), x, self.ws, self.dz, self.grads)
        t0 = self.model.trainable_offset      # a frozen front end (first in the flat buffers) is left out of the update
        lowp = None if self.lowp is None else self.lowp[t0:]
        if adam is None:
            B.codistill_sgd_step(self.master[t0:], self.momentum[t0:], self.grads[t0:], lowp, lr, momentum, weight_decay,
                                 nesterov)
        else:   # the momentum buffer holds Adam's first moment
            if self.second_moment is None:
                self.second_moment = torch.zeros_like(self.momentum)
            self.updates += 1
            B.codistill_adam_step(self.master[t0:], self.momentum[t0:], self.second_moment[t0:], self.grads[t0:], lowp, lr,
                                  self.updates, adam[0], adam[1], adam[2], weight_decay)

    def step(self, x, y, alpha, lr, momentum, weight_decay=0.0, label_smoothing=0.0,
             dist_kind=B.CD_DIST_MSE_LOGITS, mse_reduction=B.CD_MEAN_ALL, ignore_index=-1, nesterov=False, adam=None,
             temperature=1.0):
        """x: [B,H,W,3] device tensor in the model dtype (the Transformer: int32 [B, source + target tokens]);
        y: int32 device tensor, one target per row of logits.  adam = (beta1, beta2, eps) replaces the momentum-SGD
        update by Adam (momentum and nesterov are then unused)."""
        if self.overlap_peers and self.peers:
            main = torch.cuda.current_stream()
            self.side.wait_stream(main)           # x, the peer parameters and the last step's reads are in order
            with torch.cuda.stream(self.side):
                for pm, pp, pl in zip(self.peers, self.peer_params, self.peer_logits):
                    B.codistill_forward(pm, pp, x, self.ws_peer, pl, False)
            self.forward_local(x)
            main.wait_stream(self.side)           # the loss needs every model's logits
        else:
            self.forward_local(x)
            for pm, pp, pl in zip(self.peers, self.peer_params, self.peer_logits):
                B.codistill_forward(pm, pp, x, self.ws_peer, pl, False)
        self.finish(x, y, self.peer_logits, alpha, lr, momentum, weight_decay, label_smoothing, dist_kind, mse_reduction,
                    ignore_index, nesterov, adam, temperature)
