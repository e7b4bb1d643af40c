"""Several codistillation steps of n models on one GPU, in the checkpoint-exchange or the prediction-exchange form.

Host logic only (paper, Algorithm 1 and Section 3): every model owns a StepRunner; the copies of its
peers' parameters that it distils against are refreshed every `exchange_every` updates by device
copies of the peers' current weights, and stay stale in between.  Schedules are plain functions of
the update index.  Every step runs through the four C-ABI calls.
"""
import torch

from . import binding as B
from .runner import StepRunner


class CodistillTrainer:
    def __init__(self, models, batch, device="cuda:0"):
        """models: one binding.Model per participant (same dtype).  Peer slots are models of the peers' architectures."""
        self.n = len(models)
        self.models = models
        self.runners = []
        for i, m in enumerate(models):
            peers = [B.Model(models[j].arch, models[j].dtype) for j in range(self.n) if j != i]
            self.runners.append(StepRunner(m, peers, batch, device))
        self.k = 0

    def load(self, thetas):
        """thetas[i]: float32 host array in model i's flat layout.  The stale copies start equal to them."""
        for i, r in enumerate(self.runners):
            r.load(thetas[i], [thetas[j] for j in range(self.n) if j != i])
        self.first = [r.master.clone() for r in self.runners]

    def distance_from_init(self):
        """L2 distance of every model's fp32 weights from the ones loaded (the diagnostic the paper's appendix plots:
        codistillation keeps the parameters closer to their initial values).  Synchronises."""
        return [float(torch.linalg.vector_norm((r.master - f).double())) for r, f in zip(self.runners, self.first)]

    def exchange(self):
        """Refresh every model's stale copies from the peers' current weights (device to device)."""
        # Stream order is enough: every step has joined its side streams back into the current stream, and
        # the next step's side stream waits for the current stream before it reads the copies.
        for i, r in enumerate(self.runners):
            src = [self.runners[j].params() for j in range(self.n) if j != i]
            for dst, s in zip(r.peer_params, src):
                dst.copy_(s)

    def step(self, batches, exchange_every, alpha, lr, momentum, weight_decay=0.0, label_smoothing=0.0,
             dist_kind=B.CD_DIST_MSE_LOGITS, exchange="checkpoints"):
        """One update of every model.  batches(k, i) -> (x, y) device tensors.  Returns the [n][3] losses as device tensors.
        exchange = "predictions": the other implementation of Section 3.  All models process the minibatch
        batches(k, 0); on every exchange_every-th update each distils against the logits the others just computed
        (their one forward pass each), on the other updates the distillation term is left out."""
        k = self.k
        sched = lambda s: s(k) if callable(s) else s
        kw = dict(weight_decay=sched(weight_decay), label_smoothing=sched(label_smoothing), dist_kind=dist_kind)
        out = []
        if exchange == "predictions":
            x, y = batches(k, 0)
            for r in self.runners:
                r.forward_local(x)
            send = k % exchange_every == 0
            for i, r in enumerate(self.runners):
                peers = [q.logits for j, q in enumerate(self.runners) if j != i] if send else []
                r.finish(x, y, peers, sched(alpha), sched(lr), momentum, **kw)
                out.append(r.loss.clone())
        elif exchange == "checkpoints":
            if k % exchange_every == 0:
                self.exchange()
            for i, r in enumerate(self.runners):
                x, y = batches(k, i)
                r.step(x, y, sched(alpha), sched(lr), momentum, **kw)
                out.append(r.loss.clone())
        else:
            raise ValueError(exchange)
        self.k += 1
        return out
