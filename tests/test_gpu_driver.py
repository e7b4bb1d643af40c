"""GPU parity of several codistillation updates of two and three models (checkpoint exchange every T
updates, scheduled alpha / learning rate / weight decay) against the oracle's driver."""
import numpy as np
import pytest
import torch

from oracle import nets
from oracle.driver import codistill_train
from paper_2010_02838_amd import synth

from gpu_util import rel

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n,T", [(2, 2), (3, 1), (2, 4)])
def test_tiny_cnn_fp32_trajectory(n, T):
    from paper_2010_02838_amd import binding as B
    from paper_2010_02838_amd.driver import CodistillTrainer
    from paper_2010_02838_amd.runner import pack_flat, unpack_flat
    arch = nets.tiny_cnn()
    steps, batch, res = 6, 8, 16
    th = [synth.he_init(arch.params, 1 + i, jitter=0.05) for i in range(n)]
    host = lambda k, i: (synth.images(batch, res, res, 3, seed=100 + 7 * k + i), synth.labels(batch, 10, seed=300 + 7 * k + i))
    alpha, lr, wd = (lambda k: 0.5 * 1.1 ** k), (lambda k: 0.1 / (1 + 0.5 * k)), (lambda k: 1e-3 * 0.5 ** k)
    smooth = lambda k: 0.2 * 0.5 ** k
    ref = codistill_train(arch, [t.astype(np.float64) for t in th],
                          lambda k, i: (host(k, i)[0].astype(np.float64), host(k, i)[1]), steps, T, alpha, lr, 0.9,
                          weight_decay=wd, label_smoothing=smooth)
    kw = dict(in_h=res, in_w=res)
    models = [B.Model(B.arch_preset(B.CD_ARCH_TINY_CNN, **kw), B.CD_F32) for _ in range(n)]
    tr = CodistillTrainer(models, batch)
    tr.load([pack_flat(models[i], th[i]) for i in range(n)])
    dev = lambda k, i: (torch.from_numpy(host(k, i)[0]).to("cuda:0"), torch.from_numpy(host(k, i)[1]).to("cuda:0"))
    for k in range(steps):
        losses = tr.step(dev, T, alpha, lr, 0.9, weight_decay=wd, label_smoothing=smooth)
        for i in range(n):
            got = losses[i].cpu().numpy()[:3]
            np.testing.assert_allclose(got, ref["loss"][k][i], rtol=2e-4, atol=1e-6)
    torch.cuda.synchronize()
    np.testing.assert_allclose(tr.distance_from_init(), ref["distance_from_init"][-1], rtol=1e-4)
    for i in range(n):
        got = unpack_flat(models[i], tr.runners[i].master.cpu().numpy())
        assert rel(got, ref["theta"][i]) <= 1e-4


@pytest.mark.parametrize("n,T", [(2, 1), (3, 2)])
def test_tiny_cnn_fp32_prediction_exchange(n, T):
    """The prediction-exchange form: one forward pass per model on a shared minibatch, logits swapped every T updates."""
    from paper_2010_02838_amd import binding as B
    from paper_2010_02838_amd.driver import CodistillTrainer
    from paper_2010_02838_amd.runner import pack_flat, unpack_flat
    arch = nets.tiny_cnn()
    steps, batch, res = 5, 8, 16
    th = [synth.he_init(arch.params, 1 + i, jitter=0.05) for i in range(n)]
    host = lambda k, i: (synth.images(batch, res, res, 3, seed=100 + 7 * k + i), synth.labels(batch, 10, seed=300 + 7 * k + i))
    alpha = lambda k: 0.5 * 1.1 ** k
    ref = codistill_train(arch, [t.astype(np.float64) for t in th],
                          lambda k, i: (host(k, i)[0].astype(np.float64), host(k, i)[1]), steps, T, alpha, 0.1, 0.9,
                          exchange="predictions")
    models = [B.Model(B.arch_preset(B.CD_ARCH_TINY_CNN, in_h=res, in_w=res), B.CD_F32) for _ in range(n)]
    tr = CodistillTrainer(models, batch)
    tr.load([pack_flat(models[i], th[i]) for i in range(n)])
    dev = lambda k, i: (torch.from_numpy(host(k, i)[0]).to("cuda:0"), torch.from_numpy(host(k, i)[1]).to("cuda:0"))
    for k in range(steps):
        losses = tr.step(dev, T, alpha, 0.1, 0.9, exchange="predictions")
        for i in range(n):
            np.testing.assert_allclose(losses[i].cpu().numpy()[:3], ref["loss"][k][i], rtol=2e-4, atol=1e-6)
    torch.cuda.synchronize()
    for i in range(n):
        assert rel(unpack_flat(models[i], tr.runners[i].master.cpu().numpy()), ref["theta"][i]) <= 1e-4
