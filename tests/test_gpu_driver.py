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


@pytest.mark.parametrize("n,T", [(2, 2), (3, 3)])
def test_small_resnet_bf16_trajectory(n, T):
    """Six updates of n bf16 ResNets (basic blocks on the matrix-core kernels) with checkpoint exchange every T.
    Every update of every model is checked teacher forced: the oracle's step from the weights and the stale copies
    the GPU model holds at that update gives the loss terms (stated tolerance 2e-2) and, applied to the GPU's own
    gradient, the new weights and momentum; the stale copies must be the peers' bf16 weights of the last exchange,
    bit for bit, and must not follow the peers' updates in between.  The free-running float64 trajectory from the
    same start is compared on the loss of every update as well."""
    from oracle.step import codistill_step
    from oracle.sgd import sgd_step
    from paper_2010_02838_amd import binding as B
    from paper_2010_02838_amd.driver import CodistillTrainer
    from paper_2010_02838_amd.runner import pack_flat, unpack_flat, to_device
    arch = nets.resnet20(widths=(16, 24, 40), blocks=(1, 2, 1))
    kw = dict(widths=[16, 24, 40], blocks=[1, 2, 1], stem_width=16, in_h=20, in_w=20, classes=10)
    steps, batch, res, mu = 6, 8, 20, 0.9
    th = [synth.round_bf16(synth.he_init(arch.params, 1 + i, jitter=0.1)) for i in range(n)]
    host = lambda k, i: (synth.round_bf16(synth.images(batch, res, res, 3, seed=100 + 7 * k + i)),
                         synth.labels(batch, 10, seed=300 + 7 * k + i))
    alpha, lr, wd = (lambda k: 0.5 * 1.2 ** k), (lambda k: 0.05 / (1 + 0.25 * k)), (lambda k: 1e-3 * 0.5 ** k)
    free = codistill_train(arch, [t.astype(np.float64) for t in th],
                           lambda k, i: (host(k, i)[0].astype(np.float64), host(k, i)[1]), steps, T, alpha, lr, mu,
                           weight_decay=wd)
    models = [B.Model(B.arch_preset(B.CD_ARCH_RESNET_BASIC, **kw), B.CD_BF16) for _ in range(n)]
    assert models[0].param_table() == [(a, tuple(s), k, f) for a, s, k, f in arch.params]
    tr = CodistillTrainer(models, batch)
    tr.load([pack_flat(models[i], th[i]) for i in range(n)])
    dev = lambda k, i: (to_device(host(k, i)[0], torch.bfloat16), torch.from_numpy(host(k, i)[1]).to("cuda:0"))
    bits = lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)
    dense = lambda m, b: unpack_flat(m, synth.bf16_to_f32(b)).astype(np.float64)
    stale, worst, worst_free = None, 0.0, 0.0
    for k in range(steps):
        torch.cuda.synchronize()
        before = [(r.master.cpu().numpy().copy(), r.momentum.cpu().numpy().copy(), bits(r.lowp).copy()) for r in tr.runners]
        if k % T == 0:
            stale = [b[2] for b in before]            # what an exchange at this update hands out
        losses = tr.step(dev, T, alpha, lr, mu, weight_decay=wd)
        torch.cuda.synchronize()
        for i, r in enumerate(tr.runners):
            peers = [j for j in range(n) if j != i]
            for slot, j in zip(r.peer_params, peers):
                np.testing.assert_array_equal(bits(slot), stale[j])
                assert not np.array_equal(bits(slot), bits(tr.runners[j].lowp))   # the peer has moved on since
            x, y = host(k, i)
            ref = codistill_step(arch, dense(models[i], before[i][2]), [dense(models[j], stale[j]) for j in peers],
                                 x.astype(np.float64), y, alpha(k), lr(k), mu, weight_decay=wd(k))
            got = losses[i].cpu().numpy()[:3].astype(np.float64)
            e = float(np.abs(got - ref["loss"]).max() / abs(ref["loss"][0]))
            worst = max(worst, e)
            assert e <= 2e-2, (k, i, got, ref["loss"])
            worst_free = max(worst_free, float(np.abs(got - free["loss"][k][i]).max() / abs(free["loss"][k][i][0])))
            w_new, v_new = sgd_step(before[i][0].astype(np.float64), before[i][1].astype(np.float64),
                                    r.grads.cpu().numpy().astype(np.float64), lr(k), mu, wd(k), False)
            assert rel(r.master.cpu().numpy(), w_new) <= 1e-6 and rel(r.momentum.cpu().numpy(), v_new) <= 1e-6
            np.testing.assert_array_equal(bits(r.lowp), synth.bf16_bits(r.master.cpu().numpy()))
    print("bf16 trajectory n=%d T=%d: worst loss error, teacher forced %.2e, against the free-running float64 run %.2e"
          % (n, T, worst, worst_free))
    assert worst_free <= 2e-2
