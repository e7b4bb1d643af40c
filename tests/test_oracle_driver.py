"""Pins of the oracle's multi-step driver (Algorithm 1 in the checkpoint-exchange form of Section 3):
what the stale copies are at every update, simultaneity of the updates, the alpha = 0 special case,
and the behaviour codistillation is for (the models' predictions move towards each other)."""
import numpy as np

from oracle import nets
from oracle.driver import codistill_train
from oracle.step import codistill_step, unflatten
from paper_2010_02838_amd import synth

ARCH = nets.tiny_cnn()


def _thetas(n):
    return [synth.he_init(ARCH.params, 1 + i, jitter=0.05).astype(np.float64) for i in range(n)]


def _batches(k, i):
    return synth.images(6, 10, 10, 3, seed=100 + 7 * k + i).astype(np.float64), synth.labels(6, 10, seed=300 + 7 * k + i)


def test_alpha_zero_is_independent_sgd():
    th = _thetas(2)
    a = codistill_train(ARCH, th, _batches, 5, 1, 0.0, 0.1, 0.9, weight_decay=1e-3)
    b = codistill_train(ARCH, th, _batches, 5, 3, 0.0, 0.1, 0.9, weight_decay=1e-3)
    for i in range(2):
        np.testing.assert_array_equal(a["theta"][i], b["theta"][i])
        t, v = th[i].copy(), None
        for k in range(5):
            x, y = _batches(k, i)
            out = codistill_step(ARCH, t, [], x, y, 0.0, 0.1, 0.9, v=v, weight_decay=1e-3)
            t, v = out["theta"], out["v"]
        np.testing.assert_allclose(a["theta"][i], t, atol=1e-15)


def test_stale_copies_and_simultaneous_updates():
    th = _thetas(3)
    T, steps = 2, 5
    smooth = lambda k: 0.2 * 0.5 ** k          # label smoothing decayed over training (Section 4, translation)
    r = codistill_train(ARCH, th, _batches, steps, T, lambda k: 0.5 * 1.1 ** k, lambda k: 0.1 / (1 + k), 0.9,
                        label_smoothing=smooth)
    assert r["refreshed"] == [0, 2, 4]
    # replay by hand: the copies are the parameters at the last multiple of T, taken before that update
    theta, v = [t.copy() for t in th], [None] * 3
    for k in range(steps):
        if k % T == 0:
            stale = [t.copy() for t in theta]
        new = []
        for i in range(3):
            x, y = _batches(k, i)
            out = codistill_step(ARCH, theta[i], [stale[j] for j in range(3) if j != i], x, y, 0.5 * 1.1 ** k,
                                 0.1 / (1 + k), 0.9, v=v[i], label_smoothing=smooth(k))
            np.testing.assert_allclose(r["loss"][k][i], out["loss"], rtol=1e-14)
            new.append((out["theta"], out["v"]))
        theta, v = [a for a, _ in new], [b for _, b in new]
    for i in range(3):
        np.testing.assert_allclose(r["theta"][i], theta[i], atol=1e-15)
        assert r["distance_from_init"][-1][i] == np.linalg.norm(theta[i] - th[i])
    assert r["distance_from_init"].shape == (steps, 3) and np.all(r["distance_from_init"] > 0)
    # with T = 1 model 1 distils against model 0's parameters from before model 0's update of the same iteration
    r1 = codistill_train(ARCH, th[:2], _batches, 1, 1, 1.0, 0.1, 0.0)
    x, y = _batches(0, 1)
    ref = codistill_step(ARCH, th[1], [th[0]], x, y, 1.0, 0.1, 0.0)
    np.testing.assert_allclose(r1["theta"][1], ref["theta"], atol=1e-15)


def test_models_move_towards_each_other():
    th = _thetas(2)
    fixed = lambda k, i: (synth.images(16, 10, 10, 3, seed=5).astype(np.float64), synth.labels(16, 10, seed=6))
    x, _ = fixed(0, 0)

    def gap(thetas):
        z = [nets.forward(ARCH, unflatten(ARCH, t), x)[0] for t in thetas]
        return float(((z[0] - z[1]) ** 2).mean())

    solo = codistill_train(ARCH, th, fixed, 40, 1, 0.0, 0.05, 0.9)
    co = codistill_train(ARCH, th, fixed, 40, 1, 1.0, 0.05, 0.9)
    stale = codistill_train(ARCH, th, fixed, 40, 8, 4.0, 0.05, 0.9)
    # trained alone the two models drift apart; distilling against each other pulls their logits together,
    # also against copies that are 8 updates old
    assert gap(solo["theta"]) > gap(th)
    assert gap(co["theta"]) < 0.05 * gap(solo["theta"])
    assert gap(stale["theta"]) < 0.5 * gap(th)
    for r in (solo, co, stale):                       # the task loss goes down on the fixed batch
        assert (r["loss"][-1, :, 1] < r["loss"][0, :, 1]).all()
    assert co["loss"][-1, :, 2].max() < 0.1 * co["loss"][0, :, 2].min()   # and so does the distillation term


def test_prediction_exchange():
    """The other implementation of Section 3.  With an exchange at every update and the same minibatch for all
    models it is the checkpoint form with T = 1 (fresh copies predict on that minibatch); between exchanges a
    model takes plain supervised steps whatever alpha is."""
    th = _thetas(3)
    same = lambda k, i: _batches(k, 0)
    a = codistill_train(ARCH, th, same, 4, 1, 0.8, 0.1, 0.9, exchange="predictions")
    b = codistill_train(ARCH, th, same, 4, 1, 0.8, 0.1, 0.9, exchange="checkpoints")
    for i in range(3):
        np.testing.assert_array_equal(a["theta"][i], b["theta"][i])
    np.testing.assert_array_equal(a["loss"], b["loss"])
    # T = 3: updates 1 and 2 have no distillation term
    c = codistill_train(ARCH, th, _batches, 3, 3, 0.8, 0.1, 0.9, exchange="predictions")
    assert c["refreshed"] == [0]
    assert np.all(c["loss"][0, :, 2] > 0) and np.all(c["loss"][1:, :, 2] == 0)
    t, v = th[1].copy(), None
    x, y = _batches(0, 0)                                   # model 1 sees model 0's minibatch (coordinated sampling)
    out = codistill_step(ARCH, t, [th[0], th[2]], x, y, 0.8, 0.1, 0.9)
    t, v = out["theta"], out["v"]
    for k in (1, 2):
        x, y = _batches(k, 0)
        out = codistill_step(ARCH, t, [], x, y, 123.0, 0.1, 0.9, v=v)
        t, v = out["theta"], out["v"]
    np.testing.assert_allclose(c["theta"][1], t, atol=1e-15)
