"""Pins of the oracle's LayerNorm and of its Transformer output block (feed-forward sublayer, residual,
post-LayerNorm, projection onto the vocabulary): closed forms, invariants, a library routine, finite
differences.  The block as a whole is also covered by the library-autograd and finite-difference step
tests in test_oracle_step.py.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import layers as L
from oracle import nets
from oracle.step import codistill_step
from paper_2010_02838_amd import synth


def _case(rows=7, d=12, seed=0):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((rows, 1, 1, d)) * 2.0 + 0.7
    g = 1.0 + 0.3 * rng.standard_normal(d)
    b = 0.2 * rng.standard_normal(d)
    dy = rng.standard_normal(x.shape)
    return x, g, b, dy


def test_layernorm_closed_forms():
    x, g, b, dy = _case()
    d = x.shape[-1]
    y, (xhat, rstd) = L.layernorm_forward(x, np.ones(d), np.zeros(d))
    var = x.var(axis=-1, keepdims=True)
    # rows have zero mean and variance var / (var + eps)
    np.testing.assert_allclose(y.mean(axis=-1), 0.0, atol=1e-14)
    np.testing.assert_allclose(y.var(axis=-1, keepdims=True), var / (var + 1e-5), rtol=1e-12)
    # affine part
    y2, _ = L.layernorm_forward(x, g, b)
    np.testing.assert_allclose(y2, y * g + b, atol=1e-14)
    # a row of one repeated value normalises to beta (variance 0: only eps in the denominator)
    yc, _ = L.layernorm_forward(np.full((1, 1, 1, d), 3.25), g, b)
    np.testing.assert_allclose(yc[0, 0, 0], b, atol=1e-12)
    # two-element rows: xhat = +-(a-b)/2 / sqrt((a-b)^2/4 + eps)
    a2 = np.array([[[[1.5, -0.5]]]])
    y3, _ = L.layernorm_forward(a2, np.ones(2), np.zeros(2))
    h = 1.0 / np.sqrt(1.0 + 1e-5)
    np.testing.assert_allclose(y3[0, 0, 0], [h, -h], rtol=1e-14)


def test_layernorm_invariants():
    x, g, b, dy = _case(seed=1)
    y, cache = L.layernorm_forward(x, g, b)
    # shifting a row by a constant changes nothing; scaling it changes the result only through eps
    y_shift, _ = L.layernorm_forward(x + 11.0, g, b)
    np.testing.assert_allclose(y_shift, y, atol=1e-12)
    var = x.var(axis=-1, keepdims=True)
    y_scale, _ = L.layernorm_forward(3.0 * x, g, b)
    np.testing.assert_allclose(y_scale - b, (y - b) * np.sqrt((var + 1e-5) / (var + 1e-5 / 9.0)), rtol=1e-11, atol=1e-13)
    dx, dg, db = L.layernorm_backward(dy, g, cache)
    xhat, rstd = cache
    # the input gradient of a row sums to zero, and its component along xhat is the eps remainder
    np.testing.assert_allclose(dx.sum(axis=-1), 0.0, atol=1e-13)
    gg = dy * g
    np.testing.assert_allclose((dx * xhat).sum(axis=-1, keepdims=True),
                               rstd * (gg * xhat).sum(axis=-1, keepdims=True) * 1e-5 / (var + 1e-5), rtol=1e-9, atol=1e-15)
    np.testing.assert_allclose(db, dy.sum(axis=(0, 1, 2)), atol=1e-13)


def test_layernorm_matches_library():
    x, g, b, dy = _case(rows=6, d=10, seed=2)
    y, cache = L.layernorm_forward(x, g, b)
    dx, dg, db = L.layernorm_backward(dy, g, cache)
    xt, gt, bt = (torch.tensor(v, requires_grad=True) for v in (x, g, b))
    yt = F.layer_norm(xt, (x.shape[-1],), gt, bt, 1e-5)
    yt.backward(torch.tensor(dy))
    np.testing.assert_allclose(y, yt.detach().numpy(), atol=1e-13)
    np.testing.assert_allclose(dx, xt.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dg, gt.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(db, bt.grad.numpy(), atol=1e-12)


def test_layernorm_backward_by_finite_differences():
    x, g, b, dy = _case(rows=3, d=6, seed=3)
    _, cache = L.layernorm_forward(x, g, b)
    dx, dg, db = L.layernorm_backward(dy, g, cache)
    f = lambda xx, gg, bb: float((L.layernorm_forward(xx, gg, bb)[0] * dy).sum())
    h = 1e-6
    rng = np.random.default_rng(0)
    for _ in range(6):
        i = tuple(int(rng.integers(0, n)) for n in x.shape)
        e = np.zeros_like(x); e[i] = h
        assert (f(x + e, g, b) - f(x - e, g, b)) / (2 * h) == pytest.approx(dx[i], rel=1e-6, abs=1e-8)
    for j in range(x.shape[-1]):
        e = np.zeros_like(g); e[j] = h
        assert (f(x, g + e, b) - f(x, g - e, b)) / (2 * h) == pytest.approx(dg[j], rel=1e-6, abs=1e-8)
        assert (f(x, g, b + e) - f(x, g, b - e)) / (2 * h) == pytest.approx(db[j], rel=1e-6, abs=1e-8)


def test_transformer_head_structure():
    a = nets.transformer_head()
    # 512*2048 + 2048 + 2048*512 + 512 (feed-forward) + 2*512 (LayerNorm) + 32768*512 (projection)
    assert a.n_params() == 512 * 2048 + 2048 + 2048 * 512 + 512 + 1024 + 32768 * 512
    small = nets.transformer_head(8, 16, 12)
    rng = np.random.default_rng(4)
    P = {n: rng.standard_normal(s) * 0.3 for n, s, _, _ in small.params}
    x = rng.standard_normal((5, 1, 1, 8))
    z, _ = nets.forward(small, P, x)
    # written out: h + W2 relu(W1 h + b1) + b2 -> LayerNorm -> projection; rows are independent
    hrow = x[:, 0, 0, :]
    u = np.maximum(hrow @ P["ffn.w1.w"][:, 0, 0, :].T + P["ffn.w1.b"], 0.0) @ P["ffn.w2.w"][:, 0, 0, :].T + P["ffn.w2.b"]
    s = hrow + u
    sn = (s - s.mean(1, keepdims=True)) / np.sqrt(s.var(1, keepdims=True) + 1e-5)
    np.testing.assert_allclose(z, (sn * P["ffn.ln.gamma"] + P["ffn.ln.beta"]) @ P["proj.w"].T, atol=1e-12)
    z1, _ = nets.forward(small, P, x[2:3])
    np.testing.assert_allclose(z1[0], z[2], atol=1e-12)


def test_transformer_head_step_with_label_smoothing():
    # the translation workload trains with label smoothing 0.1 and alpha = 1: identical peer -> no
    # distillation term, and its gradient vanishes; finite differences of the smoothed loss
    arch = nets.transformer_head(8, 16, 12)
    th = synth.he_init(arch.params, 1, jitter=0.1).astype(np.float64)
    x = synth.images(6, 1, 1, 8, seed=0).astype(np.float64)
    y = synth.labels(6, 12, seed=3)
    same = codistill_step(arch, th, [th.copy()], x, y, 1.0, 0.0, 0.0, label_smoothing=0.1)
    plain = codistill_step(arch, th, [], x, y, 0.0, 0.0, 0.0, label_smoothing=0.1)
    assert same["loss"][2] == 0.0
    np.testing.assert_allclose(same["grad"], plain["grad"], atol=1e-15)
    thp = synth.he_init(arch.params, 2, jitter=0.1).astype(np.float64)
    out = codistill_step(arch, th, [thp], x, y, 1.0, 0.0, 0.0, label_smoothing=0.1)
    loss_at = lambda t: codistill_step(arch, t, [thp], x, y, 1.0, 0.0, 0.0, label_smoothing=0.1)["loss"][0]
    d = np.random.default_rng(1).standard_normal(th.size)
    d /= np.linalg.norm(d)
    h = 1e-5
    assert (loss_at(th + h * d) - loss_at(th - h * d)) / (2 * h) == pytest.approx(float(out["grad"].dot(d)), rel=1e-6)
