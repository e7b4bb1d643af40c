"""Pins of the oracle's Adam update: closed forms and torch's own optimiser."""
import numpy as np
import torch

from oracle.adam import adam_step


def test_constant_gradient_closed_form():
    # the bias-corrected averages of a constant are that constant: every step moves w by lr * g / (|g| + eps)
    rng = np.random.default_rng(0)
    w0, g = rng.standard_normal(40), rng.standard_normal(40) * 3
    g[:4] = 0.0                                      # no gradient, no movement
    w, m, v = w0, np.zeros(40), np.zeros(40)
    lr, eps = 0.01, 1e-8
    for t in range(1, 6):
        w, m, v = adam_step(w, m, v, g, lr, t, eps=eps)
        np.testing.assert_allclose(w, w0 - t * lr * g / (np.abs(g) + eps), rtol=1e-12, atol=1e-15)
    np.testing.assert_array_equal(w[:4], w0[:4])
    # first step from zero state: m = (1 - beta1) g, v = (1 - beta2) g^2
    _, m1, v1 = adam_step(w0, np.zeros(40), np.zeros(40), g, lr, 1, beta1=0.9, beta2=0.98)
    np.testing.assert_allclose(m1, 0.1 * g, rtol=1e-12)
    np.testing.assert_allclose(v1, 0.02 * g * g, rtol=1e-12)


def test_against_torch_adam():
    rng = np.random.default_rng(1)
    w0 = rng.standard_normal(64)
    for wd in (0.0, 0.05):
        p = torch.nn.Parameter(torch.tensor(w0))
        opt = torch.optim.Adam([p], lr=3e-3, betas=(0.9, 0.98), eps=1e-8, weight_decay=wd)
        w, m, v = w0, np.zeros(64), np.zeros(64)
        for t in range(1, 8):
            g = rng.standard_normal(64) * (1.0 + t)
            p.grad = torch.tensor(g)
            opt.step()
            w, m, v = adam_step(w, m, v, g, 3e-3, t, weight_decay=wd)
            np.testing.assert_allclose(w, p.detach().numpy(), rtol=1e-12, atol=1e-14)


def test_inputs_are_not_modified_and_sign_of_the_step():
    w0, g = np.ones(5), np.array([1.0, -2.0, 0.5, -0.1, 3.0])
    m0, v0 = np.zeros(5), np.zeros(5)
    w, m, v = adam_step(w0, m0, v0, g, 0.1, 1)
    assert (w0 == 1).all() and (m0 == 0).all() and (v0 == 0).all()
    assert (np.sign(w0 - w) == np.sign(g)).all()
