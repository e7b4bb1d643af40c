"""Pins for the oracle's loss: closed forms, invariants and library special cases.

None of these retype the oracle's formula; each is a value fixed by the
mathematics (or a library routine) that a dropped term, wrong sign, wrong
normaliser or transposed operand would break.
"""
import math

import numpy as np
import pytest
import scipy.special
import torch

from oracle.loss import codistill_loss_grad, log_softmax


def rnd(rows, cols, seed, sigma=2.0):
    return np.random.default_rng(seed).standard_normal((rows, cols)) * sigma


@pytest.mark.parametrize("cols", [10, 1000, 32768])
@pytest.mark.parametrize("eps", [0.0, 0.1])
def test_ce_zero_logits_is_log_c(cols, eps):
    rows = 4
    z = np.zeros((rows, cols))
    t = np.arange(rows) % cols
    (tot, task, dist), dz = codistill_loss_grad(z, None, t, alpha=1.0, label_smoothing=eps)
    assert task == pytest.approx(math.log(cols), rel=1e-14)
    assert tot == task and dist == 0.0
    # gradient rows are (1/C - q)/N
    q = np.full((rows, cols), eps / cols)
    q[np.arange(rows), t] += 1 - eps
    np.testing.assert_allclose(dz, (1.0 / cols - q) / rows, rtol=0, atol=1e-16)


def test_ce_printed_constants():
    # ln 10, ln 1000, 15 ln 2: values fixed by the class counts of the workloads
    for cols, val in [(10, 2.302585092994046), (1000, 6.907755278982137), (32768, 10.397207708399179)]:
        (_, task, _), _ = codistill_loss_grad(np.zeros((2, cols)), None, [0, 1], 0.0)
        assert abs(task - val) < 1e-13


def test_ce_shift_invariance_and_row_sums():
    z = rnd(6, 17, 0)
    t = np.array([0, 3, 16, 5, 5, 2])
    (a, _, _), dza = codistill_loss_grad(z, None, t, 0.0, label_smoothing=0.05)
    (b, _, _), dzb = codistill_loss_grad(z + np.arange(6)[:, None] * 3.7, None, t, 0.0, label_smoothing=0.05)
    assert a == pytest.approx(b, rel=1e-13)
    np.testing.assert_allclose(dza, dzb, atol=1e-15)
    np.testing.assert_allclose(dza.sum(axis=1), 0, atol=1e-15)


def test_ce_matches_torch_cross_entropy():
    z = rnd(9, 33, 1)
    t = np.random.default_rng(2).integers(0, 33, 9)
    t[4] = -1
    for eps in (0.0, 0.1):
        zt = torch.tensor(z, requires_grad=True)
        l = torch.nn.functional.cross_entropy(zt, torch.tensor(t), ignore_index=-1, label_smoothing=eps)
        l.backward()
        (_, task, _), dz = codistill_loss_grad(z, None, t, 0.0, label_smoothing=eps)
        # torch's smoothed loss with ignore_index normalises the same way only for eps=0;
        # check eps>0 on the rows-all-valid case below
        if eps == 0.0:
            assert task == pytest.approx(l.item(), rel=1e-13)
            np.testing.assert_allclose(dz, zt.grad.numpy(), atol=1e-15)
    t2 = np.where(t < 0, 0, t)
    zt = torch.tensor(z, requires_grad=True)
    l = torch.nn.functional.cross_entropy(zt, torch.tensor(t2), label_smoothing=0.1)
    l.backward()
    (_, task, _), dz = codistill_loss_grad(z, None, t2, 0.0, label_smoothing=0.1)
    assert task == pytest.approx(l.item(), rel=1e-13)
    np.testing.assert_allclose(dz, zt.grad.numpy(), atol=1e-15)


@pytest.mark.parametrize("dist", ["mse", "kl"])
def test_identical_peer_gives_zero_distillation(dist):
    z = rnd(5, 12, 3)
    t = np.array([1, 2, 3, 4, 5])
    (tot, task, d), dz = codistill_loss_grad(z, [z.copy()], t, alpha=0.7, dist=dist)
    (_, task0, _), dz0 = codistill_loss_grad(z, None, t, alpha=0.7)
    assert d == 0.0 and tot == task == task0
    np.testing.assert_array_equal(dz, dz0)


@pytest.mark.parametrize("dist", ["mse", "kl"])
def test_alpha_zero_is_plain_cross_entropy(dist):
    z, zp = rnd(5, 12, 4), rnd(5, 12, 5)
    t = np.array([1, 2, 3, 4, 5])
    (tot, task, _), dz = codistill_loss_grad(z, [zp], t, alpha=0.0, dist=dist)
    (_, task0, _), dz0 = codistill_loss_grad(z, None, t, alpha=1.0)
    assert tot == task == task0
    np.testing.assert_array_equal(dz, dz0)


def test_mse_constant_offset_closed_form():
    # z' = z + c  =>  D = c^2 (mean over all elements), C c^2 (mean over rows); the
    # gradient is NOT shift invariant: row sums are 2 alpha (-c) C /(N C) = -2 alpha c / N
    z = rnd(7, 11, 6)
    t = np.zeros(7, dtype=int)
    c, alpha = 0.3, 0.5
    (_, _, d), dz = codistill_loss_grad(z, [z + c], t, alpha, dist="mse")
    assert d == pytest.approx(c * c, rel=1e-12)
    (_, _, _), dz0 = codistill_loss_grad(z, None, t, alpha)
    np.testing.assert_allclose((dz - dz0).sum(axis=1), -2 * alpha * c / 7, rtol=1e-12)
    (_, _, dr), dzr = codistill_loss_grad(z, [z + c], t, alpha, dist="mse", mse_reduction="mean_rows")
    assert dr == pytest.approx(11 * c * c, rel=1e-12)
    np.testing.assert_allclose(dzr - dz0, 11 * (dz - dz0), rtol=1e-12)


def test_mse_matches_torch_mse_loss_and_expectation():
    z, zp = rnd(64, 50, 7, 3.0), rnd(64, 50, 8, 3.0)
    t = np.random.default_rng(9).integers(0, 50, 64)
    alpha = 0.5
    zt = torch.tensor(z, requires_grad=True)
    l = torch.nn.functional.cross_entropy(zt, torch.tensor(t)) + alpha * torch.nn.functional.mse_loss(zt, torch.tensor(zp))
    l.backward()
    (tot, _, d), dz = codistill_loss_grad(z, [zp], t, alpha, dist="mse")
    assert tot == pytest.approx(l.item(), rel=1e-13)
    np.testing.assert_allclose(dz, zt.grad.numpy(), atol=1e-15)
    # independent N(0, sigma^2) logits: E[D] = 2 sigma^2 = 18
    assert abs(d - 18.0) < 6 * 18.0 * math.sqrt(2.0 / (64 * 50))


def test_kl_library_special_cases():
    z, zp = rnd(8, 21, 10), rnd(8, 21, 11)
    t = np.arange(8)
    (tot, task, d), dz = codistill_loss_grad(z, [zp], t, 1.0, dist="kl")
    p, pp = np.exp(log_softmax(z)), np.exp(log_softmax(zp))
    assert d == pytest.approx(scipy.special.rel_entr(pp, p).sum() / 8, rel=1e-12)
    zt = torch.tensor(z, requires_grad=True)
    kl = torch.nn.functional.kl_div(torch.log_softmax(zt, 1), torch.softmax(torch.tensor(zp), 1), reduction="batchmean")
    (torch.nn.functional.cross_entropy(zt, torch.tensor(t)) + kl).backward()
    assert d == pytest.approx(kl.item(), rel=1e-12)
    np.testing.assert_allclose(dz, zt.grad.numpy(), atol=1e-15)
    assert d >= 0
    np.testing.assert_allclose(dz.sum(axis=1), 0, atol=1e-15)
    # invariant to constant shifts of either operand
    (_, _, d2), dz2 = codistill_loss_grad(z + 5.0, [zp - 3.0], t, 1.0, dist="kl")
    assert d2 == pytest.approx(d, rel=1e-12)
    np.testing.assert_allclose(dz2, dz, atol=1e-15)


def test_kl_temperature_against_torch_and_its_high_temperature_limit():
    z, zp = rnd(6, 17, 12), rnd(6, 17, 13)
    t = np.arange(6)
    for tau in (0.5, 1.0, 3.0):
        (tot, task, d), dz = codistill_loss_grad(z, [zp], t, 0.7, dist="kl", temperature=tau)
        zt = torch.tensor(z, requires_grad=True)
        kl = tau * tau * torch.nn.functional.kl_div(torch.log_softmax(zt / tau, 1), torch.softmax(torch.tensor(zp) / tau, 1),
                                                    reduction="batchmean")
        ce = torch.nn.functional.cross_entropy(zt, torch.tensor(t))
        (ce + 0.7 * kl).backward()
        assert d == pytest.approx(kl.item(), rel=1e-12)
        assert task == pytest.approx(ce.item(), rel=1e-12)       # the supervised term keeps temperature 1
        np.testing.assert_allclose(dz, zt.grad.numpy(), atol=1e-15)
    # tau = 1 is the default
    assert codistill_loss_grad(z, [zp], t, 0.7, dist="kl")[0] == codistill_loss_grad(z, [zp], t, 0.7, dist="kl", temperature=1.0)[0]
    # tau -> infinity: tau^2 KL tends to half the squared distance of the centred logit rows, per class
    delta = zp - z
    delta = delta - delta.mean(axis=1, keepdims=True)
    limit = (delta ** 2).sum() / (2 * 17) / 6
    (_, _, dbig), _ = codistill_loss_grad(z, [zp], t, 1.0, dist="kl", temperature=1e4)
    assert dbig == pytest.approx(limit, rel=2e-3)


def test_centered_mse_invariances_and_reduction_to_plain_mse():
    z, zp = rnd(9, 13, 30), rnd(9, 13, 31)
    t = np.random.default_rng(32).integers(0, 13, 9)
    alpha = 0.7
    (_, _, d), dz = codistill_loss_grad(z, [zp], t, alpha, dist="mse_centered")
    (_, _, _), dz0 = codistill_loss_grad(z, None, t, alpha)
    # a per-row constant added to either model's logits changes nothing
    shift = np.random.default_rng(33).standard_normal((9, 1)) * 4
    (_, _, d2), dz2 = codistill_loss_grad(z, [zp + shift], t, alpha, dist="mse_centered")
    assert d2 == pytest.approx(d, rel=1e-12)
    np.testing.assert_allclose(dz2, dz, atol=1e-15)
    # so a peer that differs by a constant per row is at distance zero, with the plain CE gradient
    (_, _, d3), dz3 = codistill_loss_grad(z, [z + shift], t, alpha, dist="mse_centered")
    assert abs(d3) < 1e-28
    np.testing.assert_allclose(dz3, dz0, atol=1e-15)
    # the distillation part of the gradient sums to zero over the classes of each row
    np.testing.assert_allclose((dz - dz0).sum(axis=1), 0, atol=1e-15)
    # rows that already have zero mean: identical to the uncentred term
    zc, zpc = z - z.mean(axis=1, keepdims=True), zp - zp.mean(axis=1, keepdims=True)
    a, dza = codistill_loss_grad(zc, [zpc], t, alpha, dist="mse_centered")
    b, dzb = codistill_loss_grad(zc, [zpc], t, alpha, dist="mse")
    np.testing.assert_allclose(a, b, rtol=1e-13)
    np.testing.assert_allclose(dza, dzb, atol=1e-15)
    # variance decomposition: uncentred = centred + squared difference of the row means
    (_, _, du), _ = codistill_loss_grad(z, [zp], t, alpha, dist="mse")
    gap = ((z.mean(axis=1) - zp.mean(axis=1)) ** 2).mean()
    assert du == pytest.approx(d + gap, rel=1e-12)
    # torch: mse_loss of the centred tensors, differentiated through the centring
    zt = torch.tensor(z, requires_grad=True)
    zpt = torch.tensor(zp)
    l = torch.nn.functional.cross_entropy(zt, torch.tensor(t)) + alpha * torch.nn.functional.mse_loss(
        zt - zt.mean(1, keepdim=True), zpt - zpt.mean(1, keepdim=True))
    l.backward()
    (tot, _, _), _ = codistill_loss_grad(z, [zp], t, alpha, dist="mse_centered")
    assert tot == pytest.approx(l.item(), rel=1e-13)
    np.testing.assert_allclose(dz, zt.grad.numpy(), atol=1e-15)
    # mean over rows instead of over all elements: C times larger
    (_, _, dr), dzr = codistill_loss_grad(z, [zp], t, alpha, dist="mse_centered", mse_reduction="mean_rows")
    assert dr == pytest.approx(13 * d, rel=1e-12)
    np.testing.assert_allclose(dzr - dz0, 13 * (dz - dz0), rtol=1e-11, atol=1e-16)


@pytest.mark.parametrize("dist", ["mse", "kl", "mse_centered"])
def test_n_way_average(dist):
    # Algorithm 1 averages D over the n-1 peers: two identical peers == one peer
    z, zp, zq = rnd(4, 9, 12), rnd(4, 9, 13), rnd(4, 9, 14)
    t = np.array([0, 1, 2, 3])
    one, dz1 = codistill_loss_grad(z, [zp], t, 0.8, dist=dist)
    two, dz2 = codistill_loss_grad(z, [zp, zp], t, 0.8, dist=dist)
    np.testing.assert_allclose(one, two, rtol=1e-14)
    np.testing.assert_allclose(dz1, dz2, atol=1e-16)
    # and two different peers give the mean of the two single-peer terms
    a, _ = codistill_loss_grad(z, [zp], t, 0.8, dist=dist)
    b, _ = codistill_loss_grad(z, [zq], t, 0.8, dist=dist)
    c, _ = codistill_loss_grad(z, [zp, zq], t, 0.8, dist=dist)
    assert c[2] == pytest.approx(0.5 * (a[2] + b[2]), rel=1e-13)


@pytest.mark.parametrize("dist", ["mse", "kl", "mse_centered"])
def test_ignored_rows(dist):
    z, zp = rnd(6, 8, 15), rnd(6, 8, 16)
    t = np.array([1, -1, 3, -1, 0, 7])
    full, dz = codistill_loss_grad(z, [zp], t, 0.6, label_smoothing=0.1, dist=dist)
    keep = t != -1
    sub, dzs = codistill_loss_grad(z[keep], [zp[keep]], t[keep], 0.6, label_smoothing=0.1, dist=dist)
    np.testing.assert_allclose(full, sub, rtol=1e-14)
    np.testing.assert_allclose(dz[keep], dzs, atol=1e-16)
    assert np.all(dz[~keep] == 0)
    out, dz0 = codistill_loss_grad(z, [zp], np.full(6, -1), 0.6, dist=dist)
    assert out == (0.0, 0.0, 0.0) and np.all(dz0 == 0)


@pytest.mark.parametrize("dist,red", [("mse", "mean_all"), ("mse", "mean_rows"), ("kl", "mean_all"),
                                      ("mse_centered", "mean_all"), ("mse_centered", "mean_rows")])
def test_gradient_by_finite_differences(dist, red):
    z, zp = rnd(3, 5, 17, 1.0), rnd(3, 5, 18, 1.0)
    t = np.array([4, -1, 2])
    kw = dict(alpha=0.9, label_smoothing=0.1, dist=dist, mse_reduction=red)
    _, dz = codistill_loss_grad(z, [zp], t, **kw)
    h = 1e-6
    for i in range(3):
        for j in range(5):
            zp_, zm_ = z.copy(), z.copy()
            zp_[i, j] += h
            zm_[i, j] -= h
            fd = (codistill_loss_grad(zp_, [zp], t, **kw)[0][0] - codistill_loss_grad(zm_, [zp], t, **kw)[0][0]) / (2 * h)
            assert abs(fd - dz[i, j]) < 1e-8
