"""The allocation-free variant of the loss entry point against the one that takes a caller scratch: same results,
bit for bit (the same kernels), on calls in a row that share the library's device array."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2010_02838_amd import synth

pytestmark = pytest.mark.gpu


def _both(rows, cols, mode, npeers, seed):
    from paper_2010_02838_amd import binding as B
    dev = "cuda:0"
    dk = {"mse": B.CD_DIST_MSE_LOGITS, "kl": B.CD_DIST_KL, "mse_centered": B.CD_DIST_MSE_CENTERED}[mode]
    z = torch.from_numpy(synth.logits(rows, cols, 3.0, seed=seed)).to(dev)
    peers = [torch.from_numpy(synth.logits(rows, cols, 3.0, seed=seed + 100 + j)).to(dev) for j in range(npeers)]
    t = synth.labels(rows, cols, seed=seed + 7)
    t[rows // 3] = -1
    tt = torch.from_numpy(t.astype(np.int32)).to(dev)
    scratch = torch.empty(B.loss_scratch_bytes(rows, cols), dtype=torch.uint8, device=dev)
    l0, l1 = torch.zeros(4, device=dev), torch.full((4,), 7.0, device=dev)
    d0, d1 = torch.empty_like(z), torch.full_like(z, 7.0)
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats(dev)["allocation.all.allocated"]
    B.codistill_loss_grad(z, peers, tt, l0, d0, scratch, 0.5, 0.1, dk)
    B.codistill_loss_grad_static(z, peers, tt, l1, d1, 0.5, 0.1, dk)
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats(dev)["allocation.all.allocated"] == before   # torch's allocator was not asked
    return l0.cpu().numpy(), l1.cpu().numpy(), d0.cpu().numpy(), d1.cpu().numpy(), (z, peers, t)


@pytest.mark.parametrize("mode,npeers", [("mse", 1), ("kl", 1), ("mse_centered", 1), ("kl", 2), ("mse", 0)])
def test_static_scratch_matches_caller_scratch_on_successive_calls(mode, npeers):
    from oracle.loss import codistill_loss_grad as oracle_loss
    # two calls in a row on the same GPU, the second with fewer (and narrower) rows: the array keeps the first
    # call's contents and the second must not see them
    for rows, cols, seed in ((300, 4100 if mode == "kl" and npeers == 2 else 4096, 1), (37, 1000, 2)):
        l0, l1, d0, d1, (z, peers, t) = _both(rows, cols, mode, npeers, seed)
        np.testing.assert_array_equal(l0.view(np.int32), l1.view(np.int32))
        np.testing.assert_array_equal(d0, d1)
        (tot, task, dist), dref = oracle_loss(z.cpu().numpy(), [p.cpu().numpy() for p in peers], t, 0.5, 0.1, mode)
        assert np.linalg.norm(d1 - dref) <= 1e-5 * np.linalg.norm(dref)
        assert abs(l1[0] - tot) <= 1e-5 * abs(tot) and abs(l1[1] - task) <= 1e-5 * abs(task)


def test_static_scratch_row_limit_is_an_error():
    from paper_2010_02838_amd import binding as B
    dev = "cuda:0"
    rows = 65537
    z = torch.zeros(rows, 4, device=dev)
    t = torch.zeros(rows, dtype=torch.int32, device=dev)
    loss, dz = torch.full((4,), 3.0, device=dev), torch.full_like(z, 3.0)
    with pytest.raises(B.CodistillError) as e:
        B.codistill_loss_grad_static(z, [], t, loss, dz, 1.0)
    assert e.value.code == B.CD_ERR_INVALID_ARG and "65536" in str(e.value)
    torch.cuda.synchronize()
    assert float(dz.min()) == 3.0 and float(loss.min()) == 3.0    # nothing was launched
    B.codistill_loss_grad_static(z[:65536], [], t[:65536], loss, dz[:65536], 1.0)   # the limit itself is accepted
    torch.cuda.synchronize()
    assert abs(float(loss[1]) - np.log(4.0)) < 1e-5
