"""ResNet-50 at the benchmarked size (batch 256, 224x224, 1000 classes, bf16) through the C ABI, in the launch
configuration bench.py times (peer forward and weight gradients on second streams).

The float64 oracle cannot hold this batch (about 270 MB per sample), so the step is checked on outputs the
oracle's definitions give one by one from the tensors the kernels consumed (read back from the workspace):
sampled convolution outputs, data gradients and weight gradients as plain float64 sums, BatchNorm statistics
and outputs of sampled channels, the loss on the logits, the update rule, and run-to-run determinism.
These launches have 6272-tile grids, 12544 statistics chunks and split counts that no small case reaches.
"""
import numpy as np
import pytest
import torch

from oracle import nets
from oracle.loss import codistill_loss_grad as oracle_loss
from paper_2010_02838_amd import synth
from gpu_util import Case, rel

pytestmark = pytest.mark.gpu

BF16_STEP = 2.0 ** -8     # one bf16 rounding of the result (2^-9 relative), with a factor two of margin


@pytest.fixture(scope="module")
def full():
    c = Case(dict(kind=2), nets.resnet50(), "bf16", 256, 224, 1000, jitter=0.0)
    got = c.gpu(alpha=1.0, lr=0.1, mu=0.9)
    ops, tensors = c.model.graph(c.batch)
    yield c, got, ops, tensors
    del c.runner
    torch.cuda.empty_cache()


def dev_tensor(c, tensors, t, grad=False):
    """Tensor t of the workspace as a [B,H,W,C] bf16 view on the device (no copy)."""
    d = tensors[t]
    n = c.batch * d["h"] * d["w"] * d["c"]
    off = d["grad_offset"] if grad else d["act_offset"]
    return c.runner.ws[off:off + 2 * n].view(torch.bfloat16).view(c.batch, d["h"], d["w"], d["c"])


def host(x):
    return x.float().cpu().numpy().astype(np.float64)


def conv_ops(ops):
    return [(i, o) for i, o in enumerate(ops) if o["kind"] == "conv"]


def weights(c, ops, o):
    names = [n for n, _, _, _ in c.ref_arch.params]
    return c.per_tensor(c.th.astype(np.float64))[names[o["param_w"]]], names[o["param_w"]]


def test_sampled_convolution_outputs(full):
    c, got, ops, tensors = full
    rng = np.random.default_rng(0)
    xin = torch.from_numpy(c.x).to("cuda:0")    # already rounded to bf16 values
    worst = 0.0
    for i, o in conv_ops(ops):
        w, name = weights(c, ops, o)             # [Cout][kh][kw][Cin]
        x4 = xin if o["x"] == 0 else dev_tensor(c, tensors, o["x"])
        y4 = dev_tensor(c, tensors, o["y"])
        B, Ho, Wo, N = y4.shape
        H, W = x4.shape[1], x4.shape[2]
        k, st, p = o["k"], o["stride"], o["pad"]
        for _ in range(24):
            b, ho, wo, n = (int(rng.integers(0, d)) for d in (B, Ho, Wo, N))
            if rng.random() < 0.3:               # borders and the last rows of the last tile
                b, ho, wo = B - 1, int(rng.choice([0, Ho - 1])), int(rng.choice([0, Wo - 1]))
            h0, w0 = ho * st - p, wo * st - p
            hs, ws = max(h0, 0), max(w0, 0)
            he, we = min(h0 + k, H), min(w0 + k, W)
            patch = host(x4[b, hs:he, ws:we, :])
            terms = patch * w[n, hs - h0:he - h0, ws - w0:we - w0, :]
            ref, rss = terms.sum(), np.sqrt((terms ** 2).sum())
            out = float(y4[b, ho, wo, n].float())
            err = abs(out - ref)
            assert err <= BF16_STEP * abs(ref) + 1e-4 * rss + 1e-30, (i, name, (b, ho, wo, n), out, ref)
            worst = max(worst, err / (abs(ref) + 1e-3 * rss + 1e-30))
    print("sampled conv outputs: worst error relative to |ref| + 1e-3 rss: %.2e" % worst)


def test_sampled_batchnorm_statistics_and_outputs(full):
    c, got, ops, tensors = full
    rng = np.random.default_rng(1)
    names = [n for n, _, _, _ in c.ref_arch.params]
    P = c.per_tensor(c.th.astype(np.float64))
    bns = [(i, o) for i, o in enumerate(ops) if o["kind"] == "bn"]
    for i, o in bns[::3] + bns[-2:]:
        x4 = dev_tensor(c, tensors, o["x"])
        C = x4.shape[3]
        c0 = int(rng.integers(0, C // 8)) * 8
        cols = host(x4[:, :, :, c0:c0 + 8]).reshape(-1, 8)
        mean, var = cols.mean(axis=0), cols.var(axis=0)
        stats = c.read(o["stats_offset"], (4, C), f32=True)
        np.testing.assert_allclose(stats[0, c0:c0 + 8], mean, rtol=1e-4, atol=1e-4 * np.sqrt(var).max())
        np.testing.assert_allclose(stats[1, c0:c0 + 8], 1.0 / np.sqrt(var + 1e-5), rtol=1e-4)
        gamma, beta = P[names[o["param_w"]]], P[names[o["param_b"]]]
        np.testing.assert_allclose(stats[2, c0:c0 + 8], gamma[c0:c0 + 8] * stats[1, c0:c0 + 8], rtol=1e-5)
        np.testing.assert_allclose(stats[3, c0:c0 + 8], beta[c0:c0 + 8] - stats[0, c0:c0 + 8] * stats[2, c0:c0 + 8],
                                   rtol=1e-4, atol=1e-5)
        if o["fused_pool"]:
            # the output tensor is not written; the pooled one is: a sampled window of each sampled channel
            q = ops[i + 1]
            p4 = dev_tensor(c, tensors, q["y"])
            for _ in range(16):
                b, ho, wo = (int(rng.integers(0, d)) for d in p4.shape[:3])
                hs, ws = max(2 * ho - 1, 0), max(2 * wo - 1, 0)
                win = host(x4[b, hs:2 * ho + 2, ws:2 * wo + 2, c0:c0 + 8])
                a = np.maximum(win * stats[2, c0:c0 + 8] + stats[3, c0:c0 + 8], 0.0).max(axis=(0, 1))
                np.testing.assert_allclose(host(p4[b, ho, wo, c0:c0 + 8]), a, rtol=BF16_STEP, atol=1e-6)
            continue
        y4 = dev_tensor(c, tensors, o["y"])
        sl = (slice(None, None, 37), slice(None), slice(None), slice(c0, c0 + 8))
        ref = host(x4[sl]) * stats[2, c0:c0 + 8] + stats[3, c0:c0 + 8]
        if o["res"] >= 0:
            ref = ref + host(dev_tensor(c, tensors, o["res"])[sl])
        if o["relu"]:
            ref = np.maximum(ref, 0.0)
        np.testing.assert_allclose(host(y4[sl]), ref, rtol=BF16_STEP, atol=1e-5)


def test_loss_and_update_rule(full):
    c, got, ops, tensors = full
    (tot, task, dist), dz = oracle_loss(got["logits"].astype(np.float64), [got["peer_logits"].astype(np.float64)],
                                        c.y, 1.0)
    np.testing.assert_allclose(got["loss"], [tot, task, dist], rtol=1e-5)
    assert rel(got["dz"], dz) <= 1e-5
    # from v = 0: v = g, theta = theta - lr v, in fp32 on fp32 master weights
    np.testing.assert_array_equal(got["v"], got["grad"])
    step = np.float32(0.1) * got["grad"]
    assert (np.abs(got["theta"] - (c.th - step)) <= 2e-7 * (np.abs(c.th) + np.abs(step)) + 1e-12).all()
    assert np.isfinite(got["grad"]).all() and np.abs(got["grad"]).max() > 0


def test_sampled_data_and_weight_gradients(full):
    """Convolutions whose input tensor has no other reader (the 3x3 and the last 1x1 of every block): the gradient
    buffer of their input is their data gradient alone."""
    c, got, ops, tensors = full
    rng = np.random.default_rng(2)
    G = c.per_tensor(got["grad"])
    readers = {}
    for o in ops:
        for t in (o["x"], o["res"]):
            if t > 0:
                readers[t] = readers.get(t, 0) + 1
    picked = [(i, o) for i, o in conv_ops(ops) if o["x"] > 0 and readers[o["x"]] == 1]
    assert len(picked) >= 32
    for i, o in picked[::4] + picked[-2:]:
        w, name = weights(c, ops, o)
        k, st, p = o["k"], o["stride"], o["pad"]
        x4 = dev_tensor(c, tensors, o["x"])
        dy4 = dev_tensor(c, tensors, o["y"], grad=True)
        dx4 = dev_tensor(c, tensors, o["x"], grad=True)
        B, H, W, Cin = x4.shape
        Ho, Wo, N = dy4.shape[1:]
        for _ in range(12):                      # dx[b,h,w,ci] = sum over taps and output channels
            b, h, wi, ci = (int(rng.integers(0, d)) for d in (B, H, W, Cin))
            if rng.random() < 0.3:
                b, h, wi = B - 1, int(rng.choice([0, H - 1])), int(rng.choice([0, W - 1]))
            ref, sq = 0.0, 0.0
            for r in range(k):
                for s in range(k):
                    hn, wn = h + p - r, wi + p - s
                    if hn % st or wn % st or not (0 <= hn // st < Ho and 0 <= wn // st < Wo):
                        continue
                    terms = host(dy4[b, hn // st, wn // st, :]) * w[:, r, s, ci]
                    ref += terms.sum()
                    sq += (terms ** 2).sum()
            out = float(dx4[b, h, wi, ci].float())
            assert abs(out - ref) <= BF16_STEP * abs(ref) + 1e-4 * np.sqrt(sq) + 1e-30, (i, name, "dx", out, ref)
        for _ in range(4):                       # dw[n,r,s,ci] = sum over every pixel of the batch
            n, r, s, ci = int(rng.integers(0, N)), int(rng.integers(0, k)), int(rng.integers(0, k)), int(rng.integers(0, Cin))
            ho = np.arange(Ho)
            wo = np.arange(Wo)
            hv = ho[(ho * st - p + r >= 0) & (ho * st - p + r < H)]
            wv = wo[(wo * st - p + s >= 0) & (wo * st - p + s < W)]
            a = host(dy4[:, hv[0]:hv[-1] + 1, wv[0]:wv[-1] + 1, n])
            bsl = x4[:, hv[0] * st - p + r:hv[-1] * st - p + r + 1:st, wv[0] * st - p + s:wv[-1] * st - p + s + 1:st, ci]
            terms = a * host(bsl)
            ref, rss = terms.sum(), np.sqrt((terms ** 2).sum())
            out = float(G[name][n, r, s, ci])
            assert abs(out - ref) <= 1e-3 * abs(ref) + 1e-3 * rss, (i, name, "dw", (n, r, s, ci), out, ref)


def test_run_to_run_determinism(full):
    c, got, ops, tensors = full
    from paper_2010_02838_amd.runner import pack_flat, unpack_flat, to_device
    r = c.runner
    r.load(pack_flat(c.model, c.th), [pack_flat(c.peer, c.thp)])
    xd = to_device(c.x, c.model.torch_dtype)
    yd = torch.from_numpy(c.y).to("cuda:0")
    r.step(xd, yd, 1.0, 0.1, 0.9)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(unpack_flat(c.model, r.grads.cpu().numpy()), got["grad"])
    np.testing.assert_array_equal(r.logits.cpu().numpy(), got["logits"])
    np.testing.assert_array_equal(r.loss.cpu().numpy()[:3].astype(np.float64), got["loss"])


def test_resnext101_grouped_convolutions_sampled():
    """The 101-layer 32x8d aggregated-transformation network at 224x224, batch 32: all 33 grouped convolutions run
    with 2 to 16 slices of 128 channels (8 to 64 channels per group); sampled outputs, data gradients and filter
    gradients as plain float64 sums over the group's channels, from the tensors the kernels consumed."""
    c = Case(dict(kind=6), nets.resnext(), "bf16", 32, 224, 1000, jitter=0.0)
    got = c.gpu(alpha=1.0, lr=0.1, mu=0.9)
    ops, tensors = c.model.graph(c.batch)
    rng = np.random.default_rng(5)
    G = c.per_tensor(got["grad"])
    names = [n for n, _, _, _ in c.ref_arch.params]
    P = c.per_tensor(c.th.astype(np.float64))
    grouped = [(i, o) for i, o in conv_ops(ops) if P[names[o["param_w"]]].shape[3] != tensors[o["x"]]["c"] and o["x"] > 0]
    assert len(grouped) == 33
    for i, o in grouped:
        name = names[o["param_w"]]
        w = P[name]                                    # [C][3][3][cg]
        C, k, _, cg = w.shape
        st, p = o["stride"], o["pad"]
        x4, y4 = dev_tensor(c, tensors, o["x"]), dev_tensor(c, tensors, o["y"])
        dy4, dx4 = dev_tensor(c, tensors, o["y"], grad=True), dev_tensor(c, tensors, o["x"], grad=True)
        B, H, W, _ = x4.shape
        Ho, Wo = y4.shape[1:3]
        for _ in range(6):                             # outputs
            b, ho, wo, n = (int(rng.integers(0, d)) for d in (B, Ho, Wo, C))
            if rng.random() < 0.3:
                b, ho, wo = B - 1, int(rng.choice([0, Ho - 1])), int(rng.choice([0, Wo - 1]))
            c0 = n // cg * cg
            h0, w0 = ho * st - p, wo * st - p
            hs, ws, he, we = max(h0, 0), max(w0, 0), min(h0 + k, H), min(w0 + k, W)
            terms = host(x4[b, hs:he, ws:we, c0:c0 + cg]) * w[n, hs - h0:he - h0, ws - w0:we - w0, :]
            ref, rss = terms.sum(), np.sqrt((terms ** 2).sum())
            out = float(y4[b, ho, wo, n].float())
            assert abs(out - ref) <= BF16_STEP * abs(ref) + 1e-4 * rss + 1e-30, (i, name, "y", out, ref)
        for _ in range(4):                             # data gradients (the input has this one reader)
            b, h, wi, ci = (int(rng.integers(0, d)) for d in (B, H, W, C))
            c0 = ci // cg * cg
            ref, sq = 0.0, 0.0
            for r in range(k):
                for s in range(k):
                    hn, wn = h + p - r, wi + p - s
                    if hn % st or wn % st or not (0 <= hn // st < Ho and 0 <= wn // st < Wo):
                        continue
                    terms = host(dy4[b, hn // st, wn // st, c0:c0 + cg]) * w[c0:c0 + cg, r, s, ci - c0]
                    ref += terms.sum()
                    sq += (terms ** 2).sum()
            out = float(dx4[b, h, wi, ci].float())
            assert abs(out - ref) <= BF16_STEP * abs(ref) + 1e-4 * np.sqrt(sq) + 1e-30, (i, name, "dx", out, ref)
        for _ in range(2):                             # filter gradients: sums over every pixel of the batch
            n, r, s, j = int(rng.integers(0, C)), int(rng.integers(0, k)), int(rng.integers(0, k)), int(rng.integers(0, cg))
            ci = n // cg * cg + j
            ho, wo = np.arange(Ho), np.arange(Wo)
            hv = ho[(ho * st - p + r >= 0) & (ho * st - p + r < H)]
            wv = wo[(wo * st - p + s >= 0) & (wo * st - p + s < W)]
            a = host(dy4[:, hv[0]:hv[-1] + 1, wv[0]:wv[-1] + 1, n])
            bsl = x4[:, hv[0] * st - p + r:hv[-1] * st - p + r + 1:st, wv[0] * st - p + s:wv[-1] * st - p + s + 1:st, ci]
            terms = a * host(bsl)
            ref, rss = terms.sum(), np.sqrt((terms ** 2).sum())
            out = float(G[name][n, r, s, j])
            assert abs(out - ref) <= 1e-3 * abs(ref) + 1e-3 * rss, (i, name, "dw", (n, r, s, j), out, ref)
    del c.runner
    torch.cuda.empty_cache()
