"""ResNet-50 at the benchmarked size (batch 256, 224x224, 1000 classes, bf16) through the C ABI, in the launch
configuration bench.py times (peer forward and weight gradients on second streams).

The float64 oracle cannot hold this batch (about 270 MB per sample), so every check applies the oracle's layer
functions (oracle.layers) to slices of the tensors the kernels consumed (read back from the workspace), chosen so
that the slice is a complete problem of its own:

  * a convolution output block needs only its receptive field: conv2d_forward on the cropped window (cut with
    explicit zeros where it leaves the image, padding 0);
  * a block of data gradients needs only the gradients of the outputs that touch it: conv2d_backward on that window;
  * a filter gradient is a sum over every pixel of the batch but separates over channels: conv2d_backward on an
    8-channel slice of x, an 8-channel slice of dy and the matching 8 x 8 block of the filter, whole batch;
  * BatchNorm is independent per channel: batchnorm_forward / batchnorm_backward on 8-channel slices over the
    whole batch (statistics, outputs, d gamma, d beta, dx; with the fused max-pool: maxpool_forward / _backward);
  * tensors with several readers: the readers' contributions, each from the oracle, are summed;
  * global average pool and the dense layer run whole.

These launches have 6272-tile grids, 12544 statistics chunks and split counts that no small case reaches.
"""
import numpy as np
import pytest
import torch

from oracle import layers as L
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


TOL_BF16_TENSOR = 5e-3   # a block the kernel rounds to bf16 (2^-9 relative per element, twice if accumulated), L2
TOL_F32_TENSOR = 1e-3    # fp32 results of fp32 accumulation over up to 3.2e6 bf16 products, L2
R = 6                    # side of a sampled block of pixels


def window(c, x4, b, r0, r1, q0, q1):
    """Rows r0..r1-1 and columns q0..q1-1 of sample b as float64 [1, r1-r0, q1-q0, C]; zeros outside the image."""
    H, W, C = x4.shape[1:]
    out = np.zeros((1, r1 - r0, q1 - q0, C))
    rs, re, qs, qe = max(r0, 0), min(r1, H), max(q0, 0), min(q1, W)
    if rs < re and qs < qe:
        out[0, rs - r0:re - r0, qs - q0:qe - q0, :] = host(x4[b, rs:re, qs:qe, :])
    return out


def blocks(rng, B, H, W, n):
    """n sampled R x R blocks (sample, first row, first column): random ones, the four corners, the last rows of
    the last sample (the ragged end of the last tile)."""
    r = min(R, H)
    out = [(int(rng.integers(0, B)), int(rng.integers(0, H - r + 1)), int(rng.integers(0, W - r + 1))) for _ in range(n)]
    out += [(B - 1, H - r, W - r), (0, 0, 0), (B - 1, 0, W - r), (int(rng.integers(0, B)), H - r, 0)]
    return out, r


def conv_dx_block(c, o, w, x4, dy4, b, h0, w0, r):
    """The oracle's data gradient of convolution o on input pixels [h0, h0+r) x [w0, w0+r) of sample b, from the
    gradients of the outputs that touch them."""
    k, st, p = o["k"], o["stride"], o["pad"]
    Ho, Wo = dy4.shape[1:3]
    lo = lambda a: max(0, -((-(a + p - k + 1)) // st))          # first output row / column that reaches a
    hi = lambda a, n: min(n - 1, (a + p) // st)                  # last one
    ho0, ho1, wo0, wo1 = lo(h0), hi(h0 + r - 1, Ho), lo(w0), hi(w0 + r - 1, Wo)
    out = np.zeros((r, r, x4.shape[3]))
    if ho0 > ho1 or wo0 > wo1:
        return out
    dyb = host(dy4[b:b + 1, ho0:ho1 + 1, wo0:wo1 + 1, :])
    a0, q0 = ho0 * st - p, wo0 * st - p                          # origin of the outputs' receptive field
    a1, q1 = ho1 * st - p + k, wo1 * st - p + k
    xw = window(c, x4, b, a0, a1, q0, q1)
    dxw = L.conv2d_backward(xw, w, dyb, st, 0, False, True)[0][0]
    rs, re, qs, qe = max(a0, h0), min(a1, h0 + r), max(q0, w0), min(q1, w0 + r)
    out[rs - h0:re - h0, qs - w0:qe - w0, :] = dxw[rs - a0:re - a0, qs - q0:qe - q0, :]
    return out


def readers_of(ops):
    rd = {}
    for j, o in enumerate(ops):
        for t in {o["x"], o["res"]}:
            if t > 0:
                rd.setdefault(t, []).append(j)
    return rd


def test_convolution_output_blocks(full):
    """Every one of the 53 convolutions: sampled 6 x 6 blocks of output pixels, all output channels."""
    c, got, ops, tensors = full
    rng = np.random.default_rng(0)
    xin = torch.from_numpy(c.x).to("cuda:0")    # already rounded to bf16 values
    worst = 0.0
    for i, o in conv_ops(ops):
        w, name = weights(c, ops, o)             # [Cout][kh][kw][Cin]
        x4 = xin if o["x"] == 0 else dev_tensor(c, tensors, o["x"])
        y4 = dev_tensor(c, tensors, o["y"])
        B, Ho, Wo, N = y4.shape
        k, st, p = o["k"], o["stride"], o["pad"]
        picks, r = blocks(rng, B, Ho, Wo, 3)
        for b, ho, wo in picks:
            xw = window(c, x4, b, ho * st - p, (ho + r - 1) * st - p + k, wo * st - p, (wo + r - 1) * st - p + k)
            ref = L.conv2d_forward(xw, w, None, st, 0)[0]
            assert ref.shape == (r, r, N)
            out = host(y4[b, ho:ho + r, wo:wo + r, :])
            e = rel(out, ref)
            worst = max(worst, e)
            assert e <= TOL_BF16_TENSOR, (i, name, (b, ho, wo), e)
            # element by element: one bf16 rounding of the result plus fp32 accumulation noise
            assert (np.abs(out - ref) <= BF16_STEP * np.abs(ref) + 1e-3 * np.sqrt((ref ** 2).mean())).all(), (i, name)
    print("convolution output blocks: worst relative L2 error %.2e" % worst)


def test_filter_gradients_channel_blocks(full):
    """Filter gradients are sums over every pixel of the batch: an 8 x 8 channel block of every fourth
    convolution (the stem and the last one included), whole batch, all taps."""
    c, got, ops, tensors = full
    rng = np.random.default_rng(2)
    G = c.per_tensor(got["grad"])
    xin = torch.from_numpy(c.x).to("cuda:0")
    convs = conv_ops(ops)
    worst = 0.0
    for i, o in convs[::4] + convs[-1:]:
        w, name = weights(c, ops, o)
        x4 = xin if o["x"] == 0 else dev_tensor(c, tensors, o["x"])
        dy4 = dev_tensor(c, tensors, o["y"], grad=True)
        N, Cin = w.shape[0], w.shape[3]
        n0 = int(rng.integers(0, N // 8)) * 8
        c0, cw = (0, Cin) if Cin < 8 else (int(rng.integers(0, Cin // 8)) * 8, 8)
        _, dw, _ = L.conv2d_backward(host(x4[..., c0:c0 + cw]), w[n0:n0 + 8, :, :, c0:c0 + cw], host(dy4[..., n0:n0 + 8]),
                                     o["stride"], o["pad"], False, need_dx=False)
        e = rel(G[name][n0:n0 + 8, :, :, c0:c0 + cw], dw)
        worst = max(worst, e)
        assert e <= TOL_F32_TENSOR, (i, name, e)
    print("filter gradient blocks: worst relative L2 error %.2e" % worst)


def bn_dy_slice(c, ops, tensors, o, sl):
    """Gradient of the output of BatchNorm op o on channel slice sl, before the op's own ReLU: from the output's
    gradient buffer, or (a shortcut's BatchNorm whose reader hands its gradient on unwritten, res_grad 1) from
    the reading BatchNorm's output gradient gated by that op's ReLU."""
    for q in ops:
        if q["kind"] == "bn" and q["res"] == o["y"] and q["res_grad"] == 1:
            g = host(dev_tensor(c, tensors, q["y"], grad=True)[..., sl])
            return L.relu_backward(host(dev_tensor(c, tensors, q["y"])[..., sl]), g) if q["relu"] else g
    return host(dev_tensor(c, tensors, o["y"], grad=True)[..., sl])


def test_batchnorm_forward_and_backward_channel_slices(full):
    """Every third BatchNorm, the fused BatchNorm + max-pool of the stem and the last two: statistics, scale and
    shift, outputs, and the backward pass (d gamma, d beta, dx), on 8 channels over the whole batch."""
    c, got, ops, tensors = full
    rng = np.random.default_rng(1)
    names = [n for n, _, _, _ in c.ref_arch.params]
    P = c.per_tensor(c.th.astype(np.float64))
    G = c.per_tensor(got["grad"])
    bns = [(i, o) for i, o in enumerate(ops) if o["kind"] == "bn"]
    picked = {i: o for i, o in bns[::3] + bns[-2:] + [(i, o) for i, o in bns if o["fused_pool"]]}
    assert any(o["fused_pool"] for o in picked.values()) and any(o["res"] >= 0 for o in picked.values())
    worst = {"y": 0.0, "dx": 0.0, "dgamma": 0.0}
    for i, o in sorted(picked.items()):
        x4 = dev_tensor(c, tensors, o["x"])
        C = x4.shape[3]
        c0 = int(rng.integers(0, C // 8)) * 8
        sl = slice(c0, c0 + 8)
        gname, bname = names[o["param_w"]], names[o["param_b"]]
        gamma, beta = P[gname][sl], P[bname][sl]
        yr, cache = L.batchnorm_forward(host(x4[..., sl]), gamma, beta)
        _, invstd, mean, var = cache
        stats = c.read(o["stats_offset"], (4, C), f32=True)[:, sl]
        np.testing.assert_allclose(stats[0], mean, rtol=1e-4, atol=1e-4 * np.sqrt(var).max())
        np.testing.assert_allclose(stats[1], invstd, rtol=1e-4)
        np.testing.assert_allclose(stats[2], gamma * invstd, rtol=1e-4)
        np.testing.assert_allclose(stats[3], beta - mean * gamma * invstd, rtol=1e-4, atol=1e-5)
        if o["res"] >= 0:
            yr = yr + host(dev_tensor(c, tensors, o["res"])[..., sl])
        if o["relu"]:
            yr = L.relu_forward(yr)
        if o["fused_pool"]:
            # neither the output nor its gradient is written: the pooled tensor, and the pooled gradient, are
            q = ops[i + 1]
            pooled, arg = L.maxpool_forward(yr, q["k"], q["stride"], q["pad"])
            e = rel(host(dev_tensor(c, tensors, q["y"])[..., sl]), pooled)
            dy = L.maxpool_backward(yr.shape, arg, host(dev_tensor(c, tensors, q["y"], grad=True)[..., sl]),
                                    q["k"], q["stride"], q["pad"])
        else:
            e = rel(host(dev_tensor(c, tensors, o["y"])[..., sl]), yr)
            dy = bn_dy_slice(c, ops, tensors, o, sl)
        worst["y"] = max(worst["y"], e)
        assert e <= TOL_BF16_TENSOR, (i, gname, "y", e)
        if o["relu"]:
            dy = L.relu_backward(yr, dy)
        dx, dg, db = L.batchnorm_backward(dy, gamma, cache)
        eg, eb = rel(G[gname][sl], dg), rel(G[bname][sl], db)
        worst["dgamma"] = max(worst["dgamma"], eg, eb)
        assert eg <= TOL_F32_TENSOR and eb <= TOL_F32_TENSOR, (i, gname, eg, eb)
        e = rel(host(dev_tensor(c, tensors, o["x"], grad=True)[..., sl]), dx)     # a convolution output: this op is its one reader
        worst["dx"] = max(worst["dx"], e)
        assert e <= TOL_BF16_TENSOR, (i, gname, "dx", e)
    print("BatchNorm channel slices (%d ops), worst relative L2 errors: %s" % (len(picked), worst))


def test_activation_gradient_blocks(full):
    """Gradients of the tensors that convolutions read (block inputs and outputs, the tensors inside a block): sampled
    6 x 6 blocks, all channels.  A tensor with several readers (a block's input: its first convolution and the
    shortcut, a projection or the identity) gets the sum of the readers' contributions, each from the oracle."""
    c, got, ops, tensors = full
    rng = np.random.default_rng(3)
    rd = readers_of(ops)
    handed_on = {o["res"] for o in ops if o["kind"] == "bn" and o["res"] >= 0 and o["res_grad"] == 1}
    unwritten = {o["y"] for o in ops if o["kind"] == "bn" and o["fused_pool"]}
    targets = [t for t in sorted(rd) if t not in handed_on and t not in unwritten
               and all(ops[j]["kind"] in ("conv", "bn") for j in rd[t]) and any(ops[j]["kind"] == "conv" for j in rd[t])]
    multi = [t for t in targets if len(rd[t]) > 1]
    assert len(multi) >= 16 and len(targets) >= 48
    worst = {1: 0.0, 2: 0.0}
    for t in multi[::2] + [t for t in targets if len(rd[t]) == 1][::4]:
        x4, dx4 = dev_tensor(c, tensors, t), dev_tensor(c, tensors, t, grad=True)
        B, H, W, C = x4.shape
        picks, r = blocks(rng, B, H, W, 2)
        for b, h0, w0 in picks:
            ref = np.zeros((r, r, C))
            for j in rd[t]:
                o = ops[j]
                if o["kind"] == "conv":
                    w, _ = weights(c, ops, o)
                    ref += conv_dx_block(c, o, w, x4, dev_tensor(c, tensors, o["y"], grad=True), b, h0, w0, r)
                else:   # the residual input of a BatchNorm: that op's output gradient behind its ReLU
                    assert o["res"] == t and o["x"] != t
                    g = host(dev_tensor(c, tensors, o["y"], grad=True)[b, h0:h0 + r, w0:w0 + r, :])
                    ref += L.relu_backward(host(dev_tensor(c, tensors, o["y"])[b, h0:h0 + r, w0:w0 + r, :]), g) if o["relu"] else g
            e = rel(host(dx4[b, h0:h0 + r, w0:w0 + r, :]), ref)
            n = min(len(rd[t]), 2)
            worst[n] = max(worst[n], e)
            # n contributions are added one after the other into the stored bf16 gradient, each addition rounding the sum
            assert e <= TOL_BF16_TENSOR * max(1.0, np.sqrt((len(rd[t]) + 1) / 3.0)), (t, (b, h0, w0), e)
    print("activation gradient blocks, worst relative L2 error by number of readers: %s" % worst)


def test_pool_and_dense_layer_whole(full):
    """Global average pool and the dense layer at full size: forward, and the gradients of the weight matrix, the
    bias and both inputs."""
    c, got, ops, tensors = full
    names = [n for n, _, _, _ in c.ref_arch.params]
    P = c.per_tensor(c.th.astype(np.float64))
    G = c.per_tensor(got["grad"])
    gap, lin = ops[-2], ops[-1]
    assert gap["kind"] == "gap" and lin["kind"] == "linear"
    x = host(dev_tensor(c, tensors, gap["x"]))
    pooled = host(dev_tensor(c, tensors, gap["y"])).reshape(c.batch, -1)
    assert rel(pooled, L.gap_forward(x)) <= TOL_BF16_TENSOR
    w, b = P[names[lin["param_w"]]], P[names[lin["param_b"]]]
    assert rel(got["logits"], L.linear_forward(pooled, w, b)) <= 1e-4
    dx, dw, db = L.linear_backward(pooled, w, got["dz"].astype(np.float64), True)
    assert rel(G[names[lin["param_w"]]], dw) <= TOL_BF16_TENSOR      # from a bf16 copy of d loss / d logits, on the MFMA kernels
    assert rel(G[names[lin["param_b"]]], db) <= TOL_F32_TENSOR
    dpooled = host(dev_tensor(c, tensors, gap["y"], grad=True)).reshape(c.batch, -1)
    assert rel(dpooled, dx) <= TOL_BF16_TENSOR
    assert rel(host(dev_tensor(c, tensors, gap["x"], grad=True)), L.gap_backward(x.shape, dpooled)) <= TOL_BF16_TENSOR


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
