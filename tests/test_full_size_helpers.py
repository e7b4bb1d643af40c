"""The cropping logic of the full-size GPU test, checked on the CPU: a block computed from a cropped window with
the oracle's layer functions equals the same block of the oracle's whole-tensor result."""
import numpy as np
import pytest
import torch

from oracle import layers as L
from test_gpu_full_size import blocks, conv_dx_block, window


@pytest.mark.parametrize("k,st,p", [(1, 1, 0), (1, 2, 0), (3, 1, 1), (3, 2, 1), (7, 2, 3)])
def test_cropped_blocks_match_whole_tensor(k, st, p):
    rng = np.random.default_rng(k * 10 + st)
    B, H, W, C, N = 2, 17, 14, 5, 4
    x = rng.standard_normal((B, H, W, C))
    w = rng.standard_normal((N, k, k, C))
    y = L.conv2d_forward(x, w, None, st, p)
    dy = rng.standard_normal(y.shape)
    dx = L.conv2d_backward(x, w, dy, st, p, False, True)[0]
    x4, dy4 = torch.from_numpy(x), torch.from_numpy(dy)     # stand-ins for the device views
    o = dict(k=k, stride=st, pad=p)
    Ho, Wo = y.shape[1:3]
    picks, r = blocks(rng, B, Ho, Wo, 3)
    for b, ho, wo in picks:
        xw = window(None, x4, b, ho * st - p, (ho + r - 1) * st - p + k, wo * st - p, (wo + r - 1) * st - p + k)
        ref = L.conv2d_forward(xw, w, None, st, 0)[0]
        np.testing.assert_allclose(ref, y[b, ho:ho + r, wo:wo + r, :], rtol=1e-5, atol=1e-5)    # float32 round trip of x
    picks, r = blocks(rng, B, H, W, 4)
    for b, h0, w0 in picks:
        got = conv_dx_block(None, o, w, x4, dy4, b, h0, w0, r)
        np.testing.assert_allclose(got, dx[b, h0:h0 + r, w0:w0 + r, :], rtol=1e-5, atol=1e-5)
