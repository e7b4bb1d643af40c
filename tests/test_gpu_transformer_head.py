"""GPU parity of the Transformer output block (feed-forward sublayer with residual, post-LayerNorm,
projection onto the vocabulary) inside a codistillation step, through the C ABI, against the float64
oracle.  Label smoothing 0.1 and alpha = 1 as in the translation workload; hidden states ~ N(0,1).
"""
import numpy as np
import pytest
import torch

from oracle import nets
from paper_2010_02838_amd import synth

from gpu_util import Case, bf16_storage_points, rel
from test_gpu_step import check_layers, compare_bf16, compare_f32

pytestmark = pytest.mark.gpu


def head_case(dtype, rows, d, ff, vocab, jitter=0.1):
    return Case(dict(kind=3, widths=[d, ff]), nets.transformer_head(d, ff, vocab), dtype, rows, 1, vocab, jitter=jitter,
                in_c=d)


def test_head_fp32_step():
    """Any widths (plain kernels, scalar LayerNorm path), ragged everywhere."""
    c = head_case("f32", 37, 20, 44, 51)
    ref, got = c.oracle(label_smoothing=0.1), c.gpu(label_smoothing=0.1)
    compare_f32(ref, got, c.ref_arch, 2e-5, 2e-5, 5e-4, 1e-5)


@pytest.mark.parametrize("dist", ["mse", "kl"])
def test_head_fp32_vector_path(dist):
    c = head_case("f32", 70, 64, 96, 200)
    ref, got = c.oracle(label_smoothing=0.1, dist=dist, wd=1e-3), c.gpu(label_smoothing=0.1, dist=dist, wd=1e-3)
    compare_f32(ref, got, c.ref_arch, 2e-5, 2e-5, 5e-4, 1e-5)
    check_layers(c, got)


@pytest.mark.parametrize("shape", [(70, 64, 96, 200), (300, 136, 264, 1000), (130, 1024, 512, 264)])
def test_head_bf16_layers(shape):
    """Every op teacher-forced (MFMA dense layers with bias and ReLU in the epilogue, the vector LayerNorm
    kernels with one and two vectors per lane, the fp32 projection epilogue with ragged tiles)."""
    c = head_case("bf16", *shape)
    check_layers(c, c.gpu(label_smoothing=0.1))


def test_head_bf16_step():
    c = head_case("bf16", 300, 136, 264, 1000)
    compare_bf16(c, c.oracle(label_smoothing=0.1), c.oracle(label_smoothing=0.1, bf16_storage=True),
                 c.gpu(label_smoothing=0.1), label="transformer_head")


def test_head_bf16_layers_base_widths():
    """d_model 512, d_ff 2048, vocabulary 32768 (the base Transformer), 384 rows so that the float64
    oracle finishes in seconds."""
    c = head_case("bf16", 384, 512, 2048, 32768, jitter=0.0)
    check_layers(c, c.gpu(label_smoothing=0.1))


def test_head_bf16_full_size_sampled():
    """8192 target tokens, base widths: the forward pass is independent per row, so the oracle recomputes
    sampled rows of the logits and of d loss / d logits (given the GPU's own logits of those rows)."""
    from oracle import loss as OL
    rows, d, ff, vocab = 8192, 512, 2048, 32768
    c = head_case("bf16", rows, d, ff, vocab, jitter=0.0)
    got = c.gpu(label_smoothing=0.1)
    pick = np.random.default_rng(0).choice(rows, size=48, replace=False)
    P = c.per_tensor(c.th.astype(np.float64))
    Pp = c.per_tensor(c.thp.astype(np.float64))
    points = bf16_storage_points(c.ref_arch)
    z, _ = nets.forward(c.ref_arch, P, c.x[pick].astype(np.float64), perturb=points)
    zp, _ = nets.forward(c.ref_arch, Pp, c.x[pick].astype(np.float64), perturb=points)
    assert rel(got["logits"][pick], z) <= 5e-3
    assert rel(got["peer_logits"][pick], zp) <= 5e-3
    # gradient rows: the loss kernel's result for these rows from the GPU's own logits (mean over all rows)
    (_, _, _), dz = OL.codistill_loss_grad(got["logits"][pick].astype(np.float64), [got["peer_logits"][pick].astype(np.float64)],
                                           c.y[pick], 1.0, label_smoothing=0.1)
    assert rel(got["dz"][pick] * (rows / len(pick)), dz) <= 1e-5
    assert np.isfinite(got["grad"]).all() and np.isfinite(got["loss"]).all()


def test_separate_relu_mask_switch_agrees(monkeypatch):
    """CODISTILL_SEPARATE_RELU_MASK=1 runs the backward pass of the feed-forward layer's fused ReLU as a kernel of its
    own instead of in the epilogue of the data-gradient kernel: masking is exact, so the gradients agree."""
    a = head_case("bf16", 300, 136, 264, 1000).gpu(label_smoothing=0.1)
    monkeypatch.setenv("CODISTILL_SEPARATE_RELU_MASK", "1")
    c = head_case("bf16", 300, 136, 264, 1000)
    b = c.gpu(label_smoothing=0.1)
    check_layers(c, b)
    np.testing.assert_array_equal(a["logits"], b["logits"])
    assert rel(b["grad"], a["grad"].astype(np.float64)) <= 1e-6
