"""GPU parity of the encoder-decoder Transformer (bf16) through the C ABI: every op teacher-forced against
the float64 oracle, and the whole codistillation step end to end."""
import numpy as np
import pytest

from oracle import nets
from paper_2010_02838_amd import synth
from gpu_util import Case, PackedCase, rel
from test_gpu_step import check_layers, compare_bf16

pytestmark = pytest.mark.gpu

CASES = {
    # S, Ts, Tt, d, heads, d_ff, vocab, encoder layers, decoder layers
    "small": (3, 10, 7, 32, 4, 64, 64, 2, 2),                 # head dimension 8
    "ragged_vocab": (2, 5, 9, 32, 2, 40, 50, 1, 2),           # head dimension 16, vocabulary not a multiple of 8
    "long": (2, 150, 131, 128, 2, 128, 96, 1, 1),             # head dimension 64 (the matrix-core kernels); several
                                                              # query tiles and key chunks, ragged last ones
    "mid": (2, 70, 33, 64, 2, 96, 80, 1, 1),                  # head dimension 32 (matrix-core kernels as well)
    "wide": (2, 20, 17, 1024, 16, 256, 64, 1, 1),             # the width and head count of the "big" model
}


def make(name, ragged=False):
    S, Ts, Tt, d, heads, ff, vocab, ne, nd = CASES[name]
    ref = nets.transformer(S, Ts, Tt, d=d, heads=heads, d_ff=ff, vocab=vocab, enc_layers=ne, dec_layers=nd)
    return Case(dict(kind=4, widths=[d, ff, heads], blocks=[ne, nd]), ref, "bf16", S, 0, vocab, jitter=0.1,
                tokens=(Ts, Tt), ragged=ragged)


@pytest.mark.parametrize("name", list(CASES))
def test_transformer_bf16_layers(name):
    c = make(name)
    check_layers(c, c.gpu(alpha=0.5, label_smoothing=0.1))


@pytest.mark.parametrize("name", ["small", "long", "mid"])
def test_transformer_padded_sentences_bf16_layers(name):
    """Sentences of different lengths in one batch (padding = negative ids, ignored labels): both sets of attention
    kernels mask the padded keys, the embedding skips them, forward and backward."""
    c = make(name, ragged=True)
    got = c.gpu(alpha=0.5, label_smoothing=0.1)
    check_layers(c, got)
    # padded positions carry no loss gradient
    assert np.all(got["dz"][c.y < 0] == 0)


def make_packed(name, multiple=16, slack_sentences=3):
    """The ragged batch of make(name, ragged=True), handed to the library without its padding."""
    S, Ts, Tt, d, heads, ff, vocab, ne, nd = CASES[name]
    return PackedCase(make(name, ragged=True), dict(kind=4, widths=[d, ff, heads], blocks=[ne, nd]), Ts, Tt,
                      multiple=multiple, slack_sentences=slack_sentences)


@pytest.mark.parametrize("name,multiple,slack", [("small", 16, 3), ("long", 128, 0), ("mid", 1, 1), ("wide", 8, 2)])
def test_transformer_packed_sentences_bf16_layers(name, multiple, slack):
    """Sentences of different lengths one after the other, no padding rows (cd_arch_desc.max_sentences): every op against
    the oracle's layer functions on the padded form of the same batch, forward and backward, on the rows that exist.
    Stream capacities with unused rows behind the last sentence (a multiple of 16 / 128), without any (multiple 1), as
    many sentences as the model allows (slack 0), sentences longer than one 128-row attention tile ("long")."""
    c = make_packed(name, multiple, slack)
    got = c.gpu(alpha=0.5, label_smoothing=0.1)
    check_layers(c, got)
    # the rows behind the last sentence take no loss gradient, and what the attention kernels leave there is zero
    assert np.all(c.runner.dz.cpu().numpy()[len(c.tgt_map):] == 0)


def test_transformer_packed_sentences_bf16_step():
    c = make_packed("small")
    kw = dict(alpha=0.5, label_smoothing=0.1)
    compare_bf16(c, c.oracle(**kw), c.oracle(bf16_storage=True, **kw), c.gpu(**kw), label="transformer_small_packed")


def test_packed_and_padded_forms_agree():
    """The same sentences in both forms: equal losses and gradients up to the rounding order of the sums over rows."""
    c = make_packed("mid")
    kw = dict(alpha=0.5, label_smoothing=0.1)
    a, b = c.gpu(**kw), c.c0.gpu(**kw)
    np.testing.assert_allclose(a["loss"], b["loss"], rtol=1e-4)
    keep = c.valid_rows(1).reshape(-1)
    assert rel(a["logits"][keep], b["logits"][keep].astype(np.float64)) <= 1e-5
    Ga, Gb = c.per_tensor(a["grad"]), c.per_tensor(b["grad"])
    for n in Gb:
        assert rel(Ga[n], Gb[n].astype(np.float64)) <= 2e-3, n


def test_transformer_padded_sentences_bf16_step():
    c = make("small", ragged=True)
    kw = dict(alpha=0.5, label_smoothing=0.1)
    compare_bf16(c, c.oracle(**kw), c.oracle(bf16_storage=True, **kw), c.gpu(**kw), label="transformer_small_padded")


@pytest.mark.parametrize("name", ["small", "ragged_vocab"])
def test_transformer_bf16_step(name):
    c = make(name)
    kw = dict(alpha=0.5, label_smoothing=0.1)
    compare_bf16(c, c.oracle(**kw), c.oracle(bf16_storage=True, **kw), c.gpu(**kw), label="transformer_" + name)


def test_transformer_kl_step_and_base_shape_metadata():
    c = make("small")
    kw = dict(alpha=1.0, label_smoothing=0.1, dist="kl")
    compare_bf16(c, c.oracle(**kw), c.oracle(bf16_storage=True, **kw), c.gpu(**kw), label="transformer_small_kl")
    B = c.B
    base = B.Model(B.arch_preset(B.CD_ARCH_TRANSFORMER), B.CD_BF16)
    assert sum(p["size"] for p in base.params) == 60915712
    assert base.rows_per_sample == 128


@pytest.mark.timeout(900)
def test_transformer_base_size_layers():
    """The benchmarked shape (base model, 64 sentences of 128 source + 128 target tokens, vocabulary 32768, the
    two-stream launch configuration): every op of the 12 layers teacher-forced against the oracle, all elements."""
    S, Ts, Tt = 64, 128, 128
    ref = nets.transformer(S, Ts, Tt)
    c = Case(dict(kind=4), ref, "bf16", S, 0, 32768, jitter=0.1, tokens=(Ts, Tt))
    got = c.gpu(alpha=1.0, label_smoothing=0.1)
    assert np.isfinite(got["loss"]).all() and got["loss"][2] > 0
    check_layers(c, got)


@pytest.mark.timeout(1500)
def test_transformer_base_size_packed_layers():
    """The default benchmark batch (base model, sentence pairs with lengths uniform in [16, 128] up to 8192 target
    tokens, packed, rows of each stream a multiple of 128, as many sentences as the model allows, the two-stream launch
    configuration): every op of the 12 layers teacher-forced against the oracle on the padded form, all rows that exist."""
    Ts = Tt = 128
    x, y, sl, tl = synth.sentence_pairs(8192, 16, 128, 32768, seed=100)
    S = x.shape[0]
    c0 = Case(dict(kind=4), nets.transformer(S, Ts, Tt), "bf16", S, 0, 32768, jitter=0.1, tokens=(Ts, Tt))
    c0.x, c0.y = x, y
    c = PackedCase(c0, dict(kind=4), Ts, Tt, multiple=128, slack_sentences=0)
    assert len(c.tgt_map) == tl.sum() >= 8192 and c.rows_tgt < S * Tt * 0.65
    got = c.gpu(alpha=1.0, label_smoothing=0.1)
    assert np.isfinite(got["loss"]).all() and got["loss"][2] > 0
    check_layers(c, got)


def test_transformer_step_is_bit_reproducible():
    """Two runs of the same step give identical bits (no atomics anywhere: the embedding gradient has one writer per
    table row and a fixed order of additions); tokens repeat many times at this vocabulary size."""
    import torch
    from paper_2010_02838_amd.runner import pack_flat, unpack_flat
    c = make("ragged_vocab", ragged=True)
    got = c.gpu(alpha=0.5, label_smoothing=0.1)
    r = c.runner
    r.load(pack_flat(c.model, c.th), [pack_flat(c.peer, c.thp)])
    r.step(torch.from_numpy(c.x).to("cuda:0"), torch.from_numpy(c.y).to("cuda:0"), 0.5, 0.1, 0.9, label_smoothing=0.1)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(unpack_flat(c.model, r.grads.cpu().numpy()), got["grad"])
    np.testing.assert_array_equal(r.logits.cpu().numpy(), got["logits"])


def test_transformer_adam_updates_through_the_runner():
    """Two steps with the Adam update: the weights follow the oracle's Adam applied to the gradients the backward
    pass produced (update counter, moment buffers and the bf16 shadow copy are wired correctly)."""
    import torch
    from oracle.adam import adam_step
    from paper_2010_02838_amd.runner import StepRunner, pack_flat
    c = make("small")
    r = StepRunner(c.model, [c.peer], c.batch)
    r.load(pack_flat(c.model, c.th), [pack_flat(c.peer, c.thp)])
    x, y = torch.from_numpy(c.x).to("cuda:0"), torch.from_numpy(c.y).to("cuda:0")
    w = r.master.cpu().numpy().astype(np.float64)
    m, v = np.zeros_like(w), np.zeros_like(w)
    for t in (1, 2):
        r.step(x, y, 0.5, 1e-2, 0.0, label_smoothing=0.1, adam=(0.9, 0.98, 1e-8))
        torch.cuda.synchronize()
        w, m, v = adam_step(w, m, v, r.grads.cpu().numpy(), 1e-2, t, 0.9, 0.98, 1e-8)
        got = r.master.cpu().numpy()
        assert np.abs(got - w).max() <= 1e-5 * 1e-2 * t + 2e-7 * np.abs(w).max()
        bits = r.lowp.view(torch.int16).cpu().numpy().view(np.uint16)
        np.testing.assert_array_equal(bits, synth.bf16_bits(got))
    assert r.updates == 2


@pytest.mark.parametrize("name", ["mid", "long"])
def test_plain_attention_switch_bf16_layers(monkeypatch, name):
    """CODISTILL_PLAIN_ATTENTION=1 runs head dimensions 32 and 64 on the plain fp32 attention kernels instead of the
    matrix-core ones: same per-layer tolerances against the oracle, padded sentences included."""
    monkeypatch.setenv("CODISTILL_PLAIN_ATTENTION", "1")
    c = make(name, ragged=True)
    check_layers(c, c.gpu(alpha=0.5, label_smoothing=0.1))
