"""Pins of the oracle's Transformer pieces (Section 4 of the paper trains the encoder-decoder Transformer of
Vaswani et al.): attention and embedding against closed forms, invariants, brute force and torch's own routines,
and the whole encoder-decoder against a separate torch implementation with autograd."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import layers as L
from oracle import nets
from oracle.step import codistill_step, flatten, unflatten


def rnd(shape, seed, sigma=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * sigma


def test_position_signal_and_embedding():
    pe = L.sinusoid_positions(7, 8)
    np.testing.assert_allclose(pe[0], [0, 1, 0, 1, 0, 1, 0, 1], atol=1e-15)
    np.testing.assert_allclose(pe[:, 0], np.sin(np.arange(7)), atol=1e-15)
    np.testing.assert_allclose(pe[:, 1], np.cos(np.arange(7)), atol=1e-15)
    assert pe[3, 6] == pytest.approx(math.sin(3 / 10000 ** 0.75), rel=1e-14)
    table = rnd((5, 8), 1)
    tok = np.array([[0, 4, 4], [2, 0, 1]])
    x = L.embed_forward(tok, table).reshape(2, 3, 8)
    for s in range(2):
        for t in range(3):
            np.testing.assert_allclose(x[s, t], table[tok[s, t]] * math.sqrt(8) + pe[t], atol=1e-14)
    dy = rnd((6, 8), 2)
    dw = L.embed_backward(tok, table.shape, dy)
    ref = np.zeros_like(table)
    for s in range(2):
        for t in range(3):
            ref[tok[s, t]] += math.sqrt(8) * dy[s * 3 + t]
    np.testing.assert_allclose(dw, ref, atol=1e-14)
    assert np.all(dw[3] == 0)                                  # a token that does not occur


@pytest.mark.parametrize("causal", [False, True])
def test_attention_matches_torch_and_brute_force(causal):
    S, T, H, dh = 3, 6, 4, 5
    d = H * dh
    q, k, v = rnd((S * T, d), 3), rnd((S * T, d), 4), rnd((S * T, d), 5)
    out, P = L.attention_forward(q, k, v, S, H, causal)
    np.testing.assert_allclose(P.sum(axis=-1), 1.0, atol=1e-14)
    # brute force, one (sentence, head, query) at a time
    for s in range(S):
        for h in range(H):
            for i in range(T):
                n = i + 1 if causal else T
                sc = np.array([q[s * T + i, h * dh:(h + 1) * dh] @ k[s * T + j, h * dh:(h + 1) * dh] for j in range(n)]) / math.sqrt(dh)
                w = np.exp(sc - sc.max())
                w /= w.sum()
                o = sum(w[j] * v[s * T + j, h * dh:(h + 1) * dh] for j in range(n))
                np.testing.assert_allclose(out[s * T + i, h * dh:(h + 1) * dh], o, atol=1e-13)
    # torch's routine and its autograd
    tq, tk, tv = (torch.tensor(a.reshape(S, T, H, dh).transpose(0, 2, 1, 3).copy(), requires_grad=True) for a in (q, k, v))
    to = F.scaled_dot_product_attention(tq, tk, tv, is_causal=causal)
    np.testing.assert_allclose(out.reshape(S, T, H, dh).transpose(0, 2, 1, 3), to.detach().numpy(), atol=1e-12)
    dout = rnd((S * T, d), 6)
    to.backward(torch.tensor(dout.reshape(S, T, H, dh).transpose(0, 2, 1, 3).copy()))
    dq, dk, dv = L.attention_backward(q, k, v, P, dout, S, H)
    for got, t in ((dq, tq), (dk, tk), (dv, tv)):
        np.testing.assert_allclose(got.reshape(S, T, H, dh).transpose(0, 2, 1, 3), t.grad.numpy(), atol=1e-12)


def test_attention_special_cases():
    S, T, H, dh = 2, 5, 2, 4
    d = H * dh
    k, v = rnd((S * T, d), 7), rnd((S * T, d), 8)
    # zero queries: uniform weights, the output is the mean of the values (of the visible prefix when causal)
    out, _ = L.attention_forward(np.zeros((S * T, d)), k, v, S, H, False)
    np.testing.assert_allclose(out.reshape(S, T, d), np.broadcast_to(v.reshape(S, T, d).mean(axis=1, keepdims=True), (S, T, d)), atol=1e-14)
    outc, _ = L.attention_forward(np.zeros((S * T, d)), k, v, S, H, True)
    np.testing.assert_allclose(outc.reshape(S, T, d)[:, 0], v.reshape(S, T, d)[:, 0], atol=1e-14)
    np.testing.assert_allclose(outc.reshape(S, T, d)[:, 2], v.reshape(S, T, d)[:, :3].mean(axis=1), atol=1e-14)
    # without a mask the keys have no order: permuting keys and values together changes nothing
    q = rnd((S * T, d), 9)
    perm = np.array([3, 0, 4, 1, 2])
    kp = k.reshape(S, T, d)[:, perm].reshape(S * T, d)
    vp = v.reshape(S, T, d)[:, perm].reshape(S * T, d)
    np.testing.assert_allclose(L.attention_forward(q, kp, vp, S, H, False)[0], L.attention_forward(q, k, v, S, H, False)[0], atol=1e-13)
    # sentences do not see each other
    k2 = k.copy()
    k2[T:] += 1.0
    a, b = L.attention_forward(q, k, v, S, H, False)[0], L.attention_forward(q, k2, v, S, H, False)[0]
    np.testing.assert_array_equal(a[:T], b[:T])
    # different source and target lengths
    kk, vv = rnd((S * 3, d), 10), rnd((S * 3, d), 11)
    o, P = L.attention_forward(q, kk, vv, S, H, False)
    assert o.shape == (S * T, d) and P.shape == (S, H, T, 3)


def test_base_parameter_count():
    # embedding 32768 x 512 (shared three ways); 6 encoder layers of 3,152,384; 6 decoder layers of 4,204,032
    assert nets.transformer(1, 1, 1).n_params() == 16777216 + 6 * 3152384 + 6 * 4204032 == 60915712


def torch_transformer(arch, P, tok, S, Ts, Tt, d, heads):
    """The same network written with torch's own layers (no code shared with the oracle)."""
    def dense(x, n):
        return F.linear(x, P[n + ".w"].reshape(P[n + ".w"].shape[0], -1), P[n + ".b"])

    def ln(x, n):
        return F.layer_norm(x, (d,), P[n + ".gamma"], P[n + ".beta"], eps=1e-5)

    def heads_of(x, T):
        return x.reshape(S, T, heads, d // heads).transpose(1, 2)

    def attend(q, k, v, Tq, Tk, causal):
        o = F.scaled_dot_product_attention(heads_of(q, Tq), heads_of(k, Tk), heads_of(v, Tk), is_causal=causal)
        return o.transpose(1, 2).reshape(S * Tq, d)

    def pos(T):
        t = torch.arange(T, dtype=torch.float64)[:, None]
        i = torch.arange(0, d, 2, dtype=torch.float64)[None, :]
        pe = torch.zeros(T, d, dtype=torch.float64)
        pe[:, 0::2], pe[:, 1::2] = torch.sin(t / 10000 ** (i / d)), torch.cos(t / 10000 ** (i / d))
        return pe

    def embed(tk, T):
        return (F.embedding(tk, P["embed.w"]) * math.sqrt(d) + pos(T)).reshape(S * T, d)

    def self_att(x, p, T, causal):
        qkv = dense(x, p + ".qkv")
        o = attend(qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:], T, T, causal)
        return ln(x + dense(o, p + ".out"), p + ".ln")

    def ffn(x, p):
        return ln(x + dense(torch.relu(dense(x, p + ".ffn.w1")), p + ".ffn.w2"), p + ".ffn.ln")

    n_enc = sum(1 for n, _, _, _ in arch.params if n.endswith(".self.qkv.w") and n.startswith("enc"))
    n_dec = sum(1 for n, _, _, _ in arch.params if n.endswith(".self.qkv.w") and n.startswith("dec"))
    x = embed(tok[:, :Ts], Ts)
    for i in range(n_enc):
        x = ffn(self_att(x, "enc%d.self" % i, Ts, False), "enc%d" % i)
    y = embed(tok[:, Ts:], Tt)
    for i in range(n_dec):
        p = "dec%d" % i
        y = self_att(y, p + ".self", Tt, True)
        kv = dense(x, p + ".cross.kv")
        o = attend(dense(y, p + ".cross.q"), kv[:, :d], kv[:, d:], Tt, Ts, False)
        y = ln(y + dense(o, p + ".cross.out"), p + ".cross.ln")
        y = ffn(y, p)
    return F.linear(y, P["embed.w"])


def tiny():
    S, Ts, Tt, d, heads, vocab = 2, 5, 4, 16, 4, 13
    arch = nets.transformer(S, Ts, Tt, d=d, heads=heads, d_ff=24, vocab=vocab, enc_layers=2, dec_layers=2)
    rng = np.random.default_rng(0)
    theta = np.concatenate([rng.standard_normal(int(np.prod(s))) * (1.0 if k in ("bn_gamma",) else 0.3) for _, s, k, _ in arch.params])
    tok = rng.integers(0, vocab, (S, Ts + Tt))
    y = rng.integers(0, vocab, S * Tt)
    return arch, theta, tok, y, (S, Ts, Tt, d, heads, vocab)


def test_encoder_decoder_matches_torch_autograd():
    arch, theta, tok, y, (S, Ts, Tt, d, heads, vocab) = tiny()
    P = unflatten(arch, theta)
    z, tape = nets.forward(arch, P, tok)
    tP = {k: torch.tensor(v, requires_grad=True) for k, v in P.items()}
    zt = torch_transformer(arch, tP, torch.tensor(tok), S, Ts, Tt, d, heads)
    np.testing.assert_allclose(z, zt.detach().numpy(), atol=1e-11)
    assert z.shape == (S * Tt, vocab)
    dz = rnd(z.shape, 5)
    (zt * torch.tensor(dz)).sum().backward()
    grads = nets.backward(arch, P, tape, dz)
    assert set(grads) == set(P)
    for n in P:
        np.testing.assert_allclose(grads[n], tP[n].grad.numpy(), atol=1e-10, err_msg=n)
    # the target tokens of a later position do not reach an earlier position's logits (causal decoder)
    tok2 = tok.copy()
    tok2[:, -1] = (tok2[:, -1] + 1) % vocab
    z2, _ = nets.forward(arch, P, tok2)
    np.testing.assert_array_equal(z.reshape(S, Tt, vocab)[:, :-1], z2.reshape(S, Tt, vocab)[:, :-1])
    assert np.abs(z.reshape(S, Tt, vocab)[:, -1] - z2.reshape(S, Tt, vocab)[:, -1]).max() > 1e-6


def test_codistillation_step_by_finite_differences():
    arch, theta, tok, y, _ = tiny()
    thp = theta + rnd(theta.shape, 9, 0.05)
    kw = dict(alpha=0.7, lr=0.1, momentum=0.9, label_smoothing=0.1, dist="kl")
    out = codistill_step(arch, theta, [thp], tok, y, **kw)
    rng = np.random.default_rng(4)
    h = 1e-6
    for j in rng.choice(theta.size, 12, replace=False):
        tp, tm = theta.copy(), theta.copy()
        tp[j] += h
        tm[j] -= h
        fd = (codistill_step(arch, tp, [thp], tok, y, **kw)["loss"][0] - codistill_step(arch, tm, [thp], tok, y, **kw)["loss"][0]) / (2 * h)
        assert abs(fd - out["grad"][j]) <= 1e-6 * max(1.0, abs(fd))
    # an identical peer adds nothing
    same = codistill_step(arch, theta, [theta], tok, y, **kw)
    assert abs(same["loss"][2]) < 1e-14


def test_attention_key_lengths_match_truncation_and_torch_mask():
    S, T, H, dh = 3, 6, 2, 4
    d = H * dh
    q, k, v = rnd((S * T, d), 20), rnd((S * T, d), 21), rnd((S * T, d), 22)
    klen = np.array([6, 2, 4])
    out, P = L.attention_forward(q, k, v, S, H, False, klen)
    for s in range(S):
        n = klen[s]
        assert np.all(P[s, :, :, n:] == 0)
        # the same sentence alone, cut to its length (all T queries kept)
        o1, _ = L.attention_forward(q[s * T:(s + 1) * T], k[s * T:s * T + n], v[s * T:s * T + n], 1, H, False)
        np.testing.assert_allclose(out[s * T:(s + 1) * T], o1, atol=1e-14)
    mask = torch.tensor(np.arange(T)[None, :] < klen[:, None])[:, None, None, :]
    tq, tk, tv = (torch.tensor(a.reshape(S, T, H, dh).transpose(0, 2, 1, 3).copy(), requires_grad=True) for a in (q, k, v))
    to = F.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask)
    np.testing.assert_allclose(out.reshape(S, T, H, dh).transpose(0, 2, 1, 3), to.detach().numpy(), atol=1e-12)
    dout = rnd((S * T, d), 23)
    to.backward(torch.tensor(dout.reshape(S, T, H, dh).transpose(0, 2, 1, 3).copy()))
    dq, dk, dv = L.attention_backward(q, k, v, P, dout, S, H)
    for got, t in ((dq, tq), (dk, tk), (dv, tv)):
        np.testing.assert_allclose(got.reshape(S, T, H, dh).transpose(0, 2, 1, 3), t.grad.numpy(), atol=1e-12)
    assert np.all(dk.reshape(S, T, d)[1, 2:] == 0) and np.all(dv.reshape(S, T, d)[1, 2:] == 0)   # padded keys: no gradient


def test_padded_batch_equals_its_sentences_run_alone():
    """Sentences of different lengths padded into one batch (negative ids): the logits of every real target position,
    and the parameter gradients when the padded positions carry no loss gradient, are those of the sentences run one
    at a time at their own lengths."""
    S, Ts, Tt, d, heads, vocab = 3, 6, 5, 16, 4, 11
    kw = dict(d=d, heads=heads, d_ff=24, vocab=vocab, enc_layers=2, dec_layers=2)
    arch = nets.transformer(S, Ts, Tt, **kw)
    rng = np.random.default_rng(3)
    theta = np.concatenate([rng.standard_normal(int(np.prod(s))) * 0.3 for _, s, _, _ in arch.params])
    P = unflatten(arch, theta)
    slen, tlen = [6, 3, 1], [2, 5, 4]
    tok = rng.integers(0, vocab, (S, Ts + Tt))
    for s in range(S):
        tok[s, slen[s]:Ts] = -1
        tok[s, Ts + tlen[s]:] = -1
    z, tape = nets.forward(arch, P, tok)
    z3 = z.reshape(S, Tt, vocab)
    dz = rnd(z.shape, 6).reshape(S, Tt, vocab)
    for s in range(S):
        dz[s, tlen[s]:] = 0.0
    grads = nets.backward(arch, P, tape, dz.reshape(z.shape))
    total = {n: np.zeros_like(v) for n, v in P.items()}
    for s in range(S):
        one = nets.transformer(1, slen[s], tlen[s], **kw)
        t1 = np.concatenate([tok[s, :slen[s]], tok[s, Ts:Ts + tlen[s]]])[None, :]
        z1, tape1 = nets.forward(one, P, t1)
        np.testing.assert_allclose(z3[s, :tlen[s]], z1, atol=1e-11)
        g1 = nets.backward(one, P, tape1, dz[s, :tlen[s]])
        for n in total:
            total[n] += g1[n]
    for n in total:
        np.testing.assert_allclose(grads[n], total[n], atol=1e-10, err_msg=n)
    # padding changes nothing for the others: another sentence's padding length is invisible to sentence 0
    tok2 = tok.copy()
    tok2[1, 2] = -1
    z2, _ = nets.forward(arch, P, tok2)
    np.testing.assert_array_equal(z3[0], z2.reshape(S, Tt, vocab)[0])
