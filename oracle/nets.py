"""Architectures as op lists, and a plain forward / backward interpreter.

Test infrastructure (see the package docstring).  The paper names its
architectures (Section 3: ResNet50 with 1000 classes, whose 32-bit size it
gives as 8e8 bits) without defining them; these are the standard definitions:

  tiny_cnn   conv3x3(3->16)+bias, ReLU, conv3x3(16->32)+bias, ReLU, global
             average pool, linear(32->10)+bias; stride 1, zero padding 1.
  resnet20   CIFAR-style: conv3x3(3->16)-BN-ReLU, 3 stages x 3 basic blocks
             (widths 16/32/64, stride 2 entering stages 2 and 3, projection
             shortcut = 1x1 stride-2 conv + BN where the width changes), global
             average pool, linear(64->10)+bias.  Convs followed by BN carry no bias.
  resnet50   7x7-s2-p3 stem (64) - BN - ReLU - 3x3-s2-p1 max-pool, bottleneck
             stages 3/4/6/3 with widths 64/128/256/512 (x4 expansion), stride 2
             on the 3x3 conv of the first block of stages 2-4, projection
             shortcut in the first block of every stage, global average pool,
             linear(2048->classes)+bias.

  wide_resnet_split  the modified Wide-ResNet 28x10 of the multi-view experiment (Section 5); see the builder.

  transformer_head  the last position-wise sublayers of a Transformer decoder (Section 4 trains the
             Transformer of Vaswani et al.; base size: d_model 512, d_ff 2048, vocabulary 32768): the
             feed-forward sublayer W2 relu(W1 h + b1) + b2 with its residual connection and
             post-LayerNorm, then the output projection onto the vocabulary (no bias).  Input: the
             hidden states h, one row per target token, as a [rows, 1, 1, d_model] tensor (the dense
             layers are 1x1 convolutions over it).  The attention sublayers and the embeddings
             are not part of it.

  transformer  the encoder-decoder Transformer that Section 4 trains (Vaswani et al.; base size: 6 + 6
             layers, d_model 512, 8 heads, d_ff 2048, vocabulary 32768, shared by source, target and
             output projection).  Input: integer token ids [S, Ts + Tt], per sentence the Ts source
             tokens, then the Tt (shifted) target tokens; every sentence has the same lengths (no
             padding).  Embedding rows times sqrt(d_model) plus the sinusoidal position signal; an
             encoder layer is self-attention and feed-forward sublayers, each with a residual connection
             followed by LayerNorm (post-LN); a decoder layer is causal self-attention, attention over
             the encoder output, and feed-forward; the logits are the decoder output times the
             transposed embedding table (tied, no bias).  The three (two) input projections of an
             attention sublayer are one dense layer d -> 3d (d -> d for the queries and d -> 2d for
             keys and values of the encoder output), with biases; no dropout.

An architecture is (param_table, ops).  param_table is an ordered list of
(name, shape, kind, fan_in); ops is a list of dicts over integer tensor ids
(tensor 0 is the input image batch, the last op writes the logits).

Sensitivity studies.  `forward` takes an optional `perturb` map {tensor id: function}: the tensor
is replaced by function(tensor) as soon as it has been computed, before any op reads it.  Tests use
it to measure how far a small perturbation of chosen intermediate tensors (for instance rounding
them to a shorter floating-point format) moves the float64 result.  perturb=None (the default) is
the plain float64 definition; nothing in this package decides which tensors to perturb.
"""
import numpy as np
from . import layers as L


def op_params(o):
    """Names of the parameters an op uses."""
    keys = {"conv": ("w", "b"), "linear": ("w", "b"), "embed": ("w",), "bn": ("gamma", "beta"),
            "layernorm": ("gamma", "beta")}.get(o["op"], ())
    return [o[k] for k in keys if o.get(k)]


class Arch:
    def __init__(self, name):
        self.name = name
        self.params = []      # (name, shape, kind, fan_in)
        self.ops = []
        self.frozen = set()   # names of parameters in front of a frozen cut (never updated)
        self.n_tensors = 1    # tensor 0 = input

    def _t(self):
        self.n_tensors += 1
        return self.n_tensors - 1

    def _p(self, name, shape, kind, fan_in=0):
        self.params.append((name, tuple(shape), kind, fan_in))
        return name

    def conv(self, x, name, cin, cout, k, stride, pad, bias, groups=1):
        w = self._p(name + ".w", (cout, k, k, cin // groups), "conv_w", cin // groups * k * k)
        b = self._p(name + ".b", (cout,), "bias") if bias else None
        y = self._t()
        self.ops.append(dict(op="conv", x=x, y=y, w=w, b=b, stride=stride, pad=pad))
        return y

    def bn(self, x, name, c):
        g = self._p(name + ".gamma", (c,), "bn_gamma")
        b = self._p(name + ".beta", (c,), "bn_beta")
        y = self._t()
        self.ops.append(dict(op="bn", x=x, y=y, gamma=g, beta=b))
        return y

    def relu(self, x):
        y = self._t()
        self.ops.append(dict(op="relu", x=x, y=y))
        return y

    def add(self, a, b):
        y = self._t()
        self.ops.append(dict(op="add", a=a, b=b, y=y))
        return y

    def maxpool(self, x, k, stride, pad):
        y = self._t()
        self.ops.append(dict(op="maxpool", x=x, y=y, k=k, stride=stride, pad=pad))
        return y

    def gap(self, x):
        y = self._t()
        self.ops.append(dict(op="gap", x=x, y=y))
        return y

    def frozen_slice(self, x, c0, n):
        """Channels c0 .. c0+n of x.  Everything in front of it is frozen: no gradient passes it."""
        y = self._t()
        self.ops.append(dict(op="slice", x=x, y=y, c0=c0, n=n))
        self.frozen = {name for o in self.ops for name in op_params(o)}
        return y

    def layernorm(self, x, name, c):
        g = self._p(name + ".gamma", (c,), "bn_gamma")
        b = self._p(name + ".beta", (c,), "bn_beta")
        y = self._t()
        self.ops.append(dict(op="layernorm", x=x, y=y, gamma=g, beta=b))
        return y

    def linear(self, x, name, fin, fout, bias=True):
        w = self._p(name + ".w", (fout, fin), "linear_w", fin)
        b = self._p(name + ".b", (fout,), "bias") if bias else None
        y = self._t()
        self.ops.append(dict(op="linear", x=x, y=y, w=w, b=b))
        return y

    def embed(self, name, vocab, d, col0, T, table=None):
        """Rows of the embedding table for the tokens in columns col0 .. col0+T of the input."""
        w = table if table is not None else self._p(name + ".w", (vocab, d), "embed_w", d)
        y = self._t()
        self.ops.append(dict(op="embed", x=0, y=y, w=w, col0=col0, T=T))
        return y, w

    def attention(self, q, q_col, kv, k_col, v_col, d, heads, S, causal, key_tokens):
        """q, k, v are column ranges of width d of tensors q and kv (which may be the same tensor).  key_tokens =
        (first column, count): the columns of the token input whose sentences the keys come from; their lengths
        (padding excluded) limit the keys each sentence attends to."""
        y = self._t()
        self.ops.append(dict(op="attn", x=q, kv=kv, y=y, q_col=q_col, k_col=k_col, v_col=v_col, d=d, heads=heads,
                             S=S, causal=causal, key_tokens=key_tokens))
        return y

    def tied_linear(self, x, w):
        """Logits against an existing [vocab, d] table (no bias)."""
        y = self._t()
        self.ops.append(dict(op="linear", x=x, y=y, w=w, b=None))
        return y

    def n_params(self):
        return int(sum(int(np.prod(s)) for _, s, _, _ in self.params))


def tiny_cnn(classes=10):
    a = Arch("tiny_cnn")
    t = a.conv(0, "conv1", 3, 16, 3, 1, 1, bias=True)
    t = a.relu(t)
    t = a.conv(t, "conv2", 16, 32, 3, 1, 1, bias=True)
    t = a.relu(t)
    t = a.gap(t)
    a.linear(t, "fc", 32, classes)
    return a


def resnet20(classes=10, widths=(16, 32, 64), blocks=(3, 3, 3)):
    a = Arch("resnet20")
    t = a.conv(0, "stem.conv", 3, widths[0], 3, 1, 1, bias=False)
    t = a.relu(a.bn(t, "stem.bn", widths[0]))
    cin = widths[0]
    for si, (wd, nb) in enumerate(zip(widths, blocks)):
        for bi in range(nb):
            stride = 2 if (si > 0 and bi == 0) else 1
            p = "s%d.b%d" % (si + 1, bi)
            u = a.conv(t, p + ".conv1", cin, wd, 3, stride, 1, bias=False)
            u = a.relu(a.bn(u, p + ".bn1", wd))
            u = a.conv(u, p + ".conv2", wd, wd, 3, 1, 1, bias=False)
            u = a.bn(u, p + ".bn2", wd)
            if stride != 1 or cin != wd:
                sc = a.conv(t, p + ".down.conv", cin, wd, 1, stride, 0, bias=False)
                sc = a.bn(sc, p + ".down.bn", wd)
            else:
                sc = t
            t = a.relu(a.add(u, sc))
            cin = wd
    t = a.gap(t)
    a.linear(t, "fc", cin, classes)
    return a


def wide_resnet_split(split=0, n_splits=8, classes=10, widths=(160, 320, 640), blocks=(4, 4, 4), stem=16):
    """The modified Wide-ResNet of the paper's multi-view experiment (Section 5): a Wide-ResNet 28x10 (three stages of
    four blocks, widths 160 / 320 / 640 behind a 16-channel 3x3 stem) whose first block is kept frozen; the 160
    channels it produces are cut into n_splits = 8 parts of 20 and the rest of the network receives part `split`
    only.  The paper gives no more than this; the block is the basic block of resnet20 above (the reading taken: the
    experiment is about which channels the trainable part sees, not about the order of BatchNorm and convolution
    inside a block).  Frozen: the backward pass stops at the cut and the front end's gradients are zero."""
    a = Arch("wide_resnet_split")
    t = a.conv(0, "stem.conv", 3, stem, 3, 1, 1, bias=False)
    t = a.relu(a.bn(t, "stem.bn", stem))
    cin = stem
    for si, (wd, nb) in enumerate(zip(widths, blocks)):
        for bi in range(nb):
            stride = 2 if (si > 0 and bi == 0) else 1
            p = "s%d.b%d" % (si + 1, bi)
            u = a.conv(t, p + ".conv1", cin, wd, 3, stride, 1, bias=False)
            u = a.relu(a.bn(u, p + ".bn1", wd))
            u = a.conv(u, p + ".conv2", wd, wd, 3, 1, 1, bias=False)
            u = a.bn(u, p + ".bn2", wd)
            if stride != 1 or cin != wd:
                sc = a.conv(t, p + ".down.conv", cin, wd, 1, stride, 0, bias=False)
                sc = a.bn(sc, p + ".down.bn", wd)
            else:
                sc = t
            t = a.relu(a.add(u, sc))
            cin = wd
            if si == 0 and bi == 0:
                cin = wd // n_splits
                t = a.frozen_slice(t, split * cin, cin)
    t = a.gap(t)
    a.linear(t, "fc", cin, classes)
    return a


def resnet18(classes=1000, widths=(64, 128, 256, 512), blocks=(2, 2, 2, 2), stem=64):
    """The basic-block network with the ImageNet front end (7x7 stride-2 stem, 3x3 stride-2 max-pool): the smaller
    model of the paper's pairs of different architectures (Section 5)."""
    a = Arch("resnet18")
    t = a.conv(0, "stem.conv", 3, stem, 7, 2, 3, bias=False)
    t = a.relu(a.bn(t, "stem.bn", stem))
    t = a.maxpool(t, 3, 2, 1)
    cin = stem
    for si, (wd, nb) in enumerate(zip(widths, blocks)):
        for bi in range(nb):
            stride = 2 if (si > 0 and bi == 0) else 1
            p = "s%d.b%d" % (si + 1, bi)
            u = a.conv(t, p + ".conv1", cin, wd, 3, stride, 1, bias=False)
            u = a.relu(a.bn(u, p + ".bn1", wd))
            u = a.conv(u, p + ".conv2", wd, wd, 3, 1, 1, bias=False)
            u = a.bn(u, p + ".bn2", wd)
            if stride != 1 or cin != wd:
                sc = a.conv(t, p + ".down.conv", cin, wd, 1, stride, 0, bias=False)
                sc = a.bn(sc, p + ".down.bn", wd)
            else:
                sc = t
            t = a.relu(a.add(u, sc))
            cin = wd
    t = a.gap(t)
    a.linear(t, "fc", cin, classes)
    return a


def resnext(classes=1000, widths=(256, 512, 1024, 2048), outs=(256, 512, 1024, 2048), groups=32, blocks=(3, 4, 23, 3),
            stem=64):
    """The bottleneck network with a grouped 3x3 convolution (aggregated transformations; the defaults are the
    101-layer 32x8d model, widths (128, ..., 1024) and blocks (3, 4, 6, 3) the 50-layer 32x4d one): the largest
    model of the paper's pairs of different architectures (Section 5).  widths: channels of the grouped
    convolution per stage; outs: channels of the block's output."""
    a = Arch("resnext")
    t = a.conv(0, "stem.conv", 3, stem, 7, 2, 3, bias=False)
    t = a.relu(a.bn(t, "stem.bn", stem))
    t = a.maxpool(t, 3, 2, 1)
    cin = stem
    for si, (wd, out, nb) in enumerate(zip(widths, outs, blocks)):
        for bi in range(nb):
            stride = 2 if (si > 0 and bi == 0) else 1
            p = "s%d.b%d" % (si + 1, bi)
            u = a.conv(t, p + ".conv1", cin, wd, 1, 1, 0, bias=False)
            u = a.relu(a.bn(u, p + ".bn1", wd))
            u = a.conv(u, p + ".conv2", wd, wd, 3, stride, 1, bias=False, groups=groups)
            u = a.relu(a.bn(u, p + ".bn2", wd))
            u = a.conv(u, p + ".conv3", wd, out, 1, 1, 0, bias=False)
            u = a.bn(u, p + ".bn3", out)
            if bi == 0:
                sc = a.conv(t, p + ".down.conv", cin, out, 1, stride, 0, bias=False)
                sc = a.bn(sc, p + ".down.bn", out)
            else:
                sc = t
            t = a.relu(a.add(u, sc))
            cin = out
    t = a.gap(t)
    a.linear(t, "fc", cin, classes)
    return a


def resnet50(classes=1000, widths=(64, 128, 256, 512), blocks=(3, 4, 6, 3), stem=64):
    a = Arch("resnet50")
    t = a.conv(0, "stem.conv", 3, stem, 7, 2, 3, bias=False)
    t = a.relu(a.bn(t, "stem.bn", stem))
    t = a.maxpool(t, 3, 2, 1)
    cin = stem
    for si, (wd, nb) in enumerate(zip(widths, blocks)):
        for bi in range(nb):
            stride = 2 if (si > 0 and bi == 0) else 1
            p = "s%d.b%d" % (si + 1, bi)
            u = a.conv(t, p + ".conv1", cin, wd, 1, 1, 0, bias=False)
            u = a.relu(a.bn(u, p + ".bn1", wd))
            u = a.conv(u, p + ".conv2", wd, wd, 3, stride, 1, bias=False)
            u = a.relu(a.bn(u, p + ".bn2", wd))
            u = a.conv(u, p + ".conv3", wd, 4 * wd, 1, 1, 0, bias=False)
            u = a.bn(u, p + ".bn3", 4 * wd)
            if bi == 0:
                sc = a.conv(t, p + ".down.conv", cin, 4 * wd, 1, stride, 0, bias=False)
                sc = a.bn(sc, p + ".down.bn", 4 * wd)
            else:
                sc = t
            t = a.relu(a.add(u, sc))
            cin = 4 * wd
    t = a.gap(t)
    a.linear(t, "fc", cin, classes)
    return a


def transformer_head(d_model=512, d_ff=2048, vocab=32768):
    a = Arch("transformer_head")
    u = a.conv(0, "ffn.w1", d_model, d_ff, 1, 1, 0, bias=True)
    u = a.relu(u)
    u = a.conv(u, "ffn.w2", d_ff, d_model, 1, 1, 0, bias=True)
    t = a.layernorm(a.add(u, 0), "ffn.ln", d_model)
    a.linear(t, "proj", d_model, vocab, bias=False)
    return a


def transformer(S, Ts, Tt, d=512, heads=8, d_ff=2048, vocab=32768, enc_layers=6, dec_layers=6):
    a = Arch("transformer")

    def dense(x, name, fin, fout):
        return a.conv(x, name, fin, fout, 1, 1, 0, bias=True)

    def add_norm(x, sub, name):
        return a.layernorm(a.add(sub, x), name, d)

    def ffn(x, p):
        u = a.relu(dense(x, p + ".ffn.w1", d, d_ff))
        return add_norm(x, dense(u, p + ".ffn.w2", d_ff, d), p + ".ffn.ln")

    def self_attention(x, p, causal):
        qkv = dense(x, p + ".qkv", d, 3 * d)
        o = a.attention(qkv, 0, qkv, d, 2 * d, d, heads, S, causal, (Ts, Tt) if causal else (0, Ts))
        return add_norm(x, dense(o, p + ".out", d, d), p + ".ln")

    x, table = a.embed("embed", vocab, d, 0, Ts)
    for i in range(enc_layers):
        x = ffn(self_attention(x, "enc%d.self" % i, False), "enc%d" % i)
    memory = x
    y, _ = a.embed("embed", vocab, d, Ts, Tt, table=table)
    for i in range(dec_layers):
        p = "dec%d" % i
        y = self_attention(y, p + ".self", True)
        q = dense(y, p + ".cross.q", d, d)
        kv = dense(memory, p + ".cross.kv", d, 2 * d)
        o = a.attention(q, 0, kv, 0, d, d, heads, S, False, (0, Ts))
        y = add_norm(y, dense(o, p + ".cross.out", d, d), p + ".cross.ln")
        y = ffn(y, p)
    a.tied_linear(y, table)
    return a


def forward(arch, params, x, running=None, bn_eval=False, perturb=None):
    """Training-mode forward.  params: dict name -> float64 array.  Returns (logits, tape).
    perturb: optional {tensor id: function}; see the module docstring.
    running: list with one [mean, var] pair per BatchNorm op, in graph order.  With bn_eval the BatchNorms
    normalise with these averages (evaluation mode; the tape then cannot be used for a backward pass);
    otherwise they use the batch's statistics and, if running is given, update it in place."""
    T = {0: np.asarray(x, dtype=np.float64)}
    cache = {}
    bn_index = 0
    for i, o in enumerate(arch.ops):
        k = o["op"]
        if k == "conv":
            b = params[o["b"]] if o["b"] else None
            T[o["y"]] = L.conv2d_forward(T[o["x"]], params[o["w"]], b, o["stride"], o["pad"])
        elif k == "bn":
            if bn_eval:
                T[o["y"]] = L.batchnorm_eval(T[o["x"]], params[o["gamma"]], params[o["beta"]], *running[bn_index])
            else:
                T[o["y"]], cache[i] = L.batchnorm_forward(T[o["x"]], params[o["gamma"]], params[o["beta"]])
                if running is not None:
                    rows = T[o["x"]].size // T[o["x"]].shape[-1]
                    running[bn_index][:] = L.batchnorm_running_update(running[bn_index][0], running[bn_index][1], cache[i], rows)
            bn_index += 1
        elif k == "relu":
            T[o["y"]] = L.relu_forward(T[o["x"]])
        elif k == "add":
            T[o["y"]] = T[o["a"]] + T[o["b"]]
        elif k == "maxpool":
            T[o["y"]], cache[i] = L.maxpool_forward(T[o["x"]], o["k"], o["stride"], o["pad"])
        elif k == "gap":
            T[o["y"]] = L.gap_forward(T[o["x"]])
        elif k == "slice":
            T[o["y"]] = T[o["x"]][..., o["c0"]:o["c0"] + o["n"]].copy()
        elif k == "layernorm":
            T[o["y"]], cache[i] = L.layernorm_forward(T[o["x"]], params[o["gamma"]], params[o["beta"]])
        elif k == "embed":
            tok = T[0][:, o["col0"]:o["col0"] + o["T"]]
            T[o["y"]] = L.embed_forward(tok, params[o["w"]]).reshape(-1, 1, 1, params[o["w"]].shape[1])
        elif k == "attn":
            d = o["d"]
            q2 = T[o["x"]].reshape(T[o["x"]].shape[0], -1)
            kv2 = T[o["kv"]].reshape(T[o["kv"]].shape[0], -1)
            q, kk, v = q2[:, o["q_col"]:o["q_col"] + d], kv2[:, o["k_col"]:o["k_col"] + d], kv2[:, o["v_col"]:o["v_col"] + d]
            c0, n = o["key_tokens"]
            out, P = L.attention_forward(q, kk, v, o["S"], o["heads"], o["causal"], L.sentence_lengths(T[0][:, c0:c0 + n]))
            T[o["y"]], cache[i] = out.reshape(-1, 1, 1, d), P
        elif k == "linear":
            xin = T[o["x"]]
            T[o["y"]] = L.linear_forward(xin.reshape(xin.shape[0], -1), params[o["w"]],
                                         params[o["b"]] if o["b"] else None)
        else:
            raise ValueError(k)
        if perturb is not None and o["y"] in perturb:
            T[o["y"]] = perturb[o["y"]](T[o["y"]])
    return T[arch.ops[-1]["y"]], (T, cache)


def backward(arch, params, tape, dlogits):
    """Gradient of the scalar loss with respect to every parameter, given d loss / d logits."""
    T, cache = tape
    G = {arch.ops[-1]["y"]: np.asarray(dlogits, dtype=np.float64)}
    grads = {}

    def acc(t, g):
        if t == 0 or g is None:
            return
        G[t] = g if t not in G else G[t] + g

    def accp(name, g):       # a parameter used by several ops (the tied embedding table) sums their gradients
        grads[name] = g if name not in grads else grads[name] + g

    for i in reversed(range(len(arch.ops))):
        o = arch.ops[i]
        k = o["op"]
        if o["y"] not in G:     # in front of a frozen cut: no gradient arrives, the parameters' gradients are zero
            for name in op_params(o):
                grads.setdefault(name, np.zeros_like(params[name]))
            continue
        dy = G.pop(o["y"])
        if k == "conv":
            dx, dw, db = L.conv2d_backward(T[o["x"]], params[o["w"]], dy, o["stride"], o["pad"],
                                           o["b"] is not None, need_dx=(o["x"] != 0))
            grads[o["w"]] = dw
            if o["b"]:
                grads[o["b"]] = db
            acc(o["x"], dx)
        elif k == "bn":
            dx, dg, db = L.batchnorm_backward(dy, params[o["gamma"]], cache[i])
            grads[o["gamma"]], grads[o["beta"]] = dg, db
            acc(o["x"], dx)
        elif k == "relu":
            acc(o["x"], L.relu_backward(T[o["y"]], dy))
        elif k == "add":
            acc(o["a"], dy)
            acc(o["b"], dy)
        elif k == "maxpool":
            acc(o["x"], L.maxpool_backward(T[o["x"]].shape, cache[i], dy, o["k"], o["stride"], o["pad"]))
        elif k == "gap":
            acc(o["x"], L.gap_backward(T[o["x"]].shape, dy))
        elif k == "slice":
            pass                 # frozen cut: the gradient stops here
        elif k == "layernorm":
            dx, dg, db = L.layernorm_backward(dy, params[o["gamma"]], cache[i])
            grads[o["gamma"]], grads[o["beta"]] = dg, db
            acc(o["x"], dx)
        elif k == "embed":
            tok = T[0][:, o["col0"]:o["col0"] + o["T"]]
            accp(o["w"], L.embed_backward(tok, params[o["w"]].shape, dy))
        elif k == "attn":
            d = o["d"]
            xq, xkv = T[o["x"]], T[o["kv"]]
            q2, kv2 = xq.reshape(xq.shape[0], -1), xkv.reshape(xkv.shape[0], -1)
            q, kk, v = q2[:, o["q_col"]:o["q_col"] + d], kv2[:, o["k_col"]:o["k_col"] + d], kv2[:, o["v_col"]:o["v_col"] + d]
            dq, dk, dv = L.attention_backward(q, kk, v, cache[i], dy.reshape(-1, d), o["S"], o["heads"])
            gq, gkv = np.zeros_like(q2), np.zeros_like(kv2)
            gq[:, o["q_col"]:o["q_col"] + d] += dq
            if o["kv"] == o["x"]:
                gq[:, o["k_col"]:o["k_col"] + d] += dk
                gq[:, o["v_col"]:o["v_col"] + d] += dv
            else:
                gkv[:, o["k_col"]:o["k_col"] + d] += dk
                gkv[:, o["v_col"]:o["v_col"] + d] += dv
                acc(o["kv"], gkv.reshape(xkv.shape))
            acc(o["x"], gq.reshape(xq.shape))
        elif k == "linear":
            xin = T[o["x"]]
            dx, dw, db = L.linear_backward(xin.reshape(xin.shape[0], -1), params[o["w"]], dy, o["b"] is not None)
            accp(o["w"], dw)
            if o["b"]:
                grads[o["b"]] = db
            acc(o["x"], dx.reshape(xin.shape))
    return grads
