"""Layer definitions and their vector-Jacobian products, NumPy float64.

Test infrastructure (see the package docstring).  These are the textbook
definitions of the layers that the architectures named in the paper (Section 3:
ResNet50; Section 4) are built from, written as their defining sums.  The paper
only names the architectures; the layer conventions are the standard ones:

  * activations are [B, H, W, C]; filters are [Cout, kh, kw, Cin];
  * convolution is cross-correlation with zero padding;
  * BatchNorm normalises with the biased batch variance over (B, H, W), eps 1e-5;
  * ReLU'(0) = 0; max-pool routes the gradient to the first maximum in
    row-major window order;
  * LayerNorm (the Transformer of Section 4, which the paper only names) normalises every row
    over its last axis with the biased variance, eps 1e-5, then scales and shifts per feature.
"""
import numpy as np

BN_EPS = 1e-5


def _out_size(n, k, stride, pad):
    return (n + 2 * pad - k) // stride + 1


LN_EPS = 1e-5


# ---------------------------------------------------------------- convolution
def _groups(cin, w):
    """Grouped convolution (the ResNeXt block): the filter holds cin / groups input channels per output channel;
    output channels [g*Cout/G, (g+1)*Cout/G) read input channels [g*Cin/G, (g+1)*Cin/G) only."""
    if cin % w.shape[3] or w.shape[0] % (cin // w.shape[3]):
        raise ValueError("filter %s does not divide %d input channels into groups" % (w.shape, cin))
    return cin // w.shape[3]


def conv2d_forward(x, w, bias, stride, pad):
    """y[b,ho,wo,o] = bias[o] + sum_{r,s,c} x[b, ho*stride-pad+r, wo*stride-pad+s, c] * w[o,r,s,c]
    (within the group of o when the filter has fewer input channels than x: see _groups)."""
    G = _groups(x.shape[3], w)
    if G > 1:
        cg, og = w.shape[3], w.shape[0] // G
        y = np.concatenate([conv2d_forward(x[..., g * cg:(g + 1) * cg], w[g * og:(g + 1) * og], None, stride, pad)
                            for g in range(G)], axis=3)
        return y if bias is None else y + bias
    B, H, W, Cin = x.shape
    Cout, kh, kw, _ = w.shape
    Ho, Wo = _out_size(H, kh, stride, pad), _out_size(W, kw, stride, pad)
    xp = np.zeros((B, H + 2 * pad, W + 2 * pad, Cin))
    xp[:, pad:pad + H, pad:pad + W, :] = x
    y = np.zeros((B, Ho, Wo, Cout))
    for r in range(kh):
        for s in range(kw):
            xs = xp[:, r:r + stride * (Ho - 1) + 1:stride, s:s + stride * (Wo - 1) + 1:stride, :]
            y += xs.reshape(-1, Cin).dot(w[:, r, s, :].T).reshape(B, Ho, Wo, Cout)
    if bias is not None:
        y += bias
    return y


def conv2d_backward(x, w, dy, stride, pad, has_bias, need_dx=True):
    """Return (dx, dw, dbias) of conv2d_forward for upstream gradient dy."""
    G = _groups(x.shape[3], w)
    if G > 1:
        cg, og = w.shape[3], w.shape[0] // G
        parts = [conv2d_backward(x[..., g * cg:(g + 1) * cg], w[g * og:(g + 1) * og], dy[..., g * og:(g + 1) * og],
                                 stride, pad, False, need_dx) for g in range(G)]
        dx = np.concatenate([p[0] for p in parts], axis=3) if need_dx else None
        dw = np.concatenate([p[1] for p in parts], axis=0)
        return dx, dw, (dy.reshape(-1, dy.shape[3]).sum(axis=0) if has_bias else None)
    B, H, W, Cin = x.shape
    Cout, kh, kw, _ = w.shape
    _, Ho, Wo, _ = dy.shape
    xp = np.zeros((B, H + 2 * pad, W + 2 * pad, Cin))
    xp[:, pad:pad + H, pad:pad + W, :] = x
    dxp = np.zeros_like(xp)
    dw = np.zeros_like(w)
    dy2 = dy.reshape(-1, Cout)
    for r in range(kh):
        for s in range(kw):
            sl = (slice(None), slice(r, r + stride * (Ho - 1) + 1, stride),
                  slice(s, s + stride * (Wo - 1) + 1, stride), slice(None))
            dw[:, r, s, :] = dy2.T.dot(xp[sl].reshape(-1, Cin))
            if need_dx:
                dxp[sl] += dy2.dot(w[:, r, s, :]).reshape(B, Ho, Wo, Cin)
    dx = dxp[:, pad:pad + H, pad:pad + W, :].copy() if need_dx else None
    db = dy2.sum(axis=0) if has_bias else None
    return dx, dw, db


# ------------------------------------------------------------------ BatchNorm
def batchnorm_forward(x, gamma, beta):
    """Training-mode BatchNorm over all axes but the last.  Returns (y, cache)."""
    C = x.shape[-1]
    x2 = x.reshape(-1, C)
    mean = x2.mean(axis=0)
    var = ((x2 - mean) ** 2).mean(axis=0)          # biased
    invstd = 1.0 / np.sqrt(var + BN_EPS)
    xhat = (x2 - mean) * invstd
    y = (gamma * xhat + beta).reshape(x.shape)
    return y, (xhat, invstd, mean, var)


BN_MOMENTUM = 0.1


def batchnorm_running_update(running_mean, running_var, cache, rows, momentum=BN_MOMENTUM):
    """The averages an evaluation-mode BatchNorm uses, after one training-mode forward pass (cache from
    batchnorm_forward over `rows` rows): (1 - momentum) * old + momentum * batch value, with the unbiased batch
    variance (the convention of the common implementations; the paper is silent).  Returns (mean, var)."""
    _, _, mean, var = cache
    unbiased = var * rows / max(rows - 1, 1)
    return (1.0 - momentum) * running_mean + momentum * mean, (1.0 - momentum) * running_var + momentum * unbiased


def batchnorm_eval(x, gamma, beta, running_mean, running_var):
    """Evaluation-mode BatchNorm: normalise with the running averages instead of the batch's statistics."""
    return gamma * (x - running_mean) / np.sqrt(running_var + BN_EPS) + beta


def batchnorm_backward(dy, gamma, cache):
    """Return (dx, dgamma, dbeta)."""
    xhat, invstd, _, _ = cache
    C = dy.shape[-1]
    dy2 = dy.reshape(-1, C)
    M = dy2.shape[0]
    dbeta = dy2.sum(axis=0)
    dgamma = (dy2 * xhat).sum(axis=0)
    dx = gamma * invstd * (dy2 - dbeta / M - xhat * dgamma / M)
    return dx.reshape(dy.shape), dgamma, dbeta


# ----------------------------------------------------------------------- glue
def relu_forward(x):
    return np.maximum(x, 0.0)


def relu_backward(y, dy):
    """y is the ReLU output; the derivative at 0 is 0."""
    return dy * (y > 0.0)


def maxpool_forward(x, k, stride, pad):
    """Returns (y, argmax) with argmax the window tap index r*k+s of the first maximum."""
    B, H, W, C = x.shape
    Ho, Wo = _out_size(H, k, stride, pad), _out_size(W, k, stride, pad)
    xp = np.full((B, H + 2 * pad, W + 2 * pad, C), -np.inf)
    xp[:, pad:pad + H, pad:pad + W, :] = x
    y = np.full((B, Ho, Wo, C), -np.inf)
    arg = np.zeros((B, Ho, Wo, C), dtype=np.int64)
    for r in range(k):
        for s in range(k):
            xs = xp[:, r:r + stride * (Ho - 1) + 1:stride, s:s + stride * (Wo - 1) + 1:stride, :]
            better = xs > y                         # strict: first maximum wins
            y = np.where(better, xs, y)
            arg = np.where(better, r * k + s, arg)
    return y, arg


def maxpool_backward(x_shape, arg, dy, k, stride, pad):
    B, H, W, C = x_shape
    _, Ho, Wo, _ = dy.shape
    dxp = np.zeros((B, H + 2 * pad, W + 2 * pad, C))
    for r in range(k):
        for s in range(k):
            sl = (slice(None), slice(r, r + stride * (Ho - 1) + 1, stride),
                  slice(s, s + stride * (Wo - 1) + 1, stride), slice(None))
            dxp[sl] += dy * (arg == r * k + s)
    return dxp[:, pad:pad + H, pad:pad + W, :].copy()


def gap_forward(x):
    """Global average pool [B,H,W,C] -> [B,C]."""
    return x.mean(axis=(1, 2))


def gap_backward(x_shape, dy):
    B, H, W, C = x_shape
    return np.broadcast_to(dy[:, None, None, :] / (H * W), x_shape).copy()


def linear_forward(x, w, bias):
    """y = x w^T + bias, w is [out, in]."""
    y = x.dot(w.T)
    if bias is not None:
        y = y + bias
    return y


def linear_backward(x, w, dy, has_bias):
    dx = dy.dot(w)
    dw = dy.T.dot(x)
    db = dy.sum(axis=0) if has_bias else None
    return dx, dw, db


# ------------------------------------------------------------------ LayerNorm
def layernorm_forward(x, gamma, beta):
    """y[..., j] = gamma[j] * (x[..., j] - mean) / sqrt(var + eps) + beta[j], mean and (biased) var over j."""
    mean = x.mean(axis=-1, keepdims=True)
    var = ((x - mean) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + LN_EPS)
    xhat = (x - mean) * rstd
    return gamma * xhat + beta, (xhat, rstd)


def layernorm_backward(dy, gamma, cache):
    """Return (dx, dgamma, dbeta).  With g = dy * gamma:
    dx = rstd * (g - mean_j(g) - xhat * mean_j(g * xhat))."""
    xhat, rstd = cache
    red = tuple(range(dy.ndim - 1))
    dgamma = (dy * xhat).sum(axis=red)
    dbeta = dy.sum(axis=red)
    g = dy * gamma
    dx = rstd * (g - g.mean(axis=-1, keepdims=True) - xhat * (g * xhat).mean(axis=-1, keepdims=True))
    return dx, dgamma, dbeta


# ------------------------------------------------------------- Transformer pieces
def sinusoid_positions(T, d):
    """Fixed position signal of the Transformer: PE[t, 2i] = sin(t / 10000^(2i/d)), PE[t, 2i+1] = cos(same)."""
    t = np.arange(T, dtype=np.float64)[:, None]
    i = np.arange(0, d, 2, dtype=np.float64)[None, :]
    ang = t / np.power(10000.0, i / d)
    pe = np.zeros((T, d))
    pe[:, 0::2] = np.sin(ang)
    pe[:, 1::2] = np.cos(ang)
    return pe


def embed_forward(tokens, table):
    """tokens [S, T] integer ids -> [S*T, d]: table row times sqrt(d), plus the position signal.  A negative id
    is padding: it embeds as a zero row (the position signal is still added; nothing reads that row)."""
    S, T = tokens.shape
    d = table.shape[1]
    ids = tokens.astype(np.int64)
    rows = np.where((ids >= 0)[:, :, None], table[np.maximum(ids, 0)], 0.0)
    x = rows * np.sqrt(d) + sinusoid_positions(T, d)[None, :, :]
    return x.reshape(S * T, d)


def embed_backward(tokens, table_shape, dy):
    """Gradient of the table: every occurrence of a token adds sqrt(d) times its row of dy (padding adds nothing)."""
    d = table_shape[1]
    dw = np.zeros(table_shape)
    ids = tokens.astype(np.int64).reshape(-1)
    keep = ids >= 0
    np.add.at(dw, ids[keep], dy.reshape(-1, d)[keep] * np.sqrt(d))
    return dw


def sentence_lengths(tokens):
    """Tokens of each sentence that are not padding (negative ids; padding follows the tokens), at least 1."""
    return np.maximum((np.asarray(tokens) >= 0).sum(axis=1), 1)


def attention_forward(q, k, v, S, heads, causal, klen=None):
    """Scaled dot-product attention with several heads.  q [S*Tq, d], k, v [S*Tk, d] (sentence-major rows);
    head h owns columns h*dh .. (h+1)*dh.  P = softmax(Q K^T / sqrt(dh)) over the keys of the same sentence
    (causal: keys at positions <= the query's only; klen [S]: only the first klen[s] keys of sentence s, the rest
    is padding), output P V, heads side by side.  Returns (out, P)."""
    d = q.shape[1]
    dh = d // heads
    Tq, Tk = q.shape[0] // S, k.shape[0] // S
    Q = q.reshape(S, Tq, heads, dh).transpose(0, 2, 1, 3)
    K = k.reshape(S, Tk, heads, dh).transpose(0, 2, 1, 3)
    V = v.reshape(S, Tk, heads, dh).transpose(0, 2, 1, 3)
    s = np.einsum("shid,shjd->shij", Q, K) / np.sqrt(dh)
    if causal:
        s = np.where(np.arange(Tk)[None, :] <= np.arange(Tq)[:, None], s, -np.inf)
    if klen is not None:
        s = np.where(np.arange(Tk)[None, None, None, :] < np.asarray(klen).reshape(S, 1, 1, 1), s, -np.inf)
    s = s - s.max(axis=-1, keepdims=True)
    e = np.exp(s)
    P = e / e.sum(axis=-1, keepdims=True)
    out = np.einsum("shij,shjd->shid", P, V).transpose(0, 2, 1, 3).reshape(S * Tq, d)
    return out, P


def attention_backward(q, k, v, P, dout, S, heads):
    """Returns (dq, dk, dv).  dV = P^T dO, dP = dO V^T, dS = P (dP - rowsum(dP P)), dQ = dS K / sqrt(dh),
    dK = dS^T Q / sqrt(dh) (masked entries have P = 0 and drop out by themselves)."""
    d = q.shape[1]
    dh = d // heads
    Tq, Tk = q.shape[0] // S, k.shape[0] // S
    Q = q.reshape(S, Tq, heads, dh).transpose(0, 2, 1, 3)
    K = k.reshape(S, Tk, heads, dh).transpose(0, 2, 1, 3)
    V = v.reshape(S, Tk, heads, dh).transpose(0, 2, 1, 3)
    dO = dout.reshape(S, Tq, heads, dh).transpose(0, 2, 1, 3)
    dV = np.einsum("shij,shid->shjd", P, dO)
    dP = np.einsum("shid,shjd->shij", dO, V)
    dS = P * (dP - (dP * P).sum(axis=-1, keepdims=True))
    dQ = np.einsum("shij,shjd->shid", dS, K) / np.sqrt(dh)
    dK = np.einsum("shij,shid->shjd", dS, Q) / np.sqrt(dh)
    back = lambda a, T: a.transpose(0, 2, 1, 3).reshape(S * T, d)
    return back(dQ, Tq), back(dK, Tk), back(dV, Tk)
