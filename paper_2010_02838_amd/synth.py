"""Seeded synthetic inputs: weights, images, labels, logits.

This module only draws random numbers and rounds them; it contains none of the
training step's arithmetic, so both the GPU library's callers and the CPU test
oracle may be fed from it.  Everything comes from NumPy's PCG64 generator.

Recipes (stand-ins for the image and translation datasets of the paper's
experiments, whose shapes they keep: 32x32x3 / 10 classes, 224x224x3 / 1000
classes, 32K-symbol vocabulary):
  images   N(0,1) float32, NHWC
  labels   uniform integer class ids
  weights  He initialisation: N(0, 2/fan_in) for convolution and linear
           weights (fan_in = Cin*kh*kw or in_features), BatchNorm scale 1,
           BatchNorm shift and biases 0; `jitter` perturbs the scale/shift/bias
           tensors so that tests exercise them
  logits   N(0, sigma^2) float32
  sentence pairs  lengths uniform in [16, 128], token ids uniform, drawn until a
           batch holds about 8192 target tokens, padded with a negative id
"""
import numpy as np


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def bf16_bits(x):
    """float32 array -> uint16 array of bfloat16 bit patterns, round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = ((u >> 16) & 1) + 0x7FFF
    return ((u + r) >> 16).astype(np.uint16)


def bf16_to_f32(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def round_bf16(x):
    """Round a float32 array to the nearest bfloat16 value, returned as float32."""
    return bf16_to_f32(bf16_bits(x)).reshape(np.shape(x))


def round_bf16_f64(x):
    """Round a float64 array to the nearest bfloat16 value, returned as float64."""
    return round_bf16(np.asarray(x, dtype=np.float32)).astype(np.float64)


def he_init(param_table, seed, jitter=0.0):
    """param_table: ordered (name, shape, kind, fan_in); returns the flat float32 vector."""
    rng = _rng(seed)
    parts = []
    for _, shape, kind, fan_in in param_table:
        n = int(np.prod(shape))
        if kind in ("conv_w", "linear_w"):
            a = rng.standard_normal(n) * np.sqrt(2.0 / fan_in)
        elif kind == "embed_w":     # rows of variance 1/d: times sqrt(d) they match the position signal's scale
            a = rng.standard_normal(n) / np.sqrt(fan_in)
        elif kind == "bn_gamma":
            a = 1.0 + jitter * rng.standard_normal(n)
        else:
            a = jitter * rng.standard_normal(n)
        parts.append(a.astype(np.float32))
    return np.concatenate(parts)


def images(batch, h, w, c, seed):
    return _rng(seed).standard_normal((batch, h, w, c)).astype(np.float32)


def tokens(sentences, length, vocab, seed):
    """Uniform token ids, int32 [sentences, length] (stand-in for byte-pair encoded text)."""
    return _rng(seed).integers(0, vocab, size=(sentences, length)).astype(np.int32)


def sentence_pairs(min_target_tokens, lo, hi, vocab, seed, pad=-1):
    """A translation batch "of about min_target_tokens target tokens": sentence pairs with independent source and
    target lengths uniform in [lo, hi] are drawn until the target lengths add up to at least min_target_tokens, then
    padded to hi + hi columns with `pad` (a negative id).  Returns (x, y, src_len, tgt_len): x int32
    [sentences, 2 * hi] token ids (source part, then target part, each padded at its end), y int32
    [sentences * hi] one label per target position, `pad` on the padded ones."""
    rng = _rng(seed)
    src, tgt = [], []
    while sum(tgt) < min_target_tokens:
        src.append(int(rng.integers(lo, hi + 1)))
        tgt.append(int(rng.integers(lo, hi + 1)))
    S = len(src)
    x = rng.integers(0, vocab, size=(S, 2 * hi)).astype(np.int32)
    y = rng.integers(0, vocab, size=(S, hi)).astype(np.int32)
    for i in range(S):
        x[i, src[i]:hi] = pad
        x[i, hi + tgt[i]:] = pad
        y[i, tgt[i]:] = pad
    return x, y.reshape(-1), np.array(src), np.array(tgt)


def pack_sentences(x, y, src_len, rows_src=None, rows_tgt=None, multiple=128):
    """A padded batch of sentence pairs in packed form (layout only, no arithmetic).  x: int32 [S, src_len + T] token
    ids, every part padded at its end with negative ids; y: int32 [S * T] labels.  Returns (xp, yp, src_map, tgt_map):
    xp int32 [2, rows_src + rows_tgt]: row 0 the real tokens of all sentences one after the other (source stream,
    then target stream; negative ids in the rows behind the last sentence), row 1 every token's position inside its
    sentence; yp int32 [rows_tgt] the labels of the target rows (-1 behind the last sentence); src_map / tgt_map: for every
    used row of a stream its (sentence, position).  A part's length is the number of ids in front of its first negative
    one (at least one token).  rows_src / rows_tgt default to the token counts rounded up to `multiple`."""
    S, T = x.shape[0], x.shape[1] - src_len
    y = np.asarray(y).reshape(S, T)

    def length(row):
        neg = np.nonzero(row < 0)[0]
        return max(1, int(neg[0]) if len(neg) else len(row))

    ls = [length(x[i, :src_len]) for i in range(S)]
    lt = [length(x[i, src_len:]) for i in range(S)]
    up = lambda n: -(-n // multiple) * multiple
    rows_src = up(sum(ls)) if rows_src is None else rows_src
    rows_tgt = up(sum(lt)) if rows_tgt is None else rows_tgt
    assert sum(ls) <= rows_src and sum(lt) <= rows_tgt
    xp = np.full((2, rows_src + rows_tgt), -1, dtype=np.int32)
    xp[1] = 0
    yp = np.full(rows_tgt, -1, dtype=np.int32)
    src_map, tgt_map, rs, rt = [], [], 0, rows_src
    for i in range(S):
        xp[0, rs:rs + ls[i]] = x[i, :ls[i]]
        xp[1, rs:rs + ls[i]] = np.arange(ls[i])
        src_map += [(i, t) for t in range(ls[i])]
        rs += ls[i]
        xp[0, rt:rt + lt[i]] = x[i, src_len:src_len + lt[i]]
        xp[1, rt:rt + lt[i]] = np.arange(lt[i])
        yp[rt - rows_src:rt - rows_src + lt[i]] = y[i, :lt[i]]
        tgt_map += [(i, t) for t in range(lt[i])]
        rt += lt[i]
    return xp, yp, np.array(src_map), np.array(tgt_map)


def labels(n, classes, seed):
    return _rng(seed).integers(0, classes, size=n).astype(np.int32)


def logits(rows, cols, sigma, seed):
    return (_rng(seed).standard_normal((rows, cols), dtype=np.float32) * np.float32(sigma))
