"""Helpers shared by the GPU parity tests: build a case, run it through the C ABI, read tensors back."""
import numpy as np
import torch

from oracle.step import codistill_step
from paper_2010_02838_amd import synth


def rel(a, b):
    nb = np.linalg.norm(b)
    return float(np.linalg.norm(np.asarray(a, dtype=np.float64) - b) / (nb if nb > 0 else 1.0))


def norm_err(a, b):
    nb = np.linalg.norm(b)
    return float(abs(np.linalg.norm(np.asarray(a, dtype=np.float64)) - nb) / nb) if nb > 0 else float(np.linalg.norm(a))


def bf16_storage_points(arch):
    """Which tensors of the oracle's op list the GPU pipeline keeps in memory as bf16, as a `perturb` map of
    oracle.nets.forward (tensor id -> round to bf16): the outputs of convolutions / dense layers of the body,
    of the pools, of LayerNorm, embedding and attention, of every ReLU, and of a BatchNorm that is read as the
    shortcut operand of a residual add.  A BatchNorm followed by its ReLU (or by the add and the ReLU) is one
    kernel on the GPU, which stores only the last of those tensors; the logits stay fp32.  This is knowledge of
    the GPU pipeline and lives with the tests: the oracle only applies the map it is given."""
    readers = {}
    for o in arch.ops:
        for key in ("x", "a", "b", "kv"):
            if key in o:
                readers.setdefault(o[key], []).append((o["op"], key))
    points = {}
    for o in arch.ops:
        kind, y = o["op"], o["y"]
        if kind in ("conv", "relu", "maxpool", "gap", "layernorm", "embed", "attn"):
            points[y] = synth.round_bf16_f64
        elif kind == "bn" and all(r == ("add", "b") for r in readers.get(y, [])):
            points[y] = synth.round_bf16_f64
    return points


class Case:
    """Inputs of one codistillation step for an architecture (library preset kwargs + oracle arch)."""

    def __init__(self, arch_kw, ref_arch, dtype_name, batch, res, classes, jitter=0.1, v_scale=0.0, in_c=3, tokens=None,
                 ragged=False, peer=None):
        """tokens = (source length, target length): the input is int32 token ids and there is one row of logits
        (and one label) per target token; res is then unused.  ragged: the sentences get random lengths (one of them
        a single token, one the full length); the rest of each part is padding (-1) and its labels are -1 (ignored).
        peer = (library preset kwargs, oracle arch): the stale peer is a model of another architecture (same input and
        number of classes)."""
        from paper_2010_02838_amd import binding as B
        self.B = B
        self.dtype = B.CD_BF16 if dtype_name == "bf16" else B.CD_F32
        kw = dict(arch_kw)
        if tokens:
            arch = B.arch_preset(kw.pop("kind"), in_h=tokens[0], in_w=tokens[1], classes=classes, **kw)
        else:
            arch = B.arch_preset(kw.pop("kind"), in_h=res, in_w=res, classes=classes, **kw)
        self.model, self.peer = B.Model(arch, self.dtype), B.Model(arch, self.dtype)
        self.ref_arch, self.batch, self.res, self.classes = ref_arch, batch, res, classes
        self.peer_ref = None
        table = self.model.param_table()
        assert table == [(n, tuple(s), k, f) for n, s, k, f in ref_arch.params]
        ptable = table
        if peer:
            pkw = dict(peer[0])
            self.peer = B.Model(B.arch_preset(pkw.pop("kind"), in_h=res, in_w=res, classes=classes, **pkw), self.dtype)
            self.peer_ref = peer[1]
            ptable = self.peer.param_table()
            assert ptable == [(n, tuple(s), k, f) for n, s, k, f in self.peer_ref.params]
        self.th, self.thp = synth.he_init(table, 1, jitter), synth.he_init(ptable, 2, jitter)
        if tokens:
            self.x = synth.tokens(batch, tokens[0] + tokens[1], classes, seed=0)
            self.y = synth.labels(batch * tokens[1], classes, seed=3)
            self.th, self.thp = synth.round_bf16(self.th), synth.round_bf16(self.thp)
            if ragged:
                rng = np.random.default_rng(11)
                self.y = self.y.copy().reshape(batch, tokens[1])
                for part, (c0, n) in enumerate(((0, tokens[0]), (tokens[0], tokens[1]))):
                    lens = rng.integers(1, n + 1, batch)
                    lens[0], lens[-1] = (1, n) if part == 0 else (n, 1)
                    for s_, l in enumerate(lens):
                        self.x[s_, c0 + l:c0 + n] = -1
                        if part == 1:
                            self.y[s_, l:] = -1
                self.y = self.y.reshape(-1)
        else:
            self.x, self.y = synth.images(batch, res, res, in_c, seed=0), synth.labels(batch, classes, seed=3)
            if self.dtype == B.CD_BF16:   # both sides consume the same bf16-rounded weights and images
                self.th, self.thp, self.x = (synth.round_bf16(a) for a in (self.th, self.thp, self.x))
        self.v0 = None
        if v_scale:
            self.v0 = (np.random.default_rng(5).standard_normal(self.th.size) * v_scale).astype(np.float32)

    def oracle(self, alpha=1.0, lr=0.1, mu=0.9, wd=0.0, dist="mse", bf16_storage=False, label_smoothing=0.0):
        """The float64 step.  bf16_storage: the same exact arithmetic with the tensors of bf16_storage_points rounded
        to bf16 as they are produced (how far storage rounding alone moves the result on this workload)."""
        pa = self.ref_arch if self.peer_ref is None else self.peer_ref
        return codistill_step(self.ref_arch, self.th.astype(np.float64), [self.thp.astype(np.float64)],
                              self.x.astype(np.float64), self.y, alpha, lr, mu,
                              v=None if self.v0 is None else self.v0.astype(np.float64), weight_decay=wd, dist=dist,
                              label_smoothing=label_smoothing,
                              peer_archs=None if self.peer_ref is None else [self.peer_ref],
                              perturb=bf16_storage_points(self.ref_arch) if bf16_storage else None,
                              perturb_peers=[bf16_storage_points(pa)] if bf16_storage else None)

    def gpu(self, alpha=1.0, lr=0.1, mu=0.9, wd=0.0, dist="mse", label_smoothing=0.0):
        from paper_2010_02838_amd.runner import StepRunner, pack_flat, unpack_flat, to_device
        B, model = self.B, self.model
        r = StepRunner(model, [self.peer], self.batch)
        r.load(pack_flat(model, self.th), [pack_flat(self.peer, self.thp)],
               None if self.v0 is None else pack_flat(model, self.v0))
        xd = torch.from_numpy(self.x).to("cuda:0") if self.x.dtype == np.int32 else to_device(self.x, model.torch_dtype)
        yd = torch.from_numpy(self.y).to("cuda:0")
        r.step(xd, yd, alpha, lr, mu, weight_decay=wd, label_smoothing=label_smoothing,
               dist_kind={"kl": B.CD_DIST_KL, "mse": B.CD_DIST_MSE_LOGITS, "mse_centered": B.CD_DIST_MSE_CENTERED}[dist])
        torch.cuda.synchronize()
        self.last_step = dict(lr=lr, mu=mu, wd=wd)
        got = dict(logits=r.logits.cpu().numpy(), peer_logits=r.peer_logits[0].cpu().numpy(),
                   loss=r.loss.cpu().numpy()[:3].astype(np.float64), dz=r.dz.cpu().numpy(),
                   grad=unpack_flat(model, r.grads.cpu().numpy()), theta=unpack_flat(model, r.master.cpu().numpy()),
                   v=unpack_flat(model, r.momentum.cpu().numpy()))
        if r.lowp is not None:   # the bf16 shadow is the rounded image of the fp32 master weights
            bits = r.lowp.view(torch.int16).cpu().numpy().view(np.uint16)
            np.testing.assert_array_equal(bits, synth.bf16_bits(r.master.cpu().numpy()))
        self.runner = r
        return got

    def per_tensor(self, flat):
        off, out = 0, {}
        for name, shape, _, _ in self.ref_arch.params:
            n = int(np.prod(shape))
            out[name] = np.asarray(flat[off:off + n]).reshape(shape)
            off += n
        return out

    def read(self, offset, shape, f32=False):
        """A tensor out of the runner's workspace, as float64."""
        ws = self.runner.ws
        n = int(np.prod(shape))
        if f32 or self.dtype == self.B.CD_F32:
            a = ws[offset:offset + 4 * n].view(torch.float32).cpu().numpy()
        else:
            a = synth.bf16_to_f32(ws[offset:offset + 2 * n].view(torch.int16).cpu().numpy().view(np.uint16))
        return a.astype(np.float64).reshape(shape)


class PackedCase:
    """The sentences of a padded Transformer Case, given to the library in packed form (cd_arch_desc.max_sentences > 0:
    the tokens of all sentences one after the other, no padding rows).  The oracle knows padded batches only: its results
    on the padded form are the reference, and what the GPU returns per row of a stream is put back at the row's
    (sentence, position); rows that are padding in the padded form have no counterpart and are left out of every
    comparison (zeros on both sides)."""

    def __init__(self, c0, arch_kw, Ts, Tt, multiple=128, slack_sentences=3):
        B = c0.B
        self.c0, self.B, self.dtype, self.ref_arch, self.batch = c0, B, c0.dtype, c0.ref_arch, c0.batch
        self.x, self.y, self.th, self.thp, self.v0, self.classes = c0.x, c0.y, c0.th, c0.thp, c0.v0, c0.classes
        self.Ts, self.Tt = Ts, Tt
        self.xp, self.yp, self.src_map, self.tgt_map = synth.pack_sentences(c0.x, c0.y, Ts, multiple=multiple)
        self.rows_src = self.xp.shape[1] - len(self.yp)
        self.rows_tgt = len(self.yp)
        kw = dict(arch_kw)
        arch = B.arch_preset(kw.pop("kind"), in_h=self.rows_src, in_w=self.rows_tgt, classes=c0.classes,
                             max_sentences=c0.batch + slack_sentences, max_sentence_len=max(Ts, Tt), **kw)
        self.model, self.peer = B.Model(arch, self.dtype), B.Model(arch, self.dtype)
        assert self.model.param_table() == c0.model.param_table()
        self.per_tensor = c0.per_tensor

    def valid_rows(self, stream):
        """boolean [S, T]: the positions of a stream's padded form that hold a token"""
        T, mp = (self.Tt, self.tgt_map) if stream else (self.Ts, self.src_map)
        m = np.zeros((self.batch, T), dtype=bool)
        m[mp[:, 0], mp[:, 1]] = True
        return m

    def unpack(self, a, stream):
        """[rows of the stream, ...] -> [S * T, ...] with zeros where the padded form has padding"""
        T, mp = (self.Tt, self.tgt_map) if stream else (self.Ts, self.src_map)
        out = np.zeros((self.batch, T) + a.shape[1:], dtype=a.dtype)
        out[mp[:, 0], mp[:, 1]] = a[:len(mp)]
        return out.reshape((self.batch * T,) + a.shape[1:])

    def oracle(self, **kw):
        """The padded batch through the oracle; logits of padding rows zeroed (no counterpart on the GPU)."""
        r = dict(self.c0.oracle(**kw))
        keep = self.valid_rows(1).reshape(-1, 1)
        r["logits"] = r["logits"] * keep
        r["peer_logits"] = [z * keep for z in r["peer_logits"]]
        return r

    def gpu(self, alpha=1.0, lr=0.1, mu=0.9, wd=0.0, dist="mse", label_smoothing=0.0):
        from paper_2010_02838_amd.runner import StepRunner, pack_flat, unpack_flat
        B, model = self.B, self.model
        r = StepRunner(model, [self.peer], 1)
        r.load(pack_flat(model, self.th), [pack_flat(self.peer, self.thp)],
               None if self.v0 is None else pack_flat(model, self.v0))
        xd, yd = torch.from_numpy(self.xp[None]).to("cuda:0"), torch.from_numpy(self.yp).to("cuda:0")   # one batch element
        r.step(xd, yd, alpha, lr, mu, weight_decay=wd, label_smoothing=label_smoothing,
               dist_kind={"kl": B.CD_DIST_KL, "mse": B.CD_DIST_MSE_LOGITS, "mse_centered": B.CD_DIST_MSE_CENTERED}[dist])
        torch.cuda.synchronize()
        self.last_step = dict(lr=lr, mu=mu, wd=wd)
        self.runner = r
        self.raw_logits = r.logits.cpu().numpy()
        return dict(logits=self.unpack(self.raw_logits, 1), peer_logits=self.unpack(r.peer_logits[0].cpu().numpy(), 1),
                    loss=r.loss.cpu().numpy()[:3].astype(np.float64), dz=self.unpack(r.dz.cpu().numpy(), 1),
                    grad=unpack_flat(model, r.grads.cpu().numpy()), theta=unpack_flat(model, r.master.cpu().numpy()),
                    v=unpack_flat(model, r.momentum.cpu().numpy()))

    read = Case.read

    def graph(self):
        """The op list and tensor table of the packed model, re-expressed for the padded form: tensors get the padded
        sentence length as their height and the stream they belong to; token columns refer to the padded ids."""
        ops, tensors = self.model.graph(1)
        stream = {0: 0}
        for o in ops:
            if o["kind"] == "embed":
                stream[o["y"]] = 0 if o["k"] == 0 else 1
                o["k"], o["stride"] = (0, self.Ts) if o["k"] == 0 else (self.Ts, self.Tt)
            else:
                stream[o["y"]] = stream[o["x"]]
            if o["kind"] == "attn" and o["key_tok0"]:
                o["key_tok0"] = self.Ts
        for t, td in enumerate(tensors):
            td["stream"] = stream.get(t, 0)
            td["rows"] = td["h"]
            td["h"] = self.Tt if td["stream"] else self.Ts
        return ops, tensors

    def read_tensor(self, td, key, shape, f32=False):
        """A tensor of the packed model out of the workspace, in the padded form's shape."""
        a = self.read(td[key], (td["rows"],) + tuple(shape[2:]), f32)
        return self.unpack(a, td["stream"]).reshape(shape)

    def read_rows(self, td, offset, width):
        """per-row fp32 side data of a tensor's rows ([rows][width]) -> [S * T][width]"""
        return self.unpack(self.read(offset, (td["rows"], width), f32=True), td["stream"])
