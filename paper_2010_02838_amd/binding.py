"""Thin ctypes binding of libcodistill.so: argument marshalling only.

Every step of the training step runs in the library's HIP kernels; PyTorch is
used here for device memory (tensors) and the current stream, nothing else.
There is no fallback: if the shared library is missing, importing this module
raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcodistill.so")

CD_OK, CD_ERR_INVALID_ARG, CD_ERR_UNSUPPORTED, CD_ERR_WORKSPACE_TOO_SMALL, CD_ERR_HIP = 0, -1, -2, -3, -4
CD_F32, CD_BF16 = 0, 1
CD_DIST_MSE_LOGITS, CD_DIST_KL, CD_DIST_MSE_CENTERED = 0, 1, 2
CD_MEAN_ALL, CD_MEAN_ROWS = 0, 1
CD_BN_BATCH_STATS, CD_BN_RUNNING = 0, 1
CD_ARCH_TINY_CNN, CD_ARCH_RESNET_BASIC, CD_ARCH_RESNET_BOTTLENECK, CD_ARCH_TRANSFORMER_HEAD = 0, 1, 2, 3
CD_ARCH_TRANSFORMER = 4
CD_ARCH_RESNET_BASIC_IMAGENET = 5
CD_ARCH_RESNEXT = 6
CD_ARCH_WIDE_RESNET_SPLIT = 7
CD_MAX_STAGES, CD_NAME_LEN, CD_LOSS_MAX_PEERS = 4, 48, 8
KERNEL_CLASSES = ["conv_fprop", "conv_dgrad", "conv_wgrad", "norm", "glue", "linear", "loss", "sgd", "conv_fprop_narrow",
                  "bn_apply", "conv_fprop_wide", "attention"]
PARAM_KINDS = ["conv_w", "bias", "bn_gamma", "bn_beta", "linear_w", "embed_w"]


class ArchDesc(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("classes", ctypes.c_int32), ("in_h", ctypes.c_int32),
                ("in_w", ctypes.c_int32), ("n_stages", ctypes.c_int32),
                ("widths", ctypes.c_int32 * CD_MAX_STAGES), ("blocks", ctypes.c_int32 * CD_MAX_STAGES),
                ("stem_width", ctypes.c_int32), ("groups", ctypes.c_int32),
                ("out_widths", ctypes.c_int32 * CD_MAX_STAGES), ("n_splits", ctypes.c_int32), ("split", ctypes.c_int32),
                ("max_sentences", ctypes.c_int32), ("max_sentence_len", ctypes.c_int32)]


class TensorInfo(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char * CD_NAME_LEN), ("kind", ctypes.c_int32), ("ndim", ctypes.c_int32),
                ("shape", ctypes.c_int64 * 4), ("offset", ctypes.c_int64), ("size", ctypes.c_int64),
                ("fan_in", ctypes.c_int64), ("frozen", ctypes.c_int32)]


class OpInfo(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("x", ctypes.c_int32), ("y", ctypes.c_int32), ("res", ctypes.c_int32),
                ("relu", ctypes.c_int32), ("param_w", ctypes.c_int32), ("param_b", ctypes.c_int32),
                ("k", ctypes.c_int32), ("stride", ctypes.c_int32), ("pad", ctypes.c_int32),
                ("stats_offset", ctypes.c_int64), ("res_grad", ctypes.c_int32), ("k_col", ctypes.c_int32), ("v_col", ctypes.c_int32),
                ("fused_pool", ctypes.c_int32), ("key_tok0", ctypes.c_int32)]


class ActInfo(ctypes.Structure):
    _fields_ = [("h", ctypes.c_int32), ("w", ctypes.c_int32), ("c", ctypes.c_int32), ("is_f32", ctypes.c_int32),
                ("act_offset", ctypes.c_int64), ("grad_offset", ctypes.c_int64)]


class LossCfg(ctypes.Structure):
    _fields_ = [("alpha", ctypes.c_float), ("label_smoothing", ctypes.c_float), ("dist_kind", ctypes.c_int32),
                ("mse_reduction", ctypes.c_int32), ("ignore_index", ctypes.c_int32), ("n_peers", ctypes.c_int32),
                ("temperature", ctypes.c_float)]


if not os.path.exists(LIB_PATH):
    raise ImportError("libcodistill.so is not built: run `python -m paper_2010_02838_amd.build` "
                      "(or __graft_entry__.build()) first; there is no fallback path")
lib = ctypes.CDLL(LIB_PATH)

_vp, _i64, _i32, _f32, _sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
_SIGS = {
    "codistill_arch_preset": [_i32, ctypes.POINTER(ArchDesc)],
    "codistill_model_create": [ctypes.POINTER(ArchDesc), _i32, ctypes.POINTER(_vp)],
    "codistill_param_count": [_vp, ctypes.POINTER(_i64), ctypes.POINTER(_i64)],
    "codistill_param_info": [_vp, _i64, ctypes.POINTER(TensorInfo)],
    "codistill_workspace_bytes": [_vp, _i64, _i32, ctypes.POINTER(_sz)],
    "codistill_bn_running_elements": [_vp, ctypes.POINTER(_i64)],
    "codistill_graph_size": [_vp, ctypes.POINTER(_i64), ctypes.POINTER(_i64)],
    "codistill_op_info": [_vp, _i64, _i64, ctypes.POINTER(OpInfo)],
    "codistill_tensor_info": [_vp, _i64, _i64, ctypes.POINTER(ActInfo)],
    "codistill_forward": [_vp, _vp, _vp, _i64, _i32, _i32, _vp, _vp, _sz, _vp, _vp],
    "codistill_loss_scratch_bytes": [_i64, _i64, ctypes.POINTER(_sz)],
    "codistill_loss_grad": [_vp, ctypes.POINTER(_vp), _vp, _i64, _i64, ctypes.POINTER(LossCfg), _vp, _vp, _vp, _sz, _vp],
    "codistill_loss_grad_static": [_vp, ctypes.POINTER(_vp), _vp, _i64, _i64, ctypes.POINTER(LossCfg), _vp, _vp, _vp],
    "codistill_backward": [_vp, _vp, _vp, _i64, _vp, _sz, _vp, _vp, _vp],
    "codistill_sgd_step": [_vp, _vp, _vp, _vp, _i64, _f32, _f32, _f32, _i32, _vp],
    "codistill_adam_step": [_vp, _vp, _vp, _vp, _vp, _i64, _f32, _f32, _f32, _f32, _f32, _i64, _vp],
    "codistill_profile_enable": [_i32],
    "codistill_profile_collect": [],
    "codistill_profile_get": [_i32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(_i64),
                              ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)],
    "codistill_profile_reset": [],
    "codistill_profile_event_overhead": [ctypes.POINTER(ctypes.c_double), _vp],
}
for _n, _a in _SIGS.items():
    getattr(lib, _n).argtypes = _a
    getattr(lib, _n).restype = ctypes.c_int
lib.codistill_model_destroy.argtypes = [_vp]
lib.codistill_model_destroy.restype = None
lib.codistill_last_error.restype = ctypes.c_char_p
lib.codistill_version.restype = ctypes.c_char_p
EXPORTED = list(_SIGS) + ["codistill_model_destroy", "codistill_last_error", "codistill_version"]


class CodistillError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("codistill error %d: %s" % (code, msg))
        self.code = code


def _check(rc):
    if rc != CD_OK:
        raise CodistillError(rc, lib.codistill_last_error().decode())


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def arch_preset(kind, **overrides):
    a = ArchDesc()
    _check(lib.codistill_arch_preset(kind, ctypes.byref(a)))
    for k, v in overrides.items():
        if k in ("widths", "blocks", "out_widths"):
            for i, x in enumerate(v):
                getattr(a, k)[i] = x
            if k == "widths" and a.kind != CD_ARCH_TINY_CNN:
                a.n_stages = len(v)
        else:
            setattr(a, k, v)
    return a


class Model:
    """Host-side model description (op list, parameter table)."""

    def __init__(self, arch, dtype):
        self.arch, self.dtype = arch, dtype
        self._h = _vp()
        _check(lib.codistill_model_create(ctypes.byref(arch), dtype, ctypes.byref(self._h)))
        nt, ne = _i64(), _i64()
        _check(lib.codistill_param_count(self._h, ctypes.byref(nt), ctypes.byref(ne)))
        self.n_tensors, self.n_elements = nt.value, ne.value
        self.params = []
        for i in range(self.n_tensors):
            ti = TensorInfo()
            _check(lib.codistill_param_info(self._h, i, ctypes.byref(ti)))
            self.params.append(dict(name=ti.name.decode(), kind=PARAM_KINDS[ti.kind], shape=tuple(ti.shape[:ti.ndim]),
                                    offset=ti.offset, size=ti.size, fan_in=ti.fan_in, frozen=bool(ti.frozen)))
        # frozen tensors (a frozen front end) come first: the update covers the flat buffers from here on
        self.trainable_offset = min([p["offset"] for p in self.params if not p["frozen"]] + [self.n_elements])
        self.classes = arch.classes
        # rows of logits per element of the batch: target tokens per sentence for the Transformer, else 1
        self.rows_per_sample = arch.in_w if arch.kind == CD_ARCH_TRANSFORMER else 1
        self.torch_dtype = torch.bfloat16 if dtype == CD_BF16 else torch.float32

    def __del__(self):
        if getattr(self, "_h", None) and lib is not None:   # module globals are gone at interpreter exit
            lib.codistill_model_destroy(self._h)
            self._h = None

    def param_table(self):
        """(name, shape, kind, fan_in) in declaration order, for the input generators."""
        return [(p["name"], p["shape"], p["kind"], p["fan_in"]) for p in self.params]

    def graph(self, batch):
        """(ops, tensors) as lists of dicts: the fused op list and the workspace layout for this batch."""
        no, nt = _i64(), _i64()
        _check(lib.codistill_graph_size(self._h, ctypes.byref(no), ctypes.byref(nt)))
        ops, tensors = [], []
        kinds = ["conv", "bn", "maxpool", "gap", "linear", "layernorm", "embed", "attn", "slice"]
        for i in range(no.value):
            o = OpInfo()
            _check(lib.codistill_op_info(self._h, batch, i, ctypes.byref(o)))
            d = {f: getattr(o, f) for f, _ in OpInfo._fields_}
            d["kind"] = kinds[o.kind]
            ops.append(d)
        for i in range(nt.value):
            t = ActInfo()
            _check(lib.codistill_tensor_info(self._h, batch, i, ctypes.byref(t)))
            tensors.append({f: getattr(t, f) for f, _ in ActInfo._fields_})
        return ops, tensors

    def bn_running_elements(self):
        n = _i64()
        _check(lib.codistill_bn_running_elements(self._h, ctypes.byref(n)))
        return n.value

    def workspace_bytes(self, batch, save_for_backward):
        b = _sz()
        _check(lib.codistill_workspace_bytes(self._h, batch, int(save_for_backward), ctypes.byref(b)))
        return b.value


def codistill_forward(model, params, x, workspace, logits_out, save_for_backward, bn_mode=CD_BN_BATCH_STATS,
                      bn_running=None):
    """z = f_params(x).  params: flat tensor in the model dtype; x: [B,H,W,3]; logits_out: [B,classes] fp32."""
    batch = x.shape[0]
    _check(lib.codistill_forward(model._h, _ptr(params), _ptr(x), batch, int(save_for_backward), bn_mode, _ptr(bn_running),
                                 _ptr(workspace), workspace.numel() * workspace.element_size(), _ptr(logits_out),
                                 _stream()))


def loss_scratch_bytes(rows, cols):
    b = _sz()
    _check(lib.codistill_loss_scratch_bytes(rows, cols, ctypes.byref(b)))
    return b.value


def codistill_loss_grad(z_local, z_peers, targets, loss_out, dz_out, scratch, alpha, label_smoothing=0.0,
                        dist_kind=CD_DIST_MSE_LOGITS, mse_reduction=CD_MEAN_ALL, ignore_index=-1, temperature=1.0):
    """loss_out: float32[4] device tensor (total, task, distill, status bits)."""
    rows, cols = z_local.shape
    peers = list(z_peers) if z_peers is not None else []
    cfg = LossCfg(alpha, label_smoothing, dist_kind, mse_reduction, ignore_index, len(peers), temperature)
    arr = (_vp * max(len(peers), 1))(*[p.data_ptr() for p in peers])
    _check(lib.codistill_loss_grad(_ptr(z_local), arr if peers else None, _ptr(targets), rows, cols,
                                   ctypes.byref(cfg), _ptr(loss_out), _ptr(dz_out), _ptr(scratch),
                                   scratch.numel() * scratch.element_size(), _stream()))


def codistill_loss_grad_static(z_local, z_peers, targets, loss_out, dz_out, alpha, label_smoothing=0.0,
                               dist_kind=CD_DIST_MSE_LOGITS, mse_reduction=CD_MEAN_ALL, ignore_index=-1, temperature=1.0):
    """codistill_loss_grad without a scratch argument (the library's own fixed device array; rows <= 65536)."""
    rows, cols = z_local.shape
    peers = list(z_peers) if z_peers is not None else []
    cfg = LossCfg(alpha, label_smoothing, dist_kind, mse_reduction, ignore_index, len(peers), temperature)
    arr = (_vp * max(len(peers), 1))(*[p.data_ptr() for p in peers])
    _check(lib.codistill_loss_grad_static(_ptr(z_local), arr if peers else None, _ptr(targets), rows, cols,
                                          ctypes.byref(cfg), _ptr(loss_out), _ptr(dz_out), _stream()))


def codistill_backward(model, params, x, workspace, dlogits, grads_out):
    _check(lib.codistill_backward(model._h, _ptr(params), _ptr(x), x.shape[0], _ptr(workspace),
                                  workspace.numel() * workspace.element_size(), _ptr(dlogits), _ptr(grads_out),
                                  _stream()))


def codistill_sgd_step(master_w, momentum_v, grad, lowp_w_out, lr, momentum, weight_decay=0.0, nesterov=False):
    _check(lib.codistill_sgd_step(_ptr(master_w), _ptr(momentum_v), _ptr(grad), _ptr(lowp_w_out), master_w.numel(),
                                  lr, momentum, weight_decay, int(nesterov), _stream()))


def codistill_adam_step(master_w, exp_avg, exp_avg_sq, grad, lowp_w_out, lr, t, beta1=0.9, beta2=0.98, eps=1e-8,
                        weight_decay=0.0):
    _check(lib.codistill_adam_step(_ptr(master_w), _ptr(exp_avg), _ptr(exp_avg_sq), _ptr(grad), _ptr(lowp_w_out),
                                   master_w.numel(), lr, beta1, beta2, eps, weight_decay, int(t), _stream()))


def profile_enable(on):
    _check(lib.codistill_profile_enable(int(on)))


def profile_reset():
    _check(lib.codistill_profile_reset())


def profile_event_overhead():
    """Microseconds that the timer's event pair adds to a launch (measured on the current stream)."""
    us = ctypes.c_double()
    _check(lib.codistill_profile_event_overhead(ctypes.byref(us), _stream()))
    return us.value


def profile_collect():
    """Returns {class: dict(ms, launches, flops, bytes)} accumulated since the last reset."""
    _check(lib.codistill_profile_collect())
    out = {}
    for i, name in enumerate(KERNEL_CLASSES):
        ms, fl, by, n = ctypes.c_double(), ctypes.c_double(), ctypes.c_double(), _i64()
        _check(lib.codistill_profile_get(i, ctypes.byref(ms), ctypes.byref(n), ctypes.byref(fl), ctypes.byref(by)))
        out[name] = dict(ms=ms.value, launches=n.value, flops=fl.value, bytes=by.value)
    return out
