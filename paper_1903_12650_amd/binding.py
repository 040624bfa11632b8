"""ctypes binding of librn50_hip.so.  Same names as the C ABI (include/rn50_hip.h).

Tensors are torch CUDA (ROCm) tensors used purely as device memory; work is
enqueued on torch's current stream.  There is no CPU fallback: importing this
module fails loudly when the library has not been built.
"""
import ctypes
import os

import torch

__all__ = ["F32", "BF16", "Rn50Error", "lib_path", "conv_fwd", "conv_dgrad", "conv_wgrad", "bn_relu_fwd",
           "bn_relu_bwd", "maxpool_fwd", "maxpool_bwd", "avgpool_fwd", "avgpool_bwd", "fc_fwd", "fc_bwd",
           "xent_fwd_bwd", "lars_update", "lars_update_noalloc", "LarsTable", "profile_begin", "profile_pause", "profile_end", "profile_end_timeline", "profile_tags", "ResnetPlan", "resnet_step", "ConvDesc", "BnDesc",
           "conv_fwd_workspace_bytes", "conv_dgrad_workspace_bytes", "conv_wgrad_workspace_bytes",
           "bn_relu_fwd_workspace_bytes", "bn_relu_bwd_workspace_bytes", "raw", "conv_bn_sums_bytes",
           "conv_fwd_bn_sums", "conv_fwd_bn_in", "conv_wgrad_bn_in", "bn_relu_fwd_from_sums", "relu_mask_like", "conv_dgrad_bn_sums", "bn_relu_bwd_from_sums",
           "LrSchedule", "TrainState", "resnet_train_step", "DECAY_NONE", "DECAY_STEP", "DECAY_POLY", "DECAY_LINEAR",
           "DECAY_TABLE", "resnet_init_params", "bn_relu_infer", "top1_accuracy", "resnet_eval"]

F32, BF16 = 0, 1
_HERE = os.path.dirname(os.path.abspath(__file__))


def lib_path():
    return os.path.join(_HERE, "librn50_hip.so")


if not os.path.exists(lib_path()):
    raise ImportError("librn50_hip.so is not built: run `python paper_1903_12650_amd/build.py` (or "
                      "`python -c 'import __graft_entry__ as g; g.build()'`) first; there is no fallback path")
raw = ctypes.CDLL(lib_path())


class Rn50Error(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"rn50 error {code}: {text}")
        self.code = code


class ConvDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in ("N", "H", "W", "Cin", "Cout", "R", "S", "stride", "pad", "dtype")]


class BnDesc(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int), ("H", ctypes.c_int), ("W", ctypes.c_int), ("C", ctypes.c_int),
                ("eps", ctypes.c_float), ("dtype", ctypes.c_int), ("mode", ctypes.c_int)]


class LarsTensor(ctypes.Structure):
    _fields_ = [("w", ctypes.c_void_p), ("g", ctypes.c_void_p), ("v", ctypes.c_void_p), ("w_lowp", ctypes.c_void_p),
                ("n", ctypes.c_int64), ("weight_decay", ctypes.c_float), ("apply_trust", ctypes.c_int)]


class LarsDesc(ctypes.Structure):
    _fields_ = [("num_tensors", ctypes.c_int), ("eta", ctypes.c_float), ("momentum", ctypes.c_float),
                ("lr", ctypes.c_float), ("eps", ctypes.c_float), ("grad_dtype", ctypes.c_int)]


class StepConfig(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int), ("image_hw", ctypes.c_int), ("classes", ctypes.c_int), ("dtype", ctypes.c_int),
                ("widths", ctypes.c_int * 4), ("blocks", ctypes.c_int * 4), ("stem", ctypes.c_int),
                ("expansion", ctypes.c_int), ("bn_eps", ctypes.c_float), ("label_smoothing", ctypes.c_float),
                ("grad_scale", ctypes.c_float), ("eta", ctypes.c_float), ("momentum", ctypes.c_float),
                ("weight_decay", ctypes.c_float), ("lars_eps", ctypes.c_float)]


raw.rn50_last_error.restype = ctypes.c_char_p
raw.rn50_profile_tag.restype = ctypes.c_char_p
for _n in ("conv_fwd_workspace_bytes", "conv_dgrad_workspace_bytes", "conv_wgrad_workspace_bytes",
           "bn_relu_fwd_workspace_bytes", "bn_relu_bwd_workspace_bytes", "lars_update_workspace_bytes",
           "resnet_plan_workspace_bytes", "conv_bn_sums_bytes", "resnet_train_state_bytes",
           "bn_relu_infer_workspace_bytes"):
    if hasattr(raw, _n):
        getattr(raw, _n).restype = ctypes.c_size_t
for _n in ("resnet_plan_tensor_shape", "resnet_plan_tensor_offset", "resnet_plan_arena_elems", "resnet_plan_bn_channels",
           "resnet_plan_bn_offset", "lars_update_noalloc_max_chunks"):
    if hasattr(raw, _n):
        getattr(raw, _n).restype = ctypes.c_int64


def _check(rc):
    if rc != 0:
        raise Rn50Error(rc, raw.rn50_last_error().decode())


def _ptr(t):
    if t is None:
        return ctypes.c_void_p(0)
    assert t.is_cuda and t.is_contiguous(), "device, contiguous tensors only"
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dt(t):
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ws(nbytes, device):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


# ---------------------------------------------------------------- convolution
def _conv_desc(x_shape, w_shape, stride, pad, dtype):
    N, H, W, C = x_shape
    K, R, S, C2 = w_shape
    assert C == C2
    return ConvDesc(N, H, W, C, K, R, S, stride, pad, dtype)


def conv_fwd_workspace_bytes(desc):
    return raw.conv_fwd_workspace_bytes(ctypes.byref(desc))


def conv_dgrad_workspace_bytes(desc):
    return raw.conv_dgrad_workspace_bytes(ctypes.byref(desc))


def conv_wgrad_workspace_bytes(desc):
    return raw.conv_wgrad_workspace_bytes(ctypes.byref(desc))


def conv_fwd(x, w, stride, pad, y=None, workspace=None):
    d = _conv_desc(x.shape, w.shape, stride, pad, _dt(x))
    P = (d.H + 2 * pad - d.R) // stride + 1
    Q = (d.W + 2 * pad - d.S) // stride + 1
    if y is None:
        y = torch.empty((d.N, P, Q, d.Cout), dtype=x.dtype, device=x.device)
    if workspace is None:
        workspace = _ws(conv_fwd_workspace_bytes(d), x.device)
    _check(raw.conv_fwd(ctypes.byref(d), _ptr(x), _ptr(w), _ptr(y), _ptr(workspace),
                        ctypes.c_size_t(workspace.numel()), _stream()))
    return y


def conv_dgrad(dy, w, x_shape, stride, pad, dx=None, workspace=None):
    d = _conv_desc(x_shape, w.shape, stride, pad, _dt(dy))
    if dx is None:
        dx = torch.empty(tuple(x_shape), dtype=dy.dtype, device=dy.device)
    if workspace is None:
        workspace = _ws(conv_dgrad_workspace_bytes(d), dy.device)
    _check(raw.conv_dgrad(ctypes.byref(d), _ptr(dy), _ptr(w), _ptr(dx), _ptr(workspace),
                          ctypes.c_size_t(workspace.numel()), _stream()))
    return dx


def conv_wgrad(x, dy, w_shape, stride, pad, dw=None, workspace=None):
    d = _conv_desc(x.shape, w_shape, stride, pad, _dt(x))
    if dw is None:
        dw = torch.empty(tuple(w_shape), dtype=torch.float32, device=x.device)
    if workspace is None:
        workspace = _ws(conv_wgrad_workspace_bytes(d), x.device)
    _check(raw.conv_wgrad(ctypes.byref(d), _ptr(x), _ptr(dy), _ptr(dw), _ptr(workspace),
                          ctypes.c_size_t(workspace.numel()), _stream()))
    return dw


# ----------------------------------------------------------------- batch norm
def _bn_desc(x, eps, mode):
    C = x.shape[-1]
    m = x.numel() // C
    return BnDesc(1, 1, m, C, eps, _dt(x), mode) if x.dim() != 4 else BnDesc(x.shape[0], x.shape[1], x.shape[2], C, eps, _dt(x), mode)


def bn_relu_fwd_workspace_bytes(desc):
    return raw.bn_relu_fwd_workspace_bytes(ctypes.byref(desc))


def bn_relu_bwd_workspace_bytes(desc):
    return raw.bn_relu_bwd_workspace_bytes(ctypes.byref(desc))


def relu_mask_like(x):
    V = 8 if x.dtype == torch.bfloat16 else 4
    return torch.empty(x.numel() // V, dtype=torch.uint8, device=x.device)


def bn_relu_fwd(x, gamma, beta, residual=None, eps=1e-5, mode=1, running_mean=None, running_var=None,
                momentum=0.9, workspace=None, relu_mask=None):
    """Returns y, save_mean, save_rstd.  relu_mask: optional uint8 tensor (see relu_mask_like) to fill."""
    d = _bn_desc(x, eps, mode)
    y = torch.empty_like(x)
    mean = torch.empty(d.C, dtype=torch.float32, device=x.device)
    rstd = torch.empty(d.C, dtype=torch.float32, device=x.device)
    if workspace is None:
        workspace = _ws(bn_relu_fwd_workspace_bytes(d), x.device)
    _check(raw.bn_relu_fwd(ctypes.byref(d), _ptr(x), _ptr(gamma), _ptr(beta), _ptr(residual), _ptr(y),
                           _ptr(relu_mask), _ptr(mean),
                           _ptr(rstd), _ptr(running_mean), _ptr(running_var), ctypes.c_float(momentum),
                           _ptr(workspace), ctypes.c_size_t(workspace.numel()), _stream()))
    return y, mean, rstd


def bn_relu_bwd(dz, x, z, gamma, mean, rstd, mode=1, beta=None, dz2=None, eps=1e-5, workspace=None, relu_mask=None):
    """Returns dx, dresidual (None unless mode 2), dgamma, dbeta."""
    d = _bn_desc(x, eps, mode)
    dx = torch.empty_like(x)
    dres = torch.empty_like(x) if mode == 2 else None
    dgamma = torch.empty(d.C, dtype=torch.float32, device=x.device)
    dbeta = torch.empty(d.C, dtype=torch.float32, device=x.device)
    if workspace is None:
        workspace = _ws(bn_relu_bwd_workspace_bytes(d), x.device)
    _check(raw.bn_relu_bwd(ctypes.byref(d), _ptr(dz), _ptr(dz2), _ptr(x), _ptr(z), _ptr(relu_mask), _ptr(gamma),
                           _ptr(beta),
                           _ptr(mean), _ptr(rstd), _ptr(dx), _ptr(dres), _ptr(dgamma), _ptr(dbeta),
                           _ptr(workspace), ctypes.c_size_t(workspace.numel()), _stream()))
    return dx, dres, dgamma, dbeta


# ------------------------------------- convolution + batch norm with fused sums
def conv_bn_sums_bytes(desc):
    return raw.conv_bn_sums_bytes(ctypes.byref(desc))


def conv_fwd_bn_sums(x, w, stride, pad, y=None, workspace=None, sums=None):
    """Returns y and the handle (producer descriptor, sums buffer) bn_relu_fwd_from_sums takes."""
    d = _conv_desc(x.shape, w.shape, stride, pad, _dt(x))
    P = (d.H + 2 * pad - d.R) // stride + 1
    Q = (d.W + 2 * pad - d.S) // stride + 1
    if y is None:
        y = torch.empty((d.N, P, Q, d.Cout), dtype=x.dtype, device=x.device)
    if workspace is None:
        workspace = _ws(conv_fwd_workspace_bytes(d), x.device)
    if sums is None:
        sums = _ws(conv_bn_sums_bytes(d), x.device)
    _check(raw.conv_fwd_bn_sums(ctypes.byref(d), _ptr(x), _ptr(w), _ptr(y), _ptr(sums), ctypes.c_size_t(sums.numel()),
                                _ptr(workspace), ctypes.c_size_t(workspace.numel()), _stream()))
    return y, (d, sums)


def bn_relu_fwd_from_sums(x, handle, gamma, beta, residual=None, eps=1e-5, mode=1, running_mean=None,
                          running_var=None, momentum=0.9, relu_mask=None):
    """Returns y, save_mean, save_rstd."""
    producer, sums = handle
    d = _bn_desc(x, eps, mode)
    y = torch.empty_like(x)
    mean = torch.empty(d.C, dtype=torch.float32, device=x.device)
    rstd = torch.empty(d.C, dtype=torch.float32, device=x.device)
    _check(raw.bn_relu_fwd_from_sums(ctypes.byref(d), ctypes.byref(producer), _ptr(x), _ptr(sums), _ptr(gamma),
                                     _ptr(beta), _ptr(residual), _ptr(y), _ptr(relu_mask), _ptr(mean), _ptr(rstd),
                                     _ptr(running_mean),
                                     _ptr(running_var), ctypes.c_float(momentum), _stream()))
    return y, mean, rstd


def conv_dgrad_bn_sums(dy, w, x_shape, stride, pad, bn_x, gamma, beta, mean, rstd, dx=None, workspace=None,
                       sums=None, addend=None, relu_mask=None, addend_mask=None):
    """Returns dx (= data gradient + addend [under addend_mask]) and the handle bn_relu_bwd_from_sums takes."""
    d = _conv_desc(x_shape, w.shape, stride, pad, _dt(dy))
    if dx is None:
        dx = torch.empty(tuple(x_shape), dtype=dy.dtype, device=dy.device)
    if workspace is None:
        workspace = _ws(conv_dgrad_workspace_bytes(d), dy.device)
    if sums is None:
        sums = _ws(conv_bn_sums_bytes(d), dy.device)
    _check(raw.conv_dgrad_bn_sums(ctypes.byref(d), _ptr(dy), _ptr(w), _ptr(dx), _ptr(addend), _ptr(addend_mask), _ptr(bn_x),
                                  _ptr(relu_mask), _ptr(gamma), _ptr(beta), _ptr(mean), _ptr(rstd), _ptr(sums),
                                  ctypes.c_size_t(sums.numel()), _ptr(workspace), ctypes.c_size_t(workspace.numel()),
                                  _stream()))
    return dx, (d, sums)


def conv_fwd_bn_in(x, in_gamma, in_beta, in_mean, in_rstd, w, with_sums=False):
    """1x1 convolution of relu(bn(x)) without storing it.  Returns y (and the sums handle with with_sums)."""
    d = _conv_desc(x.shape, w.shape, 1, 0, _dt(x))
    N, H, W_, _ = x.shape
    y = torch.empty((N, H, W_, w.shape[0]), dtype=x.dtype, device=x.device)
    sums = _ws(conv_bn_sums_bytes(d), x.device) if with_sums else None
    _check(raw.conv_fwd_bn_in(ctypes.byref(d), _ptr(x), _ptr(in_gamma), _ptr(in_beta), _ptr(in_mean), _ptr(in_rstd),
                              _ptr(w), _ptr(y), _ptr(sums), ctypes.c_size_t(sums.numel() if with_sums else 0), _stream()))
    return (y, (d, sums)) if with_sums else y


def conv_wgrad_bn_in(x, in_gamma, in_beta, in_mean, in_rstd, dy, w_shape, workspace=None):
    """Weight gradient of a 1x1 convolution whose input is relu(bn(x)), without storing that input."""
    d = _conv_desc(x.shape, w_shape, 1, 0, _dt(x))
    dw = torch.empty(tuple(w_shape), dtype=torch.float32, device=x.device)
    if workspace is None:
        workspace = _ws(conv_wgrad_workspace_bytes(d), x.device)
    _check(raw.conv_wgrad_bn_in(ctypes.byref(d), _ptr(x), _ptr(in_gamma), _ptr(in_beta), _ptr(in_mean), _ptr(in_rstd),
                                _ptr(dy), _ptr(dw), _ptr(workspace), ctypes.c_size_t(workspace.numel()), _stream()))
    return dw


def bn_relu_bwd_from_sums(dz, x, handle, gamma, beta, mean, rstd, eps=1e-5, mode=1, relu_mask=None):
    """Returns dx, dresidual (None unless mode 2), dgamma, dbeta."""
    producer, sums = handle
    d = _bn_desc(x, eps, mode)
    dx = torch.empty_like(x)
    dres = torch.empty_like(x) if mode == 2 else None
    dgamma = torch.empty(d.C, dtype=torch.float32, device=x.device)
    dbeta = torch.empty(d.C, dtype=torch.float32, device=x.device)
    _check(raw.bn_relu_bwd_from_sums(ctypes.byref(d), ctypes.byref(producer), _ptr(dz), _ptr(x), _ptr(relu_mask),
                                     _ptr(gamma), _ptr(beta), _ptr(mean), _ptr(rstd), _ptr(sums), _ptr(dx),
                                     _ptr(dres), _ptr(dgamma), _ptr(dbeta), _stream()))
    return dx, dres, dgamma, dbeta


# -------------------------------------------------------------------- pooling
def maxpool_fwd(x, return_argmax=False):
    N, H, W, C = x.shape
    y = torch.empty((N, (H - 1) // 2 + 1, (W - 1) // 2 + 1, C), dtype=x.dtype, device=x.device)
    am = torch.empty(y.shape, dtype=torch.uint8, device=x.device) if return_argmax else None
    _check(raw.maxpool_fwd(N, H, W, C, _dt(x), _ptr(x), _ptr(y), _ptr(am), _stream()))
    return (y, am) if return_argmax else y


def maxpool_bwd(x, dy, dy2=None, argmax=None):
    """Winner from `argmax` (as returned by maxpool_fwd) when given, else recomputed from x."""
    N, H, W, C = x.shape
    dx = torch.empty_like(x)
    _check(raw.maxpool_bwd(N, H, W, C, _dt(x), _ptr(x), _ptr(argmax), _ptr(dy), _ptr(dy2), _ptr(dx), _stream()))
    return dx


def avgpool_fwd(x):
    N, H, W, C = x.shape
    y = torch.empty((N, C), dtype=x.dtype, device=x.device)
    _check(raw.avgpool_fwd(N, H * W, C, _dt(x), _ptr(x), _ptr(y), _stream()))
    return y


def avgpool_bwd(dy, H, W):
    N, C = dy.shape
    dx = torch.empty((N, H, W, C), dtype=dy.dtype, device=dy.device)
    _check(raw.avgpool_bwd(N, H * W, C, _dt(dy), _ptr(dy), _ptr(dx), _stream()))
    return dx


# ----------------------------------------------------------------- classifier
def fc_fwd(a, W, b):
    N, Cin = a.shape
    K = W.shape[0]
    logits = torch.empty((N, K), dtype=torch.float32, device=a.device)
    _check(raw.fc_fwd(N, Cin, K, _dt(a), _ptr(a), _ptr(W), _ptr(b), _ptr(logits), _stream()))
    return logits


def fc_bwd(a, W, dlogits):
    N, Cin = a.shape
    K = W.shape[0]
    da = torch.empty_like(a)
    dW = torch.empty((K, Cin), dtype=torch.float32, device=a.device)
    db = torch.empty(K, dtype=torch.float32, device=a.device)
    raw.fc_bwd_workspace_bytes.restype = ctypes.c_size_t
    ws = _ws(raw.fc_bwd_workspace_bytes(N, Cin, K, _dt(a)), a.device)
    _check(raw.fc_bwd(N, Cin, K, _dt(a), _ptr(a), _ptr(W), _ptr(dlogits), _ptr(da), _ptr(dW), _ptr(db), _ptr(ws),
                      ctypes.c_size_t(ws.numel()), _stream()))
    return da, dW, db


def xent_fwd_bwd(logits, labels, label_smoothing=0.0, grad_scale=1.0):
    """Returns loss (device float[1]), row_loss[N], dlogits[N,K]."""
    N, K = logits.shape
    assert logits.dtype == torch.float32 and labels.dtype == torch.int32
    loss = torch.empty(1, dtype=torch.float32, device=logits.device)
    row = torch.empty(N, dtype=torch.float32, device=logits.device)
    dl = torch.empty_like(logits)
    _check(raw.xent_fwd_bwd(N, K, _ptr(logits), _ptr(labels), ctypes.c_float(label_smoothing),
                            ctypes.c_float(grad_scale), _ptr(loss), _ptr(row), _ptr(dl), _stream()))
    return loss, row, dl


# ----------------------------------------------------------------------- LARS
class LarsTable:
    """Host and device copies of the tensor table of lars_update (built once, reused every step)."""

    def __init__(self, ws, gs, vs, weight_decays, apply_trust=None, w_lowp=None):
        T = len(ws)
        self.T = T
        self.host = (LarsTensor * T)()
        self.keep = (ws, gs, vs, w_lowp)
        self.grad_dtype = _dt(gs[0])
        for t in range(T):
            assert ws[t].dtype == torch.float32 and vs[t].dtype == torch.float32
            assert ws[t].numel() == gs[t].numel() == vs[t].numel() and _dt(gs[t]) == self.grad_dtype
            lp = w_lowp[t] if w_lowp is not None else None
            self.host[t] = LarsTensor(ws[t].data_ptr(), gs[t].data_ptr(), vs[t].data_ptr(),
                                      lp.data_ptr() if lp is not None else 0, ws[t].numel(),
                                      float(weight_decays[t]), int(1 if apply_trust is None else apply_trust[t]))
        blob = bytes(self.host)
        self.dev = torch.frombuffer(bytearray(blob), dtype=torch.uint8).to(ws[0].device)
        self.device = ws[0].device


def lars_update(table, eta, momentum, lr, eps=0.0, norms_out=None, workspace=None):
    d = LarsDesc(table.T, eta, momentum, lr, eps, table.grad_dtype)
    if workspace is None:
        workspace = _ws(raw.lars_update_workspace_bytes(ctypes.byref(d), table.host), table.device)
    _check(raw.lars_update(ctypes.byref(d), table.host, _ptr(table.dev), _ptr(norms_out), _ptr(workspace),
                           ctypes.c_size_t(workspace.numel()), _stream()))
    return norms_out


def lars_update_noalloc(table, eta, momentum, lr, eps=0.0, norms_out=None):
    """lars_update without a workspace: the library's built-in scratch array holds the partial norms."""
    d = LarsDesc(table.T, eta, momentum, lr, eps, table.grad_dtype)
    _check(raw.lars_update_noalloc(ctypes.byref(d), table.host, _ptr(table.dev), _ptr(norms_out), _stream()))
    return norms_out


# ----------------------------------------------------------------- whole step
class ResnetPlan:
    def __init__(self, N, dtype=BF16, image_hw=224, classes=1000, widths=(64, 128, 256, 512), blocks=(3, 4, 6, 3),
                 stem=64, expansion=4, bn_eps=1e-5, label_smoothing=0.0, grad_scale=1.0, eta=0.001, momentum=0.9,
                 weight_decay=5e-5, lars_eps=0.0):
        self.cfg = StepConfig(N, image_hw, classes, dtype, (ctypes.c_int * 4)(*widths), (ctypes.c_int * 4)(*blocks),
                              stem, expansion, bn_eps, label_smoothing, grad_scale, eta, momentum, weight_decay,
                              lars_eps)
        self.handle = ctypes.c_void_p()
        _check(raw.resnet_plan_create(ctypes.byref(self.cfg), ctypes.byref(self.handle)))
        self.num_tensors = raw.resnet_plan_num_tensors(self.handle)
        self.shapes, self.offsets, self.sizes = [], [], []
        for i in range(self.num_tensors):
            dims = (ctypes.c_int * 4)()
            n = raw.resnet_plan_tensor_shape(self.handle, i, dims)
            self.shapes.append(tuple(int(v) for v in dims if v > 0))
            self.sizes.append(int(n))
            self.offsets.append(int(raw.resnet_plan_tensor_offset(self.handle, i)))
        self.arena_elems = int(raw.resnet_plan_arena_elems(self.handle))
        self.workspace_bytes = int(raw.resnet_plan_workspace_bytes(self.handle))
        self.dtype = dtype
        self.N, self.classes = N, classes

    def __del__(self):
        if getattr(self, "handle", None) and self.handle.value:
            raw.resnet_plan_destroy.restype = None
            raw.resnet_plan_destroy(self.handle)
            self.handle = ctypes.c_void_p()

    def view(self, arena, i):
        return arena[self.offsets[i]:self.offsets[i] + self.sizes[i]].view(self.shapes[i])

    def fuse_conv3_input(self, on=True):
        """conv3 of every block applies conv2's BN+ReLU in its operand load (same results, other timing)."""
        _check(raw.resnet_plan_fuse_conv3_input(self.handle, int(bool(on))))


def resnet_step(plan, images, labels, master, velocity, grads, model, lr, workspace, update=True, loss_out=None,
                logits_out=None):
    if loss_out is None:
        loss_out = torch.empty(1, dtype=torch.float32, device=images.device)
    _check(raw.resnet_step(plan.handle, _ptr(images), _ptr(labels), _ptr(master), _ptr(velocity), _ptr(grads),
                           _ptr(model), ctypes.c_float(lr), int(bool(update)), _ptr(loss_out), _ptr(logits_out),
                           _ptr(workspace), ctypes.c_size_t(workspace.numel()), _stream()))
    return loss_out


# ------------------------------------------------------------ training loop
DECAY_NONE, DECAY_STEP, DECAY_POLY, DECAY_LINEAR, DECAY_TABLE = range(5)
_DECAY = {"none": DECAY_NONE, "step": DECAY_STEP, "polynomial": DECAY_POLY, "linear": DECAY_LINEAR, "table": DECAY_TABLE}


class LrSchedule(ctypes.Structure):
    """rn50_lr_schedule.  `table`: a float32 device tensor (kept alive by this object)."""
    _fields_ = [("base_lr", ctypes.c_float), ("warmup_start_lr", ctypes.c_float), ("warmup_steps", ctypes.c_int),
                ("decay", ctypes.c_int), ("total_steps", ctypes.c_int), ("end_lr", ctypes.c_float),
                ("power", ctypes.c_float), ("step_every", ctypes.c_int), ("step_factor", ctypes.c_float),
                ("table", ctypes.c_void_p), ("table_len", ctypes.c_int)]

    def __init__(self, base_lr=0.0, warmup_steps=0, warmup_start_lr=0.0, decay="none", total_steps=0, end_lr=0.0,
                 power=2.0, step_every=1, step_factor=0.1, table=None):
        super().__init__(base_lr, warmup_start_lr, warmup_steps, _DECAY.get(decay, decay), total_steps, end_lr, power,
                         step_every, step_factor, _ptr(table), 0 if table is None else table.numel())
        self._table = table


class TrainState:
    """The device-side training state of a plan: step counter, learning rate, BN moving averages."""

    def __init__(self, plan, device="cuda", first_step=0):
        self.plan = plan
        self.num_bn = raw.resnet_plan_num_bn(plan.handle)
        self.bn_channels = int(raw.resnet_plan_bn_channels(plan.handle))
        self.bn_slices = []
        for i in range(self.num_bn):
            c = ctypes.c_int()
            off = int(raw.resnet_plan_bn_offset(plan.handle, i, ctypes.byref(c)))
            self.bn_slices.append((off, c.value))
        nbytes = int(raw.resnet_train_state_bytes(plan.handle))
        assert nbytes == 256 + 8 * self.bn_channels
        self.buf = torch.empty(nbytes, dtype=torch.uint8, device=device)
        self.reset(first_step)

    def reset(self, first_step=0):
        _check(raw.resnet_train_state_init(self.plan.handle, _ptr(self.buf), ctypes.c_size_t(self.buf.numel()),
                                           ctypes.c_int64(first_step), _stream()))

    @property
    def step(self):
        return int(self.buf[:8].view(torch.int64).item())

    @property
    def lr(self):
        return float(self.buf[8:12].view(torch.float32).item())

    def _running(self, which):
        n = self.bn_channels
        arr = self.buf[256 + 4 * n * which:256 + 4 * n * (which + 1)].view(torch.float32)
        return [arr[o:o + c] for o, c in self.bn_slices]

    @property
    def running_mean(self):
        return self._running(0)

    @property
    def running_var(self):
        return self._running(1)


def resnet_train_step(plan, schedule, state, images, labels, master, velocity, grads, model, workspace, bn_momentum=0.9,
                      loss_out=None, logits_out=None):
    if loss_out is None:
        loss_out = torch.empty(1, dtype=torch.float32, device=images.device)
    _check(raw.resnet_train_step(plan.handle, ctypes.byref(schedule), _ptr(state.buf), ctypes.c_float(bn_momentum),
                                 _ptr(images), _ptr(labels), _ptr(master), _ptr(velocity), _ptr(grads), _ptr(model),
                                 _ptr(loss_out), _ptr(logits_out), _ptr(workspace), ctypes.c_size_t(workspace.numel()),
                                 _stream()))
    return loss_out


# ------------------------------------------------------------ initialization, evaluation
def resnet_init_params(plan, seed, master, velocity=None, model=None):
    _check(raw.resnet_init_params(plan.handle, ctypes.c_uint64(seed), _ptr(master), _ptr(velocity), _ptr(model), _stream()))


def bn_relu_infer(x, gamma, beta, running_mean, running_var, residual=None, eps=1e-5, mode=1):
    d = _bn_desc(x, eps, mode)
    y = torch.empty_like(x)
    ws = _ws(raw.bn_relu_infer_workspace_bytes(ctypes.byref(d)), x.device)
    _check(raw.bn_relu_infer(ctypes.byref(d), _ptr(x), _ptr(gamma), _ptr(beta), _ptr(running_mean), _ptr(running_var),
                             _ptr(residual), _ptr(y), _ptr(ws), ctypes.c_size_t(ws.numel()), _stream()))
    return y


def top1_accuracy(logits, labels):
    """Returns (pred int32[N], correct int32[1]) device tensors."""
    N, K = logits.shape
    pred = torch.empty(N, dtype=torch.int32, device=logits.device)
    correct = torch.empty(1, dtype=torch.int32, device=logits.device)
    _check(raw.top1_accuracy(N, K, _ptr(logits), _ptr(labels), _ptr(pred), _ptr(correct), _stream()))
    return pred, correct


def resnet_eval(plan, state, images, labels, master, model, workspace, logits_out=None):
    """Returns (pred int32[N], correct int32[1]) device tensors."""
    pred = torch.empty(plan.N, dtype=torch.int32, device=images.device)
    correct = torch.empty(1, dtype=torch.int32, device=images.device)
    _check(raw.resnet_eval(plan.handle, _ptr(state.buf), _ptr(images), _ptr(labels), _ptr(master), _ptr(model),
                           _ptr(logits_out), _ptr(pred), _ptr(correct), _ptr(workspace),
                           ctypes.c_size_t(workspace.numel()), _stream()))
    return pred, correct


# ------------------------------------------------------------ launch timing
def profile_begin(kernel_tag, max_records):
    _check(raw.rn50_profile_begin(kernel_tag.encode(), int(max_records)))
    profile_begin._cap = int(max_records)


def profile_pause(paused):
    raw.rn50_profile_pause(ctypes.c_int(1 if paused else 0))


def profile_end():
    """Elapsed milliseconds of every recorded launch of the tagged kernel, in launch order."""
    cap = getattr(profile_begin, "_cap", 0)
    buf = (ctypes.c_float * max(cap, 1))()
    n = raw.rn50_profile_end(buf, cap)
    if n < 0:
        _check(n)
    profile_end._n = min(n, cap)
    return [float(buf[i]) for i in range(min(n, cap))]


def profile_end_timeline():
    """(start ms after the first recorded launch began, duration ms) of every recorded launch, in launch order."""
    cap = getattr(profile_begin, "_cap", 0)
    buf, at = (ctypes.c_float * max(cap, 1))(), (ctypes.c_float * max(cap, 1))()
    n = raw.rn50_profile_end_timeline(buf, at, cap)
    if n < 0:
        _check(n)
    profile_end._n = min(n, cap)
    return [(float(at[i]), float(buf[i])) for i in range(min(n, cap))]


def profile_tags():
    """The kernel tag of every record the last profile_end returned, in the same order."""
    return [raw.rn50_profile_tag(i).decode() for i in range(getattr(profile_end, "_n", 0))]
