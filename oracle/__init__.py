"""CPU oracle: numpy-facing wrappers around oracle.c.

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by __graft_entry__.smoke() and
by bench.py's cpu_baseline leg; never by the product package.  It shares no
code with the HIP path.

Every function takes and returns numpy arrays.  Activations are NHWC, weights
KRSC.  The storage type follows the dtype of the first array argument
(float32 or float64); all sums are accumulated in double inside oracle.c.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None


def lib():
    global _LIB
    if _LIB is None:
        path = _build.LIB
        if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_build.SRC):
            _build.build()
        _LIB = ctypes.CDLL(path)
    return _LIB


def _sfx(a):
    if a.dtype == np.float32:
        return "_f32"
    if a.dtype == np.float64:
        return "_f64"
    raise TypeError(f"oracle works on float32/float64 arrays, got {a.dtype}")


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dt=None):
    if a is None:
        return None
    return np.ascontiguousarray(a, dtype=dt if dt is not None else a.dtype)


def _call(name, a0, *args):
    f = getattr(lib(), name + _sfx(a0))
    f.restype = None
    f(*args)


def out_dim(n, pad, k, stride):
    return (n + 2 * pad - k) // stride + 1


# ---------------------------------------------------------------- convolution
def conv_fwd(x, w, stride, pad):
    x = _c(x); w = _c(w, x.dtype)
    N, H, W, C = x.shape
    K, R, S, C2 = w.shape
    assert C == C2
    y = np.empty((N, out_dim(H, pad, R, stride), out_dim(W, pad, S, stride), K), x.dtype)
    _call("orc_conv_fwd", x, _p(x), _p(w), _p(y), N, H, W, C, K, R, S, stride, pad)
    return y


def conv_dgrad(dy, w, x_shape, stride, pad):
    dy = _c(dy); w = _c(w, dy.dtype)
    N, H, W, C = x_shape
    K, R, S, C2 = w.shape
    assert C == C2 and dy.shape == (N, out_dim(H, pad, R, stride), out_dim(W, pad, S, stride), K)
    dx = np.empty((N, H, W, C), dy.dtype)
    _call("orc_conv_dgrad", dy, _p(dy), _p(w), _p(dx), N, H, W, C, K, R, S, stride, pad)
    return dx


def conv_wgrad(x, dy, w_shape, stride, pad):
    x = _c(x); dy = _c(dy, x.dtype)
    N, H, W, C = x.shape
    K, R, S, C2 = w_shape
    assert C == C2 and dy.shape == (N, out_dim(H, pad, R, stride), out_dim(W, pad, S, stride), K)
    dw = np.empty((K, R, S, C), x.dtype)
    _call("orc_conv_wgrad", x, _p(x), _p(dy), _p(dw), N, H, W, C, K, R, S, stride, pad)
    return dw


# ---------------------------------------------------------- batch norm (+ReLU)
def bn_relu_fwd(x, gamma, beta, residual=None, eps=1e-5, mode=1):
    """mode 0: BN; 1: BN+ReLU; 2: BN + residual + ReLU.  Returns y, mean, rstd."""
    x = _c(x); dt = x.dtype
    gamma = _c(gamma, dt); beta = _c(beta, dt); residual = _c(residual, dt)
    C = x.shape[-1]
    m = x.size // C
    assert (mode == 2) == (residual is not None)
    y = np.empty_like(x)
    mean = np.empty(C, dt); rstd = np.empty(C, dt)
    _call("orc_bn_fwd", x, _p(x), _p(gamma), _p(beta), _p(residual), _p(y), _p(mean), _p(rstd),
          ctypes.c_int64(m), C, ctypes.c_double(eps), mode)
    return y, mean, rstd


def bn_running_update(x, running_mean, running_var, momentum=0.9):
    x = _c(x)
    C = x.shape[-1]
    rm = _c(running_mean, x.dtype).copy(); rv = _c(running_var, x.dtype).copy()
    _call("orc_bn_running", x, _p(x), _p(rm), _p(rv), ctypes.c_int64(x.size // C), C,
          ctypes.c_double(momentum))
    return rm, rv


def bn_infer(x, gamma, beta, running_mean, running_var, residual=None, eps=1e-5, mode=1):
    """BN in evaluation mode: the moving averages stand in for the batch statistics,
    y = gamma*(x - running_mean)/sqrt(running_var + eps) + beta, then the mode's tail (0: none, 1: ReLU,
    2: + residual, ReLU).  Plain numpy in double; the result has x's dtype."""
    x = _c(x)
    z = (x.astype(np.float64) - np.asarray(running_mean, np.float64)) / np.sqrt(np.asarray(running_var, np.float64) + eps)
    z = z * np.asarray(gamma, np.float64) + np.asarray(beta, np.float64)
    assert (mode == 2) == (residual is not None)
    if mode == 2:
        z = z + np.asarray(residual, np.float64)
    if mode >= 1:
        z = np.maximum(z, 0.0)
    return z.astype(x.dtype)


def top1(logits, labels):
    """Predicted class per row (the first maximum wins) and the number of rows whose prediction is the label."""
    pred = np.argmax(np.asarray(logits), axis=1).astype(np.int32)
    return pred, int((pred == np.asarray(labels)).sum())


def bn_relu_bwd(dz, x, z, gamma, mean, rstd, mode=1):
    """Returns dx, dresidual (None unless mode 2), dgamma, dbeta."""
    dz = _c(dz); dt = dz.dtype
    x = _c(x, dt); z = _c(z, dt); gamma = _c(gamma, dt); mean = _c(mean, dt); rstd = _c(rstd, dt)
    C = x.shape[-1]
    m = x.size // C
    if mode >= 1:
        assert z is not None
    dx = np.empty_like(x)
    dres = np.empty_like(x) if mode == 2 else None
    dgamma = np.empty(C, dt); dbeta = np.empty(C, dt)
    _call("orc_bn_bwd", dz, _p(dz), _p(x), _p(z), _p(gamma), _p(mean), _p(rstd), _p(dx), _p(dres),
          _p(dgamma), _p(dbeta), ctypes.c_int64(m), C, mode)
    return dx, dres, dgamma, dbeta


# -------------------------------------------------------------------- pooling
def maxpool_fwd(x, ksize=3, stride=2, pad=1, return_index=False):
    x = _c(x)
    N, H, W, C = x.shape
    P, Q = out_dim(H, pad, ksize, stride), out_dim(W, pad, ksize, stride)
    y = np.empty((N, P, Q, C), x.dtype)
    idx = np.empty((N, P, Q, C), np.int32) if return_index else None
    _call("orc_maxpool_fwd", x, _p(x), _p(y), _p(idx), N, H, W, C, ksize, stride, pad)
    return (y, idx) if return_index else y


def maxpool_bwd(x, dy, ksize=3, stride=2, pad=1):
    x = _c(x); dy = _c(dy, x.dtype)
    N, H, W, C = x.shape
    dx = np.empty_like(x)
    _call("orc_maxpool_bwd", x, _p(x), _p(dy), _p(dx), N, H, W, C, ksize, stride, pad)
    return dx


def avgpool_fwd(x):
    x = _c(x)
    N, H, W, C = x.shape
    y = np.empty((N, C), x.dtype)
    _call("orc_avgpool_fwd", x, _p(x), _p(y), N, H * W, C)
    return y


def avgpool_bwd(dy, H, W):
    dy = _c(dy)
    N, C = dy.shape
    dx = np.empty((N, H, W, C), dy.dtype)
    _call("orc_avgpool_bwd", dy, _p(dy), _p(dx), N, H * W, C)
    return dx


# ------------------------------------------------------------ classifier head
def fc_fwd(a, W, b):
    a = _c(a); W = _c(W, a.dtype); b = _c(b, a.dtype)
    N, Cin = a.shape
    K = W.shape[0]
    logits = np.empty((N, K), a.dtype)
    _call("orc_fc_fwd", a, _p(a), _p(W), _p(b), _p(logits), N, Cin, K)
    return logits


def fc_bwd(a, W, dlogits):
    a = _c(a); W = _c(W, a.dtype); dlogits = _c(dlogits, a.dtype)
    N, Cin = a.shape
    K = W.shape[0]
    da = np.empty_like(a); dW = np.empty_like(W); db = np.empty(K, a.dtype)
    _call("orc_fc_bwd", a, _p(a), _p(W), _p(dlogits), _p(da), _p(dW), _p(db), N, Cin, K)
    return da, dW, db


def xent_fwd_bwd(logits, labels, label_smoothing=0.0, grad_scale=1.0):
    """Returns loss (python float), row_loss[N], dlogits[N,K]."""
    logits = _c(logits); labels = _c(labels, np.int32)
    N, K = logits.shape
    assert labels.shape == (N,) and labels.min() >= 0 and labels.max() < K
    loss = np.empty(1, logits.dtype); row = np.empty(N, logits.dtype)
    dl = np.empty_like(logits)
    _call("orc_xent", logits, _p(logits), _p(labels), N, K, ctypes.c_double(label_smoothing),
          ctypes.c_double(grad_scale), _p(loss), _p(row), _p(dl))
    return float(loss[0]), row, dl


# ----------------------------------------------------------------------- LARS
def lars_update(ws, gs, vs, eta, momentum, lr, weight_decays, eps=0.0, apply_trust=None):
    """Multi-tensor LARS step.  ws/gs/vs: lists of arrays (not modified).

    Returns (w_new list, v_new list, norms float64 [T, 2] = (||w||, ||g||))."""
    T = len(ws)
    if apply_trust is None:
        apply_trust = [1] * T
    w_new, v_new = [], []
    norms = np.zeros((T, 2), np.float64)
    for t in range(T):
        w = _c(ws[t]).copy(); g = _c(gs[t], w.dtype); v = _c(vs[t], w.dtype).copy()
        assert w.shape == g.shape == v.shape
        nt = np.zeros(2, np.float64)
        _call("orc_lars", w, _p(w), _p(g), _p(v), ctypes.c_int64(w.size), ctypes.c_double(eta),
              ctypes.c_double(momentum), ctypes.c_double(lr), ctypes.c_double(weight_decays[t]),
              ctypes.c_double(eps), int(apply_trust[t]), _p(nt))
        norms[t] = nt
        w_new.append(w); v_new.append(v)
    return w_new, v_new, norms


def rel_l2(a, b):
    """||a-b||_2 / ||b||_2 with b the oracle value, both norms in double."""
    a = np.asarray(a, np.float64).ravel(); b = np.asarray(b, np.float64).ravel()
    nb = np.sqrt(np.dot(b, b))
    d = a - b
    nd = np.sqrt(np.dot(d, d))
    if nb == 0.0:
        return 0.0 if nd == 0.0 else float("inf")
    return float(nd / nb)
