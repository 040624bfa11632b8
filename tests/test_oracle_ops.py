"""Pins for the oracle's BN, pooling, classifier, loss and LARS operations."""
import math

import numpy as np
import pytest

import oracle as orc
import synth

SEED = synth.DEFAULT_SEED


def _rand(tag, shape, std=1.0):
    return synth.normal(SEED, tag, shape, std, np.float64)


def fd_grad(f, x, h=1e-6):
    """Central finite differences of scalar f at x (float64), element by element."""
    g = np.zeros_like(x)
    flat = x.reshape(-1); gf = g.reshape(-1)
    for i in range(flat.size):
        old = flat[i]
        flat[i] = old + h; fp = f(x)
        flat[i] = old - h; fm = f(x)
        flat[i] = old
        gf[i] = (fp - fm) / (2 * h)
    return g


# ------------------------------------------------------------------ BN forward
@pytest.mark.parametrize("dtype,tol", [(np.float64, 1e-12), (np.float32, 2e-6)])
def test_bn_invariant_zero_mean_unit_var(dtype, tol):
    """Before the affine step the normalised activations have per-channel mean 0 and
    biased variance var/(var+eps)."""
    x = (_rand("x", (4, 5, 6, 7)) * 3.0 + 1.5).astype(dtype)
    C = 7; eps = 1e-5
    y, mean, rstd = orc.bn_relu_fwd(x, np.ones(C, dtype), np.zeros(C, dtype), None, eps, 0)
    flat = y.reshape(-1, C).astype(np.float64)
    var = x.reshape(-1, C).astype(np.float64).var(axis=0)
    assert np.abs(flat.mean(axis=0)).max() < tol * 10
    np.testing.assert_allclose(flat.var(axis=0), var / (var + eps), rtol=max(tol, 1e-10) * 10)
    np.testing.assert_allclose(mean, x.reshape(-1, C).astype(np.float64).mean(axis=0), rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(rstd, 1 / np.sqrt(var + eps), rtol=1e-6)


def test_bn_constant_channel_gives_beta():
    x = np.full((2, 3, 3, 2), 4.25); x[..., 1] = _rand("c1", (2, 3, 3))
    gamma = np.array([2.0, 1.0]); beta = np.array([0.75, -0.5])
    y, _, _ = orc.bn_relu_fwd(x, gamma, beta, None, 1e-5, 0)
    np.testing.assert_allclose(y[..., 0], 0.75, atol=1e-12)


def test_bn_scale_shift_invariance():
    x = _rand("x", (3, 4, 4, 5)); g = _rand("g", (5,)); b = _rand("b", (5,))
    y1, _, _ = orc.bn_relu_fwd(x, g, b, None, 1e-12, 0)
    y2, _, _ = orc.bn_relu_fwd(3.5 * x - 2.0, g, b, None, 1e-12, 0)
    np.testing.assert_allclose(y1, y2, atol=1e-9)


def test_bn_modes_relu_and_residual():
    x = _rand("x", (2, 3, 3, 4)); g = _rand("g", (4,)); b = _rand("b", (4,)); r = _rand("r", x.shape)
    y0, _, _ = orc.bn_relu_fwd(x, g, b, None, 1e-5, 0)
    y1, _, _ = orc.bn_relu_fwd(x, g, b, None, 1e-5, 1)
    y2, _, _ = orc.bn_relu_fwd(x, g, b, r, 1e-5, 2)
    np.testing.assert_array_equal(y1, np.maximum(y0, 0))
    np.testing.assert_allclose(y2, np.maximum(y0 + r, 0), atol=1e-15)
    assert (y1 == 0).any() and (y1 > 0).any()


def test_bn_running_stats():
    x = _rand("x", (4, 3, 3, 2)) * 2 + 1
    rm, rv = orc.bn_running_update(x, np.array([1.0, -1.0]), np.array([2.0, 3.0]), 0.9)
    f = x.reshape(-1, 2)
    np.testing.assert_allclose(rm, 0.9 * np.array([1.0, -1.0]) + 0.1 * f.mean(0), rtol=1e-12)
    np.testing.assert_allclose(rv, 0.9 * np.array([2.0, 3.0]) + 0.1 * f.var(0), rtol=1e-12)


# ----------------------------------------------------------------- BN backward
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_bn_bwd_finite_differences(mode):
    x = _rand("x", (2, 3, 3, 3)); g = _rand("g", (3,)) + 1.5; b = _rand("b", (3,)) * 0.3
    r = _rand("r", x.shape) if mode == 2 else None
    T = _rand("T", x.shape)
    eps = 1e-5

    def loss(xx, gg, bb, rr):
        y, _, _ = orc.bn_relu_fwd(xx, gg, bb, rr, eps, mode)
        return float(np.sum(y * T))

    z, mean, rstd = orc.bn_relu_fwd(x, g, b, r, eps, mode)
    assert np.abs(z[z != 0]).min() > 1e-4 if mode else True      # away from the ReLU kink
    dx, dres, dg, db = orc.bn_relu_bwd(T, x, z, g, mean, rstd, mode)
    np.testing.assert_allclose(dx, fd_grad(lambda a: loss(a, g, b, r), x.copy()), rtol=1e-5, atol=1e-7)
    np.testing.assert_allclose(dg, fd_grad(lambda a: loss(x, a, b, r), g.copy()), rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(db, fd_grad(lambda a: loss(x, g, a, r), b.copy()), rtol=1e-6, atol=1e-8)
    if mode == 2:
        np.testing.assert_allclose(dres, fd_grad(lambda a: loss(x, g, b, a), r.copy()), rtol=1e-6, atol=1e-8)
    else:
        assert dres is None


def test_bn_bwd_orthogonality_and_direct_sums():
    """dx is orthogonal to the two directions BN removes; dbeta, dgamma are direct sums."""
    x = _rand("x", (3, 4, 4, 6)) * 2 + 0.5; g = _rand("g", (6,)) + 2.0; b = _rand("b", (6,))
    dz = _rand("dz", x.shape)
    z, mean, rstd = orc.bn_relu_fwd(x, g, b, None, 1e-5, 1)
    dx, _, dg, db = orc.bn_relu_bwd(dz, x, z, g, mean, rstd, 1)
    xh = (x - mean) * rstd
    gm = dz * (z > 0)
    np.testing.assert_allclose(db, gm.reshape(-1, 6).sum(0), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dg, (gm * xh).reshape(-1, 6).sum(0), rtol=1e-12, atol=1e-12)
    assert np.abs(dx.reshape(-1, 6).sum(0)).max() < 1e-10
    # sum_m dx*xhat = gamma*rstd*dgamma*(1 - var/(var+eps)): zero up to the eps term
    var = x.reshape(-1, 6).var(0)
    np.testing.assert_allclose((dx * xh).reshape(-1, 6).sum(0), g * rstd * dg * (1 - var / (var + 1e-5)),
                               rtol=1e-8, atol=1e-10)


def test_conv_then_bn_scale_invariance():
    """A conv feeding a batch-stat BN is scale invariant, so <w, dL/dw> ~ 0 (exact as eps -> 0)
    and a bias before BN would get zero gradient (sum over m of dy is 0)."""
    x = _rand("x", (2, 6, 6, 3)); w = _rand("w", (4, 3, 3, 3)); g = _rand("g", (4,)) + 1.5; b = _rand("b", (4,))
    T = _rand("T", (2, 6, 6, 4))
    y = orc.conv_fwd(x, w, 1, 1)
    z, mean, rstd = orc.bn_relu_fwd(y, g, b, None, 1e-12, 1)
    dy, _, _, _ = orc.bn_relu_bwd(T, y, z, g, mean, rstd, 1)
    dw = orc.conv_wgrad(x, dy, w.shape, 1, 1)
    assert abs(np.sum(w * dw)) < 1e-8 * np.linalg.norm(w) * np.linalg.norm(dw)
    assert np.abs(dy.reshape(-1, 4).sum(0)).max() < 1e-10


# --------------------------------------------------------------------- pooling
def test_maxpool_small_by_hand():
    # 1 image, 4x4, 1 channel; 3x3 window stride 2 pad 1 -> 2x2 outputs
    x = np.array([[1, 2, 3, 4], [5, 6, 7, 8], [9, 10, 11, 12], [13, 14, 15, 16]], np.float64).reshape(1, 4, 4, 1)
    y, idx = orc.maxpool_fwd(x, 3, 2, 1, return_index=True)
    np.testing.assert_array_equal(y.reshape(2, 2), [[6, 8], [14, 16]])
    np.testing.assert_array_equal(idx.reshape(2, 2), [[5, 7], [13, 15]])
    dx = orc.maxpool_bwd(x, np.array([1.0, 2.0, 3.0, 4.0]).reshape(1, 2, 2, 1), 3, 2, 1)
    exp = np.zeros(16); exp[[5, 7, 13, 15]] = [1, 2, 3, 4]
    np.testing.assert_array_equal(dx.reshape(-1), exp)


def test_maxpool_ties_first_wins_and_negative_inputs():
    x = np.full((1, 4, 4, 1), -3.0)                 # all equal and negative: padding must not win
    y, idx = orc.maxpool_fwd(x, 3, 2, 1, return_index=True)
    np.testing.assert_array_equal(y, -3.0)
    np.testing.assert_array_equal(idx.reshape(-1), [0, 1, 4, 5])     # first in-bounds position of each window
    dx = orc.maxpool_bwd(x, np.ones((1, 2, 2, 1)), 3, 2, 1)
    assert dx.sum() == 4.0 and dx.reshape(-1)[[0, 1, 4, 5]].tolist() == [1, 1, 1, 1]


def test_maxpool_vs_numpy_windows_and_fd():
    x = _rand("x", (2, 9, 8, 3))
    y = orc.maxpool_fwd(x, 3, 2, 1)
    xp = np.pad(x, ((0, 0), (1, 1), (1, 1), (0, 0)), constant_values=-np.inf)
    P, Q = y.shape[1:3]
    ref = np.stack([xp[:, r:r + 2 * P - 1:2, s:s + 2 * Q - 1:2, :] for r in range(3) for s in range(3)]).max(0)
    np.testing.assert_array_equal(y, ref)
    T = _rand("T", y.shape)
    dx = orc.maxpool_bwd(x, T, 3, 2, 1)
    np.testing.assert_allclose(dx, fd_grad(lambda a: float(np.sum(orc.maxpool_fwd(a, 3, 2, 1) * T)), x.copy()),
                               rtol=1e-6, atol=1e-8)
    assert abs(dx.sum() - T.sum()) < 1e-10


def test_avgpool():
    x = _rand("x", (3, 7, 7, 5))
    y = orc.avgpool_fwd(x)
    np.testing.assert_allclose(y, x.mean(axis=(1, 2)), rtol=1e-13)
    dy = _rand("dy", (3, 5))
    dx = orc.avgpool_bwd(dy, 7, 7)
    np.testing.assert_allclose(dx, np.broadcast_to(dy[:, None, None, :] / 49.0, x.shape), rtol=1e-15)


# ---------------------------------------------------------------------- FC
def test_fc_vs_matmul_and_adjoint():
    a = _rand("a", (5, 16)); W = _rand("W", (7, 16)); b = _rand("b", (7,)); dl = _rand("dl", (5, 7))
    np.testing.assert_allclose(orc.fc_fwd(a, W, b), a @ W.T + b, rtol=1e-12, atol=1e-12)
    da, dW, db = orc.fc_bwd(a, W, dl)
    np.testing.assert_allclose(da, dl @ W, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dW, dl.T @ a, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(db, dl.sum(0), rtol=1e-12, atol=1e-12)
    f = lambda aa, WW, bb: float(np.sum(orc.fc_fwd(aa, WW, bb) * dl))
    np.testing.assert_allclose(dW, fd_grad(lambda X: f(a, X, b), W.copy()), rtol=1e-6, atol=1e-8)


# ------------------------------------------------------------- softmax-CE loss
@pytest.mark.parametrize("ls", [0.0, 0.1, 0.5])
def test_xent_uniform_logits_is_log_K(ls):
    K = 1000
    loss, row, dl = orc.xent_fwd_bwd(np.full((3, K), 0.37), np.array([0, 999, 5]), ls)
    assert abs(loss - math.log(1000.0)) < 1e-12 and abs(loss - 6.907755278982137) < 1e-12
    np.testing.assert_allclose(row, math.log(K), rtol=1e-13)


@pytest.mark.parametrize("ls", [0.0, 0.1])
def test_xent_properties_and_fd(ls):
    N, K = 4, 9
    l = _rand("l", (N, K)) * 2; y = synth.labels(SEED, "y", N, K)
    loss, row, dl = orc.xent_fwd_bwd(l, y, ls, 1.0)
    assert np.abs(dl.sum(axis=1)).max() < 1e-15                       # rows of the gradient sum to 0
    loss2, _, dl2 = orc.xent_fwd_bwd(l + 123.456, y, ls, 1.0)          # shift invariance
    assert abs(loss - loss2) < 1e-12 and np.abs(dl - dl2).max() < 1e-13
    np.testing.assert_allclose(dl, fd_grad(lambda a: orc.xent_fwd_bwd(a, y, ls)[0], l.copy()), rtol=1e-6, atol=1e-9)
    _, _, dl3 = orc.xent_fwd_bwd(l, y, ls, 128.0)                      # grad_scale multiplies the gradient only
    np.testing.assert_allclose(dl3, 128.0 * dl, rtol=1e-14)
    # definition re-derived from log-softmax in numpy
    lp = l - np.log(np.exp(l - l.max(1, keepdims=True)).sum(1, keepdims=True)) - l.max(1, keepdims=True)
    q = np.full((N, K), ls / K); q[np.arange(N), y] += 1 - ls
    np.testing.assert_allclose(row, -(q * lp).sum(1), rtol=1e-12)
    assert abs(loss - row.mean()) < 1e-14


def test_xent_huge_logits_stay_finite():
    l = np.zeros((2, 5)); l[0, 1] = 1e4; l[1, 2] = -1e4
    loss, row, dl = orc.xent_fwd_bwd(l, np.array([1, 2]), 0.0)
    assert np.isfinite(loss) and np.isfinite(dl).all()
    assert abs(row[0]) < 1e-12 and abs(row[1] - 1e4 - math.log(4.0)) < 1e-9
    l32 = l.astype(np.float32)
    loss32, _, dl32 = orc.xent_fwd_bwd(l32, np.array([1, 2]), 0.0)
    assert np.isfinite(loss32) and np.isfinite(dl32).all()


# ------------------------------------------------------------------------ LARS
def _golden_lars():
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "lars_hand_example.txt")
    vals = {}
    for line in open(path):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            vals[k.strip()] = [float(t) for t in v.split(",")]
    return vals


def test_lars_hand_worked_example():
    """Two tensors worked by hand (see the fixture for the arithmetic)."""
    G = _golden_lars()
    ws = [np.array(G["w0"]), np.array(G["w1"])]
    gs = [np.array(G["g0"]), np.array(G["g1"])]
    vs = [np.array(G["v0"]), np.array(G["v1"])]
    wn, vn, norms = orc.lars_update(ws, gs, vs, eta=0.1, momentum=0.5, lr=2.0, weight_decays=[0.5, 0.0])
    np.testing.assert_allclose(norms, [[5.0, 10.0], [13.0, 0.5]], rtol=1e-14)
    np.testing.assert_allclose(vn[0], G["v0_new"], rtol=1e-13)
    np.testing.assert_allclose(wn[0], G["w0_new"], rtol=1e-13)
    np.testing.assert_allclose(vn[1], G["v1_new"], rtol=1e-13)
    np.testing.assert_allclose(wn[1], G["w1_new"], rtol=1e-13)


def test_lars_closed_form_properties():
    w = _rand("w", (300,)); g = _rand("g", (300,), 1e-3); v0 = np.zeros(300)
    eta, lr = 0.001, 1.0
    (w1,), (v1,), norms = orc.lars_update([w], [g], [v0], eta, 0.9, lr, [0.0])
    np.testing.assert_allclose(norms[0], [np.linalg.norm(w), np.linalg.norm(g)], rtol=1e-13)
    # beta = 0: ||dw|| = lr*eta*||w|| exactly, and dw does not change when g is rescaled
    assert abs(np.linalg.norm(w1 - w) - lr * eta * np.linalg.norm(w)) < 1e-12
    (w2,), _, _ = orc.lars_update([w], [37.0 * g], [v0], eta, 0.9, lr, [0.0])
    np.testing.assert_allclose(w2 - w, w1 - w, rtol=1e-10, atol=1e-15)
    # local lr closed form with weight decay
    wd = 5e-5
    (w3,), (v3,), _ = orc.lars_update([w], [g], [v0], eta, 0.9, lr, [wd])
    local = eta * np.linalg.norm(w) / (np.linalg.norm(g) + wd * np.linalg.norm(w))
    np.testing.assert_allclose(v3, lr * local * (g + wd * w), rtol=1e-12)
    np.testing.assert_allclose(w3, w - v3, rtol=1e-12)


def test_lars_reduces_to_sgd_without_trust():
    w = _rand("w", (50,)); g = _rand("g", (50,)); v = _rand("v", (50,))
    (w1,), (v1,), _ = orc.lars_update([w], [g], [v], 0.001, 0.0, 0.1, [0.01], apply_trust=[0])
    np.testing.assert_allclose(w1, w - 0.1 * (g + 0.01 * w), rtol=1e-13)     # textbook SGD + weight decay
    (w2,), (v2,), _ = orc.lars_update([w], [g], [v], 0.001, 0.9, 0.1, [0.0], apply_trust=[0])
    np.testing.assert_allclose(v2, 0.9 * v + 0.1 * g, rtol=1e-13)             # momentum form
    np.testing.assert_allclose(w2, w - v2, rtol=1e-13)


def test_lars_zero_norm_branch():
    """||w|| = 0 (BN beta at initialisation) or ||g|| = 0: trust ratio 1, plain lr."""
    g = _rand("g", (8,))
    (w1,), (v1,), n1 = orc.lars_update([np.zeros(8)], [g], [np.zeros(8)], 0.001, 0.9, 0.5, [0.0])
    np.testing.assert_allclose(w1, -0.5 * g, rtol=1e-14)
    assert n1[0, 0] == 0.0
    w = _rand("w", (8,))
    (w2,), (v2,), _ = orc.lars_update([w], [np.zeros(8)], [np.zeros(8)], 0.001, 0.9, 0.5, [0.1])
    np.testing.assert_allclose(w2, w - 0.5 * 0.1 * w, rtol=1e-14)


def test_lars_eps_in_denominator():
    w = _rand("w", (20,)); g = _rand("g", (20,))
    (_,), (v,), _ = orc.lars_update([w], [g], [np.zeros(20)], 0.01, 0.0, 1.0, [0.0], eps=0.25)
    local = 0.01 * np.linalg.norm(w) / (np.linalg.norm(g) + 0.25)
    np.testing.assert_allclose(v, local * g, rtol=1e-12)


def test_lars_f32_build():
    w = _rand("w", (5000,)).astype(np.float32); g = _rand("g", (5000,), 1e-3).astype(np.float32)
    v = np.zeros(5000, np.float32)
    a = orc.lars_update([w], [g], [v], 0.001, 0.9, 1.0, [5e-5])
    b = orc.lars_update([w.astype(np.float64)], [g.astype(np.float64)], [v.astype(np.float64)], 0.001, 0.9, 1.0, [5e-5])
    assert a[0][0].dtype == np.float32
    assert orc.rel_l2(a[0][0], b[0][0]) < 1e-7 and orc.rel_l2(a[1][0], b[1][0]) < 1e-7
