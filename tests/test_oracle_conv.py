"""Pins for the oracle's convolution passes: things fixed by mathematics or by
independent code, not by the oracle itself."""
import itertools

import numpy as np
import pytest

import oracle as orc
import synth

SEED = synth.DEFAULT_SEED


def brute_conv(x, w, stride, pad):
    """Seven nested python loops over the definition, in float64 (tiny shapes only)."""
    N, H, W, C = x.shape
    K, R, S, _ = w.shape
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    y = np.zeros((N, P, Q, K))
    for n, p, q, k in itertools.product(range(N), range(P), range(Q), range(K)):
        acc = 0.0
        for r, s, c in itertools.product(range(R), range(S), range(C)):
            ih, iw = p * stride - pad + r, q * stride - pad + s
            if 0 <= ih < H and 0 <= iw < W:
                acc += float(x[n, ih, iw, c]) * float(w[k, r, s, c])
        y[n, p, q, k] = acc
    return y


def shift_matmul_conv(x, w, stride, pad):
    """Independent formulation: zero-pad, then one strided slice x matrix product per tap."""
    N, H, W, C = x.shape
    K, R, S, _ = w.shape
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    xp = np.pad(x.astype(np.float64), ((0, 0), (pad, pad), (pad, pad), (0, 0)))
    y = np.zeros((N, P, Q, K))
    for r in range(R):
        for s in range(S):
            sl = xp[:, r:r + (P - 1) * stride + 1:stride, s:s + (Q - 1) * stride + 1:stride, :]
            y += sl @ w[:, r, s, :].astype(np.float64).T
    return y


CASES = [  # N,H,W,C,K,R,stride,pad
    (1, 5, 5, 3, 2, 3, 1, 1),
    (2, 6, 7, 2, 3, 3, 2, 1),
    (1, 9, 8, 3, 4, 7, 2, 3),
    (2, 4, 4, 5, 3, 1, 1, 0),
    (1, 6, 6, 4, 2, 1, 2, 0),
    (1, 5, 4, 2, 2, 3, 1, 0),
]


def _rand(tag, shape, dtype=np.float64):
    return synth.normal(SEED, tag, shape, 1.0, dtype)


@pytest.mark.parametrize("case", CASES)
def test_fwd_vs_python_loops(case):
    N, H, W, C, K, R, stride, pad = case
    x = _rand("x%s" % (case,), (N, H, W, C)); w = _rand("w%s" % (case,), (K, R, R, C))
    y = orc.conv_fwd(x, w, stride, pad)
    np.testing.assert_allclose(y, brute_conv(x, w, stride, pad), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("case", [(2, 14, 14, 16, 24, 3, 1, 1), (2, 15, 13, 8, 8, 3, 2, 1),
                                  (1, 32, 32, 3, 16, 7, 2, 3), (2, 14, 14, 32, 8, 1, 2, 0)])
def test_fwd_vs_shift_matmul(case):
    N, H, W, C, K, R, stride, pad = case
    x = _rand("x", (N, H, W, C)); w = _rand("w", (K, R, R, C))
    np.testing.assert_allclose(orc.conv_fwd(x, w, stride, pad), shift_matmul_conv(x, w, stride, pad),
                               rtol=1e-11, atol=1e-11)
    y32 = orc.conv_fwd(x.astype(np.float32), w.astype(np.float32), stride, pad)
    assert y32.dtype == np.float32
    assert orc.rel_l2(y32, shift_matmul_conv(x.astype(np.float32), w.astype(np.float32), stride, pad)) < 2e-7


def test_1x1_is_matmul():
    x = _rand("x", (2, 5, 6, 7)); w = _rand("w", (4, 1, 1, 7))
    y = orc.conv_fwd(x, w, 1, 0)
    np.testing.assert_allclose(y.reshape(-1, 4), x.reshape(-1, 7) @ w.reshape(4, 7).T, rtol=1e-12, atol=1e-12)


def test_delta_kernel_shifts_input():
    x = _rand("x", (1, 6, 6, 2))
    for (r, s) in [(0, 0), (1, 1), (2, 0), (0, 2)]:
        w = np.zeros((2, 3, 3, 2))
        w[0, r, s, 0] = 1.0; w[1, r, s, 1] = 1.0       # identity over channels at tap (r,s)
        y = orc.conv_fwd(x, w, 1, 1)
        xp = np.pad(x, ((0, 0), (1, 1), (1, 1), (0, 0)))
        np.testing.assert_array_equal(y, xp[:, r:r + 6, s:s + 6, :])


@pytest.mark.parametrize("R,stride,pad", [(3, 1, 1), (3, 2, 1), (7, 2, 3), (1, 2, 0)])
def test_all_ones_counts_inbounds_taps(R, stride, pad):
    H = W = 9; C = 2
    y = orc.conv_fwd(np.ones((1, H, W, C)), np.ones((1, R, R, C)), stride, pad)
    P = (H + 2 * pad - R) // stride + 1
    for p in range(P):
        for q in range(P):
            nh = sum(0 <= p * stride - pad + r < H for r in range(R))
            nw = sum(0 <= q * stride - pad + s < W for s in range(R))
            assert y[0, p, q, 0] == nh * nw * C


def test_linearity():
    x1 = _rand("x1", (1, 7, 7, 3)); x2 = _rand("x2", (1, 7, 7, 3))
    w1 = _rand("w1", (2, 3, 3, 3)); w2 = _rand("w2", (2, 3, 3, 3))
    f = lambda x, w: orc.conv_fwd(x, w, 2, 1)
    np.testing.assert_allclose(f(2 * x1 - 3 * x2, w1), 2 * f(x1, w1) - 3 * f(x2, w1), atol=1e-12)
    np.testing.assert_allclose(f(x1, 2 * w1 - 3 * w2), 2 * f(x1, w1) - 3 * f(x1, w2), atol=1e-12)


GRAD_CASES = CASES + [(2, 8, 8, 4, 6, 3, 2, 1), (1, 7, 7, 3, 2, 3, 2, 1), (2, 7, 9, 2, 3, 1, 2, 0)]


@pytest.mark.parametrize("case", GRAD_CASES)
def test_adjoint_identities(case):
    """<conv(x,w), dy> = <x, dgrad(dy,w)> = <w, wgrad(x,dy)> (exact up to rounding)."""
    N, H, W, C, K, R, stride, pad = case
    x = _rand("x", (N, H, W, C)); w = _rand("w", (K, R, R, C))
    y = orc.conv_fwd(x, w, stride, pad)
    dy = _rand("dy", y.shape)
    dx = orc.conv_dgrad(dy, w, x.shape, stride, pad)
    dw = orc.conv_wgrad(x, dy, w.shape, stride, pad)
    ref = np.sum(y * dy)
    assert abs(np.sum(x * dx) - ref) < 1e-10 * max(1.0, abs(ref))
    assert abs(np.sum(w * dw) - ref) < 1e-10 * max(1.0, abs(ref))


@pytest.mark.parametrize("case", [(1, 5, 5, 2, 2, 3, 1, 1), (1, 6, 7, 2, 2, 3, 2, 1), (1, 4, 4, 3, 2, 1, 2, 0)])
def test_grads_elementwise_bruteforce(case):
    """Every dx / dw element equals the derivative of L = <conv(x,w), dy>, which is linear in
    x and in w: the derivative along a unit vector is L(unit) exactly."""
    N, H, W, C, K, R, stride, pad = case
    x = _rand("x", (N, H, W, C)); w = _rand("w", (K, R, R, C))
    dy = _rand("dy", brute_conv(x, w, stride, pad).shape)
    dx = orc.conv_dgrad(dy, w, x.shape, stride, pad)
    dw = orc.conv_wgrad(x, dy, w.shape, stride, pad)
    for idx in np.ndindex(*x.shape):
        e = np.zeros_like(x); e[idx] = 1.0
        assert abs(np.sum(brute_conv(e, w, stride, pad) * dy) - dx[idx]) < 1e-11
    for idx in np.ndindex(*w.shape):
        e = np.zeros_like(w); e[idx] = 1.0
        assert abs(np.sum(brute_conv(x, e, stride, pad) * dy) - dw[idx]) < 1e-11


def test_f32_build_matches_f64_build():
    x = _rand("x", (2, 9, 9, 8)); w = _rand("w", (6, 3, 3, 8))
    x32, w32 = x.astype(np.float32), w.astype(np.float32)
    y = orc.conv_fwd(x32.astype(np.float64), w32.astype(np.float64), 2, 1)
    dy = _rand("dy", y.shape).astype(np.float32)
    assert orc.rel_l2(orc.conv_fwd(x32, w32, 2, 1), y) < 1e-7
    assert orc.rel_l2(orc.conv_dgrad(dy, w32, x.shape, 2, 1),
                      orc.conv_dgrad(dy.astype(np.float64), w32.astype(np.float64), x.shape, 2, 1)) < 1e-7
    assert orc.rel_l2(orc.conv_wgrad(x32, dy, w.shape, 2, 1),
                      orc.conv_wgrad(x32.astype(np.float64), dy.astype(np.float64), w.shape, 2, 1)) < 1e-7
