"""GPU parity of the convolution + batch-norm pairs whose per-channel sums are taken in the
convolution's output stage (conv_fwd_bn_sums -> bn_relu_fwd_from_sums, conv_dgrad_bn_sums ->
bn_relu_bwd_from_sums), against the oracle's separate operations, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle as orc
import synth
from gpu_util import impose_relu_decisions, TOL, assert_close, dev, host, inputs

pytestmark = pytest.mark.gpu
SEED = synth.DEFAULT_SEED


@pytest.fixture(scope="module")
def rn():
    import paper_1903_12650_amd as rn
    return rn


# (N, H, W, Cin, Cout, R, stride, pad): several row tiles with a ragged last one, ragged channel tiles,
# both strides, the stem, and a single-tile case
FUSED_SHAPES = [(2, 14, 14, 64, 64, 1, 1, 0), (3, 13, 9, 24, 40, 3, 1, 1), (2, 28, 28, 32, 136, 3, 2, 1),
                (5, 28, 28, 128, 128, 1, 1, 0), (2, 30, 30, 64, 256, 1, 2, 0), (1, 5, 5, 8, 8, 3, 1, 1),
                (2, 64, 64, 3, 64, 7, 2, 3), (40, 7, 7, 256, 64, 1, 1, 0), (3, 11, 13, 24, 40, 3, 2, 1),
                (2, 9, 7, 16, 16, 1, 2, 0),
                # 3x3 stride 1 pad 1, whole channel chunks, tiles spanning images
                (3, 9, 9, 64, 64, 3, 1, 1), (2, 5, 12, 128, 72, 3, 1, 1), (5, 7, 21, 192, 64, 3, 1, 1),
                (7, 4, 48, 64, 128, 3, 1, 1), (40, 14, 14, 64, 64, 3, 1, 1),
                # ... large enough for the eight-wave 256x128 tile (forward / data gradient): the sums' row count follows
                (16, 28, 28, 64, 512, 3, 1, 1), (16, 28, 28, 512, 64, 3, 1, 1)]


def _vec(tag, C, scale, shift):
    return (shift + scale * synth.normal(SEED, tag, (C,))).astype(np.float32)


@pytest.mark.parametrize("mode_name", ["f32", "bf16"])
@pytest.mark.parametrize("shape", FUSED_SHAPES)
def test_conv_fwd_bn_sums(rn, mode_name, shape):
    bf = mode_name == "bf16"
    tol = TOL[mode_name]
    N, H, W, C, K, R, stride, pad = shape
    x = synth.activation_nhwc(SEED, "x", N, C, H, W)
    w = synth.conv_weight_krsc(SEED, "w", K, C, R, R)
    x, w = inputs(mode_name, x, w)
    gamma, beta = _vec("g", K, 0.3, 1.0), _vec("b", K, 0.2, 0.0)
    xd, wd = dev(x, bf), dev(w, bf)
    y, sums = rn.conv_fwd_bn_sums(xd, wd, stride, pad)
    assert torch.equal(y, rn.conv_fwd(xd, wd, stride, pad)), "the sums must not change the convolution"
    assert_close(y, orc.conv_fwd(x, w, stride, pad), tol, "y")
    yh = host(y)
    res = inputs(mode_name, synth.normal(SEED, "r", yh.shape))[0]
    for mode in (0, 1, 2):
        r = res if mode == 2 else None
        z, mean, rstd = rn.bn_relu_fwd_from_sums(y, sums, dev(gamma), dev(beta), dev(r, bf) if r is not None else None,
                                                 1e-5, mode)
        z_o, mean_o, rstd_o = orc.bn_relu_fwd(yh, gamma, beta, r, 1e-5, mode)   # on the GPU path's own y
        if yh.size // K > 1:
            assert_close(z, z_o, tol, f"z mode {mode}")
            assert_close(mean, mean_o, 1e-5, "mean")
            assert_close(rstd, rstd_o, 1e-4, "rstd")
        # and the separate-pass kernels agree to rounding of the float sums
        z_u, mean_u, rstd_u = rn.bn_relu_fwd(y, dev(gamma), dev(beta), dev(r, bf) if r is not None else None, 1e-5, mode)
        assert_close(mean, host(mean_u), 1e-5, "mean vs separate pass")
        assert_close(rstd, host(rstd_u), 1e-5, "rstd vs separate pass")


def test_conv_fwd_bn_sums_large_mean_and_running_stats(rn):
    # all-positive operands: every output channel's mean is many standard deviations from zero and the
    # tiles' shifts differ, so the change of shift in the final sum is exercised
    N, H, W, C, K = 4, 20, 20, 64, 72
    x = np.abs(synth.activation_nhwc(SEED, "x", N, C, H, W)) + 3.0
    w = np.abs(synth.conv_weight_krsc(SEED, "w", K, C, 3, 3)) + 0.05
    g, b = np.ones(K, np.float32), np.zeros(K, np.float32)
    y, sums = rn.conv_fwd_bn_sums(dev(x), dev(w), 1, 1)
    yh = host(y)
    rm0 = synth.normal(SEED, "rm", (K,)); rv0 = np.abs(synth.normal(SEED, "rv", (K,))) + 1
    rm, rv = dev(rm0), dev(rv0)
    z, mean, rstd = rn.bn_relu_fwd_from_sums(y, sums, dev(g), dev(b), None, 1e-5, 0, running_mean=rm, running_var=rv,
                                             momentum=0.9)
    z_o, mean_o, rstd_o = orc.bn_relu_fwd(yh, g, b, None, 1e-5, 0)
    rm_o, rv_o = orc.bn_running_update(yh, rm0, rv0, 0.9)
    assert float(np.min(np.abs(mean_o) * rstd_o)) > 3.0, "the case must have |mean| >> std"
    assert_close(mean, mean_o, 1e-6, "mean")
    assert_close(rstd, rstd_o, 1e-4, "rstd")
    assert_close(z, z_o, 1e-3, "z")
    assert_close(rm, rm_o, 1e-6, "running_mean")
    assert_close(rv, rv_o, 1e-4, "running_var")


DGRAD_SHAPES = [s for s in FUSED_SHAPES if s[3] != 3]


@pytest.mark.parametrize("mode_name", ["f32", "bf16"])
@pytest.mark.parametrize("shape", DGRAD_SHAPES)
def test_conv_dgrad_bn_sums(rn, mode_name, shape):
    bf = mode_name == "bf16"
    tol = TOL[mode_name]
    N, H, W, C, K, R, stride, pad = shape
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - R) // stride + 1
    # the BN layer below the convolution: input bx [N,H,W,C], output z feeds the convolution
    bx = synth.activation_nhwc(SEED, "bx", N, C, H, W) * 1.3 + 0.2
    dy = synth.activation_nhwc(SEED, "dy", N, K, P, Q)
    w = synth.conv_weight_krsc(SEED, "w", K, C, R, R)
    bx, dy, w = inputs(mode_name, bx, dy, w)
    gamma, beta = _vec("g", C, 0.3, 1.0), _vec("b", C, 0.2, 0.0)
    z_o, mean_o, rstd_o = orc.bn_relu_fwd(bx, gamma, beta, None, 1e-5, 1)
    z_o = inputs(mode_name, z_o)[0]
    dyd, wd, bxd = dev(dy, bf), dev(w, bf), dev(bx, bf)
    gd, bd = dev(gamma), dev(beta)
    # The backward kernels recompute the ReLU decision from bx: with the GPU forward pass's statistics that is
    # that pass's decision bit for bit, which is recorded here and imposed on the oracle's backward pass wherever a
    # pre-activation within rounding of zero landed on the other side.
    bits = rn.relu_mask_like(bxd)
    _, md, rd = rn.bn_relu_fwd(bxd, gd, bd, None, 1e-5, 1, relu_mask=bits)
    assert_close(md, mean_o, 1e-5, "mean")
    assert_close(rd, rstd_o, 1e-4, "rstd")
    z_o, _ = impose_relu_decisions(z_o, bits)
    dz, sums = rn.conv_dgrad_bn_sums(dyd, wd, (N, H, W, C), stride, pad, bxd, gd, bd, md, rd)
    assert torch.equal(dz, rn.conv_dgrad(dyd, wd, (N, H, W, C), stride, pad)), "the sums must not change the gradient"
    assert_close(dz, orc.conv_dgrad(dy, w, (N, H, W, C), stride, pad), tol, "dz")
    dx, _, dg, db = rn.bn_relu_bwd_from_sums(dz, bxd, sums, gd, bd, md, rd)
    dx_o, _, dg_o, db_o = orc.bn_relu_bwd(host(dz).astype(np.float32), bx, z_o, gamma, mean_o, rstd_o, 1)
    if N * H * W > 1:
        assert_close(dx, dx_o, tol, "dx")
        assert_close(dg, dg_o, tol, "dgamma")
        assert_close(db, db_o, tol, "dbeta")
    # the separate-pass kernels (same mask rule) agree to rounding of the float sums
    dx_u, _, dg_u, db_u = rn.bn_relu_bwd(dz, bxd, None, gd, md, rd, 1, beta=bd)
    assert_close(dg, host(dg_u), 1e-5, "dgamma vs separate pass")
    assert_close(db, host(db_u), 1e-5, "dbeta vs separate pass")
    assert_close(dx, host(dx_u), max(1e-5, tol / 4), "dx vs separate pass")


@pytest.mark.parametrize("mode_name", ["f32", "bf16"])
@pytest.mark.parametrize("shape", DGRAD_SHAPES)
def test_conv_dgrad_bn_sums_residual_layer_with_addend(rn, mode_name, shape):
    """The BN layer below is a residual-add layer (mode 2) whose output has a second consumer: the data
    gradient adds that consumer's gradient (one rounding of the sum), takes the mask from the recorded bits."""
    bf = mode_name == "bf16"
    tol = TOL[mode_name]
    N, H, W, C, K, R, stride, pad = shape
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - R) // stride + 1
    bx = synth.activation_nhwc(SEED, "bx", N, C, H, W) * 1.3 + 0.2
    res = synth.activation_nhwc(SEED, "res", N, C, H, W)
    dy = synth.activation_nhwc(SEED, "dy", N, K, P, Q)
    add = synth.activation_nhwc(SEED, "add", N, C, H, W) * 0.7
    w = synth.conv_weight_krsc(SEED, "w", K, C, R, R)
    bx, res, dy, add, w = inputs(mode_name, bx, res, dy, add, w)
    gamma, beta = _vec("g", C, 0.3, 1.0), _vec("b", C, 0.2, 0.0)
    bxd, resd = dev(bx, bf), dev(res, bf)
    gd, bd = dev(gamma), dev(beta)
    bits = rn.relu_mask_like(bxd)
    z, md, rd = rn.bn_relu_fwd(bxd, gd, bd, resd, 1e-5, 2, relu_mask=bits)      # the layer's own forward pass
    dz, sums = rn.conv_dgrad_bn_sums(dev(dy, bf), dev(w, bf), (N, H, W, C), stride, pad, bxd, gd, bd, md, rd,
                                     addend=dev(add, bf), relu_mask=bits)
    want = orc.conv_dgrad(dy, w, (N, H, W, C), stride, pad) + add
    assert_close(dz, want, tol, "dz = data gradient + addend")
    if bf:   # one rounding of the float sum: never further from it than rounding the exact sum twice would be
        plain = host(rn.conv_dgrad(dev(dy, bf), dev(w, bf), (N, H, W, C), stride, pad))
        assert orc.rel_l2(host(dz), want) <= orc.rel_l2(synth.round_bf16(plain + add), want) * 1.05 + 1e-7
    dx, dres, dg, db = rn.bn_relu_bwd_from_sums(dz, bxd, sums, gd, bd, md, rd, mode=2, relu_mask=bits)
    dx_o, dres_o, dg_o, db_o = orc.bn_relu_bwd(host(dz).astype(np.float32), bx, host(z), gamma, host(md), host(rd), 2)
    if N * H * W > 1:
        assert_close(dx, dx_o, tol, "dx")
        assert_close(dres, dres_o, tol, "dresidual")
        assert_close(dg, dg_o, max(tol, 1e-3), "dgamma")
        assert_close(db, db_o, max(tol, 1e-3), "dbeta")
    # an addend that counts only under recorded ReLU bits (the identity shortcut's gradient, taken without
    # a masked copy) gives the bits of the call with the masked tensor
    V = 8 if bf else 4
    rng = np.random.default_rng(11)
    abits = rng.integers(0, 1 << V, size=add.size // V).astype(np.uint8)
    keep = ((abits[:, None] >> np.arange(V)[None, :]) & 1).astype(add.dtype).reshape(add.shape)
    nbytes = rn.conv_bn_sums_bytes(rn.ConvDesc(N, H, W, C, K, R, R, stride, pad, rn.BF16 if bf else rn.F32))
    zeros = lambda: torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    dz_m, sums_m = rn.conv_dgrad_bn_sums(dev(dy, bf), dev(w, bf), (N, H, W, C), stride, pad, bxd, gd, bd, md, rd,
                                         addend=dev(add, bf), relu_mask=bits, addend_mask=dev(abits), sums=zeros())
    dz_p, sums_p = rn.conv_dgrad_bn_sums(dev(dy, bf), dev(w, bf), (N, H, W, C), stride, pad, bxd, gd, bd, md, rd,
                                         addend=dev(add * keep, bf), relu_mask=bits, sums=zeros())
    assert torch.equal(dz_m, dz_p) and torch.equal(sums_m[1], sums_p[1])
    # the separate-pass kernels agree to rounding of the float sums
    dx_u, dres_u, dg_u, db_u = rn.bn_relu_bwd(dz, bxd, z, gd, md, rd, 2, beta=bd)
    assert torch.equal(dres, dres_u)
    assert_close(dg, host(dg_u), 1e-5, "dgamma vs separate pass")
    assert_close(db, host(db_u), 1e-5, "dbeta vs separate pass")
    assert_close(dx, host(dx_u), max(1e-5, tol / 4), "dx vs separate pass")


def test_fused_sums_reproducible_and_independent_of_buffer_contents(rn):
    N, H, W, C, K = 6, 28, 28, 64, 128
    x = dev(synth.activation_nhwc(SEED, "x", N, C, H, W), True)
    w = dev(synth.conv_weight_krsc(SEED, "w", K, C, 3, 3), True)
    g, b = dev(_vec("g", K, 0.3, 1.0)), dev(_vec("b", K, 0.2, 0.0))
    d = rn.ConvDesc(N, H, W, C, K, 3, 3, 1, 1, rn.BF16)
    outs = []
    for fill in (0, 0xFF):
        sums = torch.full((rn.conv_bn_sums_bytes(d),), fill, dtype=torch.uint8, device="cuda")
        y, h = rn.conv_fwd_bn_sums(x, w, 1, 1, sums=sums)
        outs.append(rn.bn_relu_fwd_from_sums(y, h, g, b, None, 1e-5, 1))
    for a, c in zip(*outs):
        assert torch.equal(a, c)


def test_fused_abi_errors(rn):
    N, H, W, C, K = 2, 8, 8, 16, 16
    x = dev(synth.activation_nhwc(SEED, "x", N, C, H, W), True)
    w = dev(synth.conv_weight_krsc(SEED, "w", K, C, 1, 1), True)
    g, b = dev(np.ones(K, np.float32)), dev(np.zeros(K, np.float32))
    small = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(rn.Rn50Error) as e:
        rn.conv_fwd_bn_sums(x, w, 1, 0, sums=small)
    assert e.value.code == -3                                   # RN50_ERR_WORKSPACE
    y, h = rn.conv_fwd_bn_sums(x, w, 1, 0)
    other = (rn.ConvDesc(N, H, W, C, 2 * K, 1, 1, 1, 0, rn.BF16), h[1])
    with pytest.raises(rn.Rn50Error) as e:
        rn.bn_relu_fwd_from_sums(y, other, g, b)
    assert e.value.code == -1                                   # RN50_ERR_INVALID: not this layer's producer
    with pytest.raises(rn.Rn50Error) as e:
        rn.bn_relu_fwd_from_sums(y, h, g, b, None, 1e-5, 2)     # mode 2 without residual
    assert e.value.code == -1
    # addend_mask without addend: rejected before the first launch, so workspace, dx and sums stay as they were
    dy = dev(synth.activation_nhwc(SEED, "dy", N, K, H, W), True)
    mask = torch.full((N * H * W * C // 8,), 0xff, dtype=torch.uint8, device="cuda")
    d = rn.ConvDesc(N, H, W, C, K, 1, 1, 1, 0, rn.BF16)
    wsb = torch.full((rn.conv_dgrad_workspace_bytes(d),), 0x5a, dtype=torch.uint8, device="cuda")
    sums = torch.full((rn.conv_bn_sums_bytes(d),), 0x5a, dtype=torch.uint8, device="cuda")
    dx = torch.full((N, H, W, C), 3.0, dtype=torch.bfloat16, device="cuda")
    gc, bc = dev(np.ones(C, np.float32)), dev(np.zeros(C, np.float32))
    with pytest.raises(rn.Rn50Error) as e:
        rn.conv_dgrad_bn_sums(dy, w, (N, H, W, C), 1, 0, x, gc, bc, bc, gc, dx=dx, workspace=wsb, sums=sums,
                              addend=None, addend_mask=mask)
    assert e.value.code == -1
    torch.cuda.synchronize()
    assert bool((wsb == 0x5a).all()) and bool((sums == 0x5a).all()) and bool((dx == 3.0).all())


# ------------------------------------------------- BN+ReLU applied in the consumer convolution's operand load
BN_IN_SHAPES = [(2, 9, 7, 24, 40), (3, 14, 14, 64, 256), (40, 14, 14, 256, 1024), (2, 8, 8, 72, 136), (40, 7, 7, 512, 2048),
                (1, 5, 5, 8, 8)]


@pytest.mark.parametrize("mode_name", ["f32", "bf16"])
@pytest.mark.parametrize("shape", BN_IN_SHAPES)
def test_conv_bn_in_equals_the_unfused_pair_and_the_oracle(rn, mode_name, shape):
    """conv_fwd_bn_in / conv_wgrad_bn_in read the BN layer's INPUT and apply BN+ReLU on the fly: bit for bit the
    convolution of the tensor bn_relu_fwd stores, and that tensor's convolution by the oracle at the mode's bar."""
    N, H, W, C, K = shape
    bf = mode_name == "bf16"
    if not bf and (C % 4 or K % 4):
        pytest.skip("channel counts must be multiples of the 16-byte vector")
    if bf and (C % 8 or K % 8):
        pytest.skip("channel counts must be multiples of the 16-byte vector")
    x, w, dy = inputs(mode_name, synth.activation_nhwc(SEED, "x", N, C, H, W) * 1.5 + 0.3,
                      synth.conv_weight_krsc(SEED, "w", K, C, 1, 1), synth.activation_nhwc(SEED, "dy", N, K, H, W))
    gamma = (1.0 + 0.2 * synth.normal(SEED, "g", (C,))).astype(np.float32)
    beta = (0.1 * synth.normal(SEED, "b", (C,))).astype(np.float32)
    xd, wd, dyd, gd, bd = dev(x, bf), dev(w, bf), dev(dy, bf), dev(gamma), dev(beta)
    z, mean, rstd = rn.bn_relu_fwd(xd, gd, bd, None, 1e-5, 1)
    y_ref = rn.conv_fwd(z, wd, 1, 0)
    dw_ref = rn.conv_wgrad(z, dyd, wd.shape, 1, 0)
    y, handle = rn.conv_fwd_bn_in(xd, gd, bd, mean, rstd, wd, with_sums=True)
    dw = rn.conv_wgrad_bn_in(xd, gd, bd, mean, rstd, dyd, wd.shape)
    torch.cuda.synchronize()
    assert torch.equal(y, y_ref), "forward differs from the convolution of the stored BN output"
    assert torch.equal(dw, dw_ref), "weight gradient differs from that of the stored BN output"
    assert_close(y, orc.conv_fwd(host(z), host(wd), 1, 0), TOL[mode_name], "y")
    assert_close(dw, orc.conv_wgrad(host(z), host(dyd), tuple(wd.shape), 1, 0), TOL[mode_name], "dw")
    # the sums it leaves for the BN layer behind it are those of conv_fwd_bn_sums on the stored tensor
    g2, b2 = dev(np.ones(K, np.float32)), dev(np.zeros(K, np.float32))
    z2, m2, r2 = rn.bn_relu_fwd_from_sums(y, handle, g2, b2)
    y3, h3 = rn.conv_fwd_bn_sums(z, wd, 1, 0)
    z3, m3, r3 = rn.bn_relu_fwd_from_sums(y3, h3, g2, b2)
    assert torch.equal(z2, z3) and torch.equal(m2, m3) and torch.equal(r2, r3)


def test_conv_bn_in_rejects_other_filters(rn):
    x = torch.zeros((1, 8, 8, 16), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((16, 3, 3, 16), dtype=torch.bfloat16, device="cuda")
    v = torch.ones(16, device="cuda")
    d = rn.ConvDesc(1, 8, 8, 16, 16, 3, 3, 1, 1, rn.BF16)
    import ctypes
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    rc = rn.raw.conv_fwd_bn_in(ctypes.byref(d), p(x), p(v), p(v), p(v), p(v), p(w), p(x), None, ctypes.c_size_t(0), None)
    assert rc == -2 and b"1x1" in rn.raw.rn50_last_error()
