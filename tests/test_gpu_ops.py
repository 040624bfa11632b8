"""GPU parity: BN(+ReLU,+add), pooling, classifier, loss and LARS kernels against the oracle,
called through the C ABI (ctypes binding)."""
import numpy as np
import pytest
import torch

import oracle as orc
import synth
from oracle import net
from gpu_util import impose_relu_decisions, TOL, assert_close, dev, host, inputs

pytestmark = pytest.mark.gpu
SEED = synth.DEFAULT_SEED


@pytest.fixture(scope="module")
def rn():
    import paper_1903_12650_amd as rn
    return rn


BN_SHAPES = [(2, 56, 56, 64), (3, 7, 7, 2048), (2, 13, 9, 24), (1, 1, 1, 8), (5, 28, 28, 128), (1, 3, 67, 40)]


@pytest.mark.parametrize("mode_name", ["f32", "bf16"])
@pytest.mark.parametrize("shape", BN_SHAPES)
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_bn_fwd_bwd(rn, mode_name, shape, mode):
    bf = mode_name == "bf16"
    N, H, W, C = shape
    x = synth.activation_nhwc(SEED, "x", N, C, H, W) * 1.7 + 0.4
    res = synth.activation_nhwc(SEED, "r", N, C, H, W)
    dz = synth.activation_nhwc(SEED, "dz", N, C, H, W)
    dz2 = synth.activation_nhwc(SEED, "dz2", N, C, H, W)
    x, res, dz, dz2 = inputs(mode_name, x, res, dz, dz2)
    gamma = (1 + 0.3 * synth.normal(SEED, "g", (C,))).astype(np.float32)
    beta = (0.2 * synth.normal(SEED, "b", (C,))).astype(np.float32)
    r = res if mode == 2 else None
    y_o, mean_o, rstd_o = orc.bn_relu_fwd(x, gamma, beta, r, 1e-5, mode)
    y, mean, rstd = rn.bn_relu_fwd(dev(x, bf), dev(gamma), dev(beta), dev(r, bf) if r is not None else None, 1e-5, mode)
    tol = TOL[mode_name]
    m = N * H * W
    if m > 1:
        assert_close(y, y_o, tol, "y")
        assert_close(mean, mean_o, 1e-5, "mean")
        assert_close(rstd, rstd_o, 1e-4, "rstd")
    # backward on the oracle's own forward values (z = oracle output in the storage type)
    z_o = inputs(mode_name, y_o)[0]
    for use_z, use_dz2 in [(True, False), (mode != 2, True)]:
        dzsum = (dz + dz2) if use_dz2 else dz
        dx_o, dres_o, dg_o, db_o = orc.bn_relu_bwd(dzsum, x, z_o, gamma, mean_o, rstd_o, mode)
        zt = dev(z_o, bf) if (use_z or mode == 2) else None
        mean_b, rstd_b = dev(mean_o), dev(rstd_o)
        if zt is None and mode == 1:
            # The ReLU decision is recomputed from x.  It is the forward pass's decision bit for bit when it is
            # given that pass's statistics, so those decisions (recorded as bits) are imposed on the oracle's
            # backward pass wherever a pre-activation within rounding of zero landed on the other side.
            bits = rn.relu_mask_like(dev(x, bf))
            _, mean_b, rstd_b = rn.bn_relu_fwd(dev(x, bf), dev(gamma), dev(beta), None, 1e-5, mode, relu_mask=bits)
            z_imp, _ = impose_relu_decisions(z_o, bits)
            dx_o, dres_o, dg_o, db_o = orc.bn_relu_bwd(dzsum, x, z_imp, gamma, mean_o, rstd_o, mode)
        dx, dres, dg, db = rn.bn_relu_bwd(dev(dz, bf), dev(x, bf), zt, dev(gamma), mean_b, rstd_b, mode,
                                          beta=dev(beta), dz2=dev(dz2, bf) if use_dz2 else None)
        if m > 1:
            assert_close(dx, dx_o, tol, "dx")
            assert_close(dg, dg_o, tol, "dgamma")
            assert_close(db, db_o, tol, "dbeta")
            if mode == 2:
                assert_close(dres, dres_o, tol, "dres")


@pytest.mark.parametrize("mode_name", ["f32", "bf16"])
@pytest.mark.parametrize("mode", [1, 2])
def test_bn_relu_mask_bits_replace_z(rn, mode_name, mode):
    """The recorded ReLU decision bits (one byte per 16-byte vector) are exactly z > 0, and the backward
    pass gives bit-identical results from them and from z."""
    bf = mode_name == "bf16"
    N, H, W, C = 3, 9, 11, 40
    x = synth.activation_nhwc(SEED, "x", N, C, H, W) * 1.3 + 0.1
    res = synth.activation_nhwc(SEED, "r", N, C, H, W)
    dz = synth.activation_nhwc(SEED, "dz", N, C, H, W)
    x, res, dz = inputs(mode_name, x, res, dz)
    gamma = (1 + 0.3 * synth.normal(SEED, "g", (C,))).astype(np.float32)
    beta = (0.2 * synth.normal(SEED, "b", (C,))).astype(np.float32)
    xd, rd = dev(x, bf), (dev(res, bf) if mode == 2 else None)
    bits = rn.relu_mask_like(xd)
    z, mean, rstd = rn.bn_relu_fwd(xd, dev(gamma), dev(beta), rd, 1e-5, mode, relu_mask=bits)
    V = 8 if bf else 4
    zh = host(z).reshape(-1, V)
    want = ((zh > 0).astype(np.int64) << np.arange(V)).sum(1)
    assert np.array_equal(bits.cpu().numpy().astype(np.int64), want)
    a = rn.bn_relu_bwd(dev(dz, bf), xd, z, dev(gamma), mean, rstd, mode, beta=dev(beta))
    b = rn.bn_relu_bwd(dev(dz, bf), xd, None, dev(gamma), mean, rstd, mode, beta=dev(beta), relu_mask=bits)
    for u, v in zip(a, b):
        assert (u is None and v is None) or torch.equal(u, v)


def test_bn_running_stats_and_large_mean(rn):
    N, H, W, C = 4, 14, 14, 32
    x = synth.activation_nhwc(SEED, "x", N, C, H, W) * 0.05 + 30.0          # mean >> std: shifted sums must cope
    g = np.ones(C, np.float32); b = np.zeros(C, np.float32)
    rm0 = synth.normal(SEED, "rm", (C,)); rv0 = np.abs(synth.normal(SEED, "rv", (C,))) + 1
    rm_o, rv_o = orc.bn_running_update(x, rm0, rv0, 0.9)
    rm, rv = dev(rm0), dev(rv0)
    y, mean, rstd = rn.bn_relu_fwd(dev(x), dev(g), dev(b), None, 1e-5, 0, running_mean=rm, running_var=rv, momentum=0.9)
    y_o, mean_o, rstd_o = orc.bn_relu_fwd(x, g, b, None, 1e-5, 0)
    assert_close(rstd, rstd_o, 1e-3, "rstd")
    assert_close(y, y_o, 2e-3, "y")
    assert_close(rm, rm_o, 1e-6, "running_mean")
    assert_close(rv, rv_o, 1e-3, "running_var")


def test_bn_bitwise_reproducible(rn):
    x = dev(synth.activation_nhwc(SEED, "x", 8, 64, 56, 56), True)
    g = dev(np.ones(64, np.float32)); b = dev(np.zeros(64, np.float32))
    a = rn.bn_relu_fwd(x, g, b, None, 1e-5, 1)
    c = rn.bn_relu_fwd(x, g, b, None, 1e-5, 1)
    for u, v in zip(a, c):
        assert torch.equal(u, v)


@pytest.mark.parametrize("mode_name", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(2, 112, 112, 64), (1, 9, 7, 8), (2, 8, 8, 16), (1, 1, 1, 8), (1, 2, 5, 24)])
def test_maxpool(rn, mode_name, shape):
    bf = mode_name == "bf16"
    N, H, W, C = shape
    x = np.maximum(synth.activation_nhwc(SEED, "x", N, C, H, W), 0)        # post-ReLU: many ties at 0
    x, = inputs("bf16", x)                                                  # coarse values: ties between positives too
    y_o = orc.maxpool_fwd(x)
    dy = synth.activation_nhwc(SEED, "dy", N, C, y_o.shape[1], y_o.shape[2])
    dy2 = synth.activation_nhwc(SEED, "dy2", N, C, y_o.shape[1], y_o.shape[2])
    dy, dy2 = inputs(mode_name, dy, dy2)
    y = rn.maxpool_fwd(dev(x, bf))
    assert np.array_equal(host(y), y_o)
    dx = rn.maxpool_bwd(dev(x, bf), dev(dy, bf))
    assert_close(dx, orc.maxpool_bwd(x, dy), 1e-6 if not bf else 4e-3, "dx")
    dx2 = rn.maxpool_bwd(dev(x, bf), dev(dy, bf), dev(dy2, bf))
    assert_close(dx2, orc.maxpool_bwd(x, dy + dy2), 1e-6 if not bf else 4e-3, "dx(dy+dy2)")
    # the recorded-winner path: same winners as the oracle's index, same gradients bit for bit
    y2, am = rn.maxpool_fwd(dev(x, bf), return_argmax=True)
    _, idx_o = orc.maxpool_fwd(x, return_index=True)
    P, Q = y_o.shape[1:3]
    pp, qq = np.meshgrid(np.arange(P), np.arange(Q), indexing="ij")
    am_h = host(am).astype(np.int64)
    ih = (2 * pp - 1)[None, :, :, None] + am_h // 3
    iw = (2 * qq - 1)[None, :, :, None] + am_h % 3
    assert np.array_equal(ih * W + iw, idx_o) and torch.equal(y2, y)
    assert torch.equal(rn.maxpool_bwd(dev(x, bf), dev(dy, bf), dev(dy2, bf), argmax=am), dx2)


@pytest.mark.parametrize("mode_name", ["f32", "bf16"])
def test_avgpool_fc_xent_chain(rn, mode_name):
    bf = mode_name == "bf16"
    tol = TOL[mode_name]
    N, H, W, C, K = 40, 7, 7, 2048, 1000
    x = np.maximum(synth.activation_nhwc(SEED, "x", N, C, H, W), 0)
    Wt = synth.normal(SEED, "W", (K, C), np.sqrt(2.0 / C)); b = 0.1 * synth.normal(SEED, "b", (K,))
    x, Wt = inputs(mode_name, x, Wt)
    lab = synth.labels(SEED, "lab", N, K)
    a_o = orc.avgpool_fwd(x)
    a = rn.avgpool_fwd(dev(x, bf))
    assert_close(a, a_o, tol, "avgpool")
    a_in = inputs(mode_name, a_o)[0]
    lo = orc.fc_fwd(a_in, Wt, b)
    logits = rn.fc_fwd(dev(a_in, bf), dev(Wt, bf), dev(b))
    assert_close(logits, lo, 1e-5, "logits")
    for ls, gs in [(0.0, 1.0), (0.1, 128.0)]:
        loss_o, row_o, dl_o = orc.xent_fwd_bwd(lo, lab, ls, gs)
        loss, row, dl = rn.xent_fwd_bwd(dev(lo), dev(lab), ls, gs)
        assert abs(float(loss.item()) - loss_o) < 1e-5 * abs(loss_o)
        assert_close(row, row_o, 1e-5, "row_loss")
        assert_close(dl, dl_o, 1e-5, "dlogits")
        assert float(dl.sum(dim=1).abs().max()) < 1e-5 * gs
    da_o, dW_o, db_o = orc.fc_bwd(a_in, Wt, dl_o)
    da, dW, db = rn.fc_bwd(dev(a_in, bf), dev(Wt, bf), dev(dl_o))
    assert_close(da, da_o, tol, "da"); assert_close(dW, dW_o, 1e-5, "dW"); assert_close(db, db_o, 1e-5, "db")
    da_in = inputs(mode_name, da_o)[0]
    dx = rn.avgpool_bwd(dev(da_in, bf), H, W)
    assert_close(dx, orc.avgpool_bwd(da_in, H, W), tol, "avgpool_bwd")


def test_xent_edge_cases(rn):
    K = 1000
    l = np.full((3, K), 0.37, np.float32)
    loss, row, dl = rn.xent_fwd_bwd(dev(l), dev(np.array([0, 999, 5], np.int32)), 0.1, 1.0)
    assert abs(float(loss.item()) - np.log(1000.0)) < 1e-5                   # uniform logits: ln K
    l = np.zeros((2, 5), np.float32); l[0, 1] = 1e4; l[1, 2] = -1e4           # huge logits stay finite
    loss, row, dl = rn.xent_fwd_bwd(dev(l), dev(np.array([1, 2], np.int32)), 0.0, 1.0)
    lo, ro, dlo = orc.xent_fwd_bwd(l, np.array([1, 2], np.int32), 0.0, 1.0)
    assert torch.isfinite(dl).all() and abs(float(loss.item()) - lo) < 1e-3 * lo
    loss, row, dl = rn.xent_fwd_bwd(dev(np.array([[0.3]], np.float32)), dev(np.array([0], np.int32)), 0.0, 1.0)
    assert float(loss.item()) == 0.0 and float(dl.abs().max()) == 0.0          # one class


def test_fc_ragged_sizes(rn):
    N, C, K = 5, 72, 37
    a = synth.normal(SEED, "a", (N, C)); W = synth.normal(SEED, "W", (K, C)); b = synth.normal(SEED, "b", (K,))
    dl = synth.normal(SEED, "dl", (N, K))
    assert_close(rn.fc_fwd(dev(a), dev(W), dev(b)), orc.fc_fwd(a, W, b), 1e-6, "logits")
    da, dW, db = rn.fc_bwd(dev(a), dev(W), dev(dl))
    da_o, dW_o, db_o = orc.fc_bwd(a, W, dl)
    assert_close(da, da_o, 1e-6, "da"); assert_close(dW, dW_o, 1e-6, "dW"); assert_close(db, db_o, 1e-6, "db")


@pytest.mark.parametrize("shape", [(40, 2048, 1000), (5, 80, 37), (64, 48, 64), (33, 144, 100), (1, 16, 8)])
def test_fc_fwd_bf16_matrix_core_path(rn, shape):
    """bf16 operands, batch <= 64, channels a multiple of 16: the classifier's forward runs on the matrix cores
    (float accumulation of exact bf16 products: float-level agreement with the oracle on the same rounded inputs)."""
    N, C, K = shape
    a = synth.round_bf16(synth.normal(SEED, "a", (N, C)))
    W = synth.round_bf16(synth.normal(SEED, "W", (K, C)) * 0.05)
    b = synth.normal(SEED, "b", (K,))
    got = rn.fc_fwd(dev(a, True), dev(W, True), dev(b))
    assert got.dtype == torch.float32 and tuple(got.shape) == (N, K)
    assert_close(got, orc.fc_fwd(a, W, b), 1e-5, "logits")


# ------------------------------------------------------------------------ LARS
def _lars_case(rn, table, grad_bf16=False, with_lowp=True, v_zero=True, apply_trust=None, eps=0.0):
    params = synth.params_from_table(SEED, table)
    grads = synth.grads_from_table(SEED, table, 1e-3)
    if grad_bf16:
        grads = [synth.round_bf16(g) for g in grads]
    vel = [np.zeros_like(p) if v_zero else synth.normal(SEED, "v" + n, p.shape, 1e-3) for p, (n, _, _) in zip(params, table)]
    wds = net.lars_hyper(table, 5e-5)
    w_o, v_o, norms_o = orc.lars_update(params, grads, vel, 0.001, 0.9, 1.0, wds, eps, apply_trust)
    # pack every tensor into one arena per kind, 256-byte aligned offsets (as the step does)
    offs, tot = [], 0
    for p in params:
        offs.append(tot); tot += (p.size + 63) // 64 * 64
    def arena(arrs, bf=False):
        a = np.zeros(tot, np.float32)
        for o, p in zip(offs, arrs):
            a[o:o + p.size] = p.ravel()
        return dev(a, bf)
    W, G, V = arena(params), arena(grads, grad_bf16), arena(vel)
    L = torch.zeros(tot, dtype=torch.bfloat16, device="cuda") if with_lowp else None
    sl = lambda A: [A[o:o + p.size] for o, p in zip(offs, params)]
    tab = rn.LarsTable(sl(W), sl(G), sl(V), wds, apply_trust, sl(L) if with_lowp else None)
    norms = torch.zeros(len(table) * 2, dtype=torch.float32, device="cuda")
    rn.lars_update(tab, 0.001, 0.9, 1.0, eps, norms_out=norms)
    torch.cuda.synchronize()
    nh = host(norms).reshape(-1, 2)
    worst = 0.0
    for t, (name, _, _) in enumerate(table):
        w, v = host(sl(W)[t]), host(sl(V)[t])
        worst = max(worst, assert_close(w, w_o[t].ravel(), TOL["lars"], name + " w"))
        assert_close(v, v_o[t].ravel(), TOL["lars"] if not grad_bf16 else 1e-6, name + " v")
        assert abs(nh[t, 0] - norms_o[t, 0]) <= 1e-6 * norms_o[t, 0] + 1e-30, name
        assert abs(nh[t, 1] - norms_o[t, 1]) <= 1e-6 * norms_o[t, 1], name
        if with_lowp:
            assert np.array_equal(host(sl(L)[t]), synth.round_bf16(w)), name
    # padding between tensors is untouched
    Wh = host(W)
    for o, p in zip(offs, params):
        pad = Wh[o + p.size:(o + p.size + 63) // 64 * 64]
        assert not pad.any()
    return worst


def test_lars_resnet50_table(rn):
    """BASELINE config 2: the 161 tensors of ResNet-50 (25.56M parameters)."""
    table = net.param_table()
    worst = _lars_case(rn, table)
    print("worst rel-L2 on w_new over 161 tensors: %.2e" % worst)


def test_lars_variants(rn):
    table = [("a.w", (5, 3, 3, 7), "conv"), ("a.gamma", (5,), "gamma"), ("a.beta", (5,), "beta"),
             ("b.w", (300, 1, 1, 129), "conv"), ("c.w", (17, 8193), "fcw"), ("c.b", (17,), "fcb"),
             ("d.w", (1, 1, 1, 1), "conv")]
    _lars_case(rn, table, v_zero=False)
    _lars_case(rn, table, grad_bf16=True, v_zero=False)
    _lars_case(rn, table, with_lowp=False, apply_trust=[1, 0, 0, 1, 1, 0, 1], eps=1e-3)


def test_lars_many_tensors_needs_two_launches(rn):
    table = [(f"t{i}.w", (3 + i % 5, 1, 1, 4), "conv") for i in range(700)]
    _lars_case(rn, table, v_zero=False)


def test_abi_error_codes(rn):
    import ctypes
    x = torch.zeros((2, 4, 4, 12), dtype=torch.bfloat16, device="cuda")        # C=12 not a multiple of 8
    g = torch.ones(12, device="cuda")
    with pytest.raises(rn.Rn50Error) as e:
        rn.bn_relu_fwd(x, g, g, None, 1e-5, 1)
    assert e.value.code == -2
    x = torch.zeros((2, 4, 4, 16), dtype=torch.bfloat16, device="cuda")
    g = torch.ones(16, device="cuda")
    with pytest.raises(rn.Rn50Error) as e:
        rn.bn_relu_fwd(x, g, g, None, 1e-5, 2)                                   # mode 2 without residual
    assert e.value.code == -1
    with pytest.raises(rn.Rn50Error) as e:
        rn.bn_relu_fwd(x, g, g, None, 1e-5, 1, workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert e.value.code == -3
    with pytest.raises(rn.Rn50Error) as e:
        rn.xent_fwd_bwd(torch.zeros((0, 5), device="cuda"), torch.zeros(0, dtype=torch.int32, device="cuda"))
    assert e.value.code == -1
    with pytest.raises(rn.Rn50Error) as e:                                      # misaligned activation pointer
        rn.bn_relu_fwd(x.view(-1)[8 * 3:8 * 3 + 2 * 4 * 3 * 16].view(2, 4, 3, 16)[..., :], g, g, None, 1e-5, 1) \
            if x.view(-1)[8 * 3:].data_ptr() % 16 else (_ for _ in ()).throw(rn.Rn50Error(-4, "aligned by chance"))
    assert e.value.code == -4
