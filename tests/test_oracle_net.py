"""Pins for the oracle's network wiring (ResNet-50 v1.5) and the whole training step."""
import numpy as np
import pytest

import oracle as orc
import synth
from oracle import net

SEED = synth.DEFAULT_SEED


def test_parameter_table_counts():
    """161 tensors, 25,557,032 parameters, 53 convolutions (ResNet-50 with a 1000-way head)."""
    t = net.param_table()
    assert len(t) == 161
    assert sum(int(np.prod(s)) for _, s, _ in t) == 25_557_032
    assert sum(k == "conv" for _, _, k in t) == 53
    assert sum(int(np.prod(s)) for _, s, k in t if k == "conv") == 23_454_912
    assert sum(1 for _, s, _ in t if int(np.prod(s)) <= 2048) == 107
    assert t[0][1] == (64, 7, 7, 3) and t[-2][1] == (1000, 2048)


def test_stem_shape_walk():
    """Appendix log: [3(4),224,224] -> (64,112,112) -> max-pool -> (64,56,56)."""
    x = np.zeros((1, 224, 224, 3), np.float32); w = np.zeros((64, 7, 7, 3), np.float32)
    y = orc.conv_fwd(x, w, 2, 3)
    assert y.shape == (1, 112, 112, 64)
    assert orc.maxpool_fwd(y, 3, 2, 1).shape == (1, 56, 56, 64)


SMALL = dict(widths=(4, 6, 8, 10), blocks=(2, 1, 2, 1))


def _small_setup(dtype, N=2, HW=32, classes=7):
    table = net.param_table(SMALL["widths"], SMALL["blocks"], stem=4, classes=classes, in_ch=3, expansion=2)
    params = synth.params_from_table(SEED, table, dtype)
    # non-trivial gamma / beta so that their gradients and the affine step are exercised
    for i, (name, shape, kind) in enumerate(table):
        if kind == "gamma":
            params[i] = (1.0 + 0.3 * synth.normal(SEED, name, shape)).astype(dtype)
        if kind in ("beta", "fcb"):
            params[i] = (0.2 * synth.normal(SEED, name, shape)).astype(dtype)
    images = synth.activation_nhwc(SEED, "img", N, 3, HW, HW, 1.0, dtype)
    labels = synth.labels(SEED, "lab", N, classes)
    return table, params, images, labels


def _torch_forward(images, labels, params, table, blocks, ls, expansion=2, bn_inputs=None):
    """The same network written with torch CPU ops (NCHW, autograd): an independent
    implementation of the wiring and of every operation.  bn_inputs: a list that receives what every
    BN layer normalizes (NHWC numpy arrays, parameter order)."""
    import torch
    import torch.nn.functional as F
    P = [torch.tensor(p, dtype=torch.float64, requires_grad=True) for p in params]
    it = iter(P)

    def cbn(x, stride, pad, relu=True, res=None):
        w, g, b = next(it), next(it), next(it)
        y = F.conv2d(x, w.permute(0, 3, 1, 2), None, stride, pad)
        if bn_inputs is not None:
            bn_inputs.append(y.detach().permute(0, 2, 3, 1).numpy())
        y = F.batch_norm(y, None, None, g, b, True, 0.1, 1e-5)
        if res is not None:
            y = y + res
        return F.relu(y) if relu else y

    x = torch.tensor(images, dtype=torch.float64).permute(0, 3, 1, 2)
    cur = F.max_pool2d(cbn(x, 2, 3), 3, 2, 1)
    for i, nb in enumerate(blocks):
        for j in range(nb):
            stride = 2 if (j == 0 and i > 0) else 1
            inp = cur
            z1 = cbn(inp, 1, 0)
            z2 = cbn(z1, stride, 1)
            # conv3's parameters come before the projection's in parameter order
            w3, g3, b3 = next(it), next(it), next(it)
            if j == 0:
                sc = cbn(inp, stride, 0, relu=False)
            else:
                sc = inp
            c3 = F.conv2d(z2, w3.permute(0, 3, 1, 2))
            if bn_inputs is not None:  # conv3 precedes the projection in parameter order
                bn_inputs.insert(len(bn_inputs) - (1 if j == 0 else 0), c3.detach().permute(0, 2, 3, 1).numpy())
            y3 = F.batch_norm(c3, None, None, g3, b3, True, 0.1, 1e-5)
            cur = F.relu(y3 + sc)
    a = cur.mean(dim=(2, 3))
    fw, fb = next(it), next(it)
    logits = a @ fw.T + fb
    loss = F.cross_entropy(logits, torch.tensor(labels, dtype=torch.long), label_smoothing=ls)
    loss.backward()
    return float(loss.detach()), logits.detach().numpy(), [p.grad.numpy() for p in P]


@pytest.mark.parametrize("ls", [0.0, 0.1])
def test_small_net_matches_torch_autograd(ls):
    table, params, images, labels = _small_setup(np.float64)
    out = net.forward_backward(images, labels, params, SMALL["widths"], SMALL["blocks"], label_smoothing=ls)
    tl, tlogits, tg = _torch_forward(images, labels, params, table, SMALL["blocks"], ls)
    assert abs(out["loss"] - tl) < 1e-10
    np.testing.assert_allclose(out["logits"], tlogits, rtol=1e-8, atol=1e-10)
    for (name, _, _), g, t in zip(table, out["grads"], tg):
        assert orc.rel_l2(g, t) < 1e-7, name


def test_small_net_finite_differences():
    """Central differences of the full loss in a sample of parameter entries (float64 build)."""
    table, params, images, labels = _small_setup(np.float64, N=2, HW=16)
    f = lambda ps: net.forward_backward(images, labels, ps, SMALL["widths"], SMALL["blocks"], label_smoothing=0.1)
    base = f(params)
    rng = np.random.default_rng(0)
    h = 1e-5
    for ti in [0, 1, 2, 3, 7, 12, 13, 14, 21, len(table) - 2, len(table) - 1]:
        p = params[ti]
        for _ in range(2):
            idx = tuple(rng.integers(0, s) for s in p.shape)
            old = p[idx]
            p[idx] = old + h; lp = f(params)["loss"]
            p[idx] = old - h; lm = f(params)["loss"]
            p[idx] = old
            fd = (lp - lm) / (2 * h)
            an = base["grads"][ti][idx]
            assert abs(fd - an) < 1e-6 * max(1.0, abs(an)) + 2e-7, (table[ti][0], idx, fd, an)


def test_conv_weights_orthogonal_to_their_gradient():
    """Every convolution feeds a batch-stat BN, so <w, dL/dw> ~ 0 for all 10+ of them."""
    table, params, images, labels = _small_setup(np.float64, N=3, HW=64)      # m >= 12 everywhere
    out = net.forward_backward(images, labels, params, SMALL["widths"], SMALL["blocks"], eps=1e-13)
    for (name, _, kind), p, g in zip(table, params, out["grads"]):
        if kind == "conv":
            assert abs(np.sum(p * g)) < 1e-6 * np.linalg.norm(p) * np.linalg.norm(g) + 1e-12, name


def test_f32_build_tracks_f64_build_through_the_net():
    table, params, images, labels = _small_setup(np.float32, N=3, HW=64)
    o32 = net.forward_backward(images, labels, params, SMALL["widths"], SMALL["blocks"])
    o64 = net.forward_backward(images.astype(np.float64), labels, [p.astype(np.float64) for p in params],
                               SMALL["widths"], SMALL["blocks"])
    assert abs(o32["loss"] - o64["loss"]) < 1e-5
    for (name, _, _), a, b in zip(table, o32["grads"], o64["grads"]):
        assert orc.rel_l2(a, b) < 2e-4, name      # ReLU masks may flip on a few near-zero values


def test_bottleneck_block_matches_torch():
    """BASELINE config-1 style block (projection shortcut) at a reduced spatial size."""
    import torch
    import torch.nn.functional as F
    N, H, C, Wd = 2, 8, 8, 4
    x = synth.activation_nhwc(SEED, "x", N, C, H, H, 1.0, np.float64)
    shapes = [(Wd, 1, 1, C), (Wd,), (Wd,), (Wd, 3, 3, Wd), (Wd,), (Wd,), (4 * Wd, 1, 1, Wd), (4 * Wd,), (4 * Wd,),
              (4 * Wd, 1, 1, C), (4 * Wd,), (4 * Wd,)]
    p = [synth.normal(SEED, f"p{i}", s, 1.0, np.float64) + (1.5 if len(s) == 1 and i % 3 == 1 else 0) for i, s in enumerate(shapes)]
    T = synth.activation_nhwc(SEED, "T", N, 4 * Wd, H // 2, H // 2, 1.0, np.float64)
    out, tape = net.bottleneck_fwd(x, p, 2, True)
    dx, grads = net.bottleneck_bwd(T, tape)

    tp = [torch.tensor(a, requires_grad=True) for a in p]
    tx = torch.tensor(x.transpose(0, 3, 1, 2).copy(), requires_grad=True)
    bn = lambda y, g, b: F.batch_norm(y, None, None, g, b, True, 0.1, 1e-5)
    cw = lambda w: w.permute(0, 3, 1, 2)
    z1 = F.relu(bn(F.conv2d(tx, cw(tp[0])), tp[1], tp[2]))
    z2 = F.relu(bn(F.conv2d(z1, cw(tp[3]), None, 2, 1), tp[4], tp[5]))
    y3 = bn(F.conv2d(z2, cw(tp[6])), tp[7], tp[8])
    sc = bn(F.conv2d(tx, cw(tp[9]), None, 2, 0), tp[10], tp[11])
    o = F.relu(y3 + sc)
    (o * torch.tensor(T.transpose(0, 3, 1, 2).copy())).sum().backward()
    assert orc.rel_l2(out, o.detach().numpy().transpose(0, 2, 3, 1)) < 1e-12
    assert orc.rel_l2(dx, tx.grad.numpy().transpose(0, 2, 3, 1)) < 1e-9
    for i, (g, t) in enumerate(zip(grads, tp)):
        assert orc.rel_l2(g, t.grad.numpy()) < 1e-9, i


def test_train_step_applies_lars_to_master_weights():
    table, params, images, labels = _small_setup(np.float32)
    model = [synth.round_bf16(p) for p in params]
    vel = [np.zeros_like(p) for p in params]
    out = net.train_step(images, labels, params, model, vel, table, widths=SMALL["widths"], blocks=SMALL["blocks"])
    wds = net.lars_hyper(table, 5e-5)
    assert sum(w > 0 for w in wds) == sum(k in ("conv", "fcw") for _, _, k in table)
    for t in (0, 1, len(table) - 1):
        w, g = params[t].astype(np.float64), out["grads"][t].astype(np.float64)
        wn, gn = np.linalg.norm(w), np.linalg.norm(g)
        local = 0.001 * wn / (gn + wds[t] * wn) if wn > 0 and gn > 0 else 1.0
        np.testing.assert_allclose(out["w_new"][t], w - local * (g + wds[t] * w), rtol=2e-6, atol=1e-9)


def test_round_bf16_helper():
    a = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.14159265, 1e-40, 65504.0], np.float32)
    r = synth.round_bf16(a)
    import torch
    np.testing.assert_array_equal(r, torch.tensor(a).to(torch.bfloat16).to(torch.float32).numpy())
    assert synth.bf16_bits(r).dtype == np.uint16


# ------------------------------------------------------------------ learning-rate control, training loop
def test_learning_rate_warmup_and_decay_patterns():
    """Sec. III-A1: gradual warm-up, then step / polynomial / linear decay -- against hand-computed values."""
    lr = net.learning_rate
    kw = dict(base_lr=8.0, warmup_steps=4, warmup_start_lr=2.0)
    assert [lr(t, **kw) for t in range(6)] == [2.0, 3.5, 5.0, 6.5, 8.0, 8.0]          # linear ramp, then flat
    assert lr(3, base_lr=1.0) == 1.0                                                   # no warm-up, no decay
    st = dict(kw, decay="step", step_every=3, step_factor=0.5)
    assert [lr(t, **st) for t in (4, 6, 7, 9, 10, 13)] == [8.0, 8.0, 4.0, 4.0, 2.0, 1.0]
    po = dict(kw, decay="polynomial", total_steps=14, end_lr=1.0, power=2.0)
    assert lr(4, **po) == 8.0 and lr(14, **po) == 1.0 and lr(40, **po) == 1.0           # ends at end_lr and stays
    assert abs(lr(9, **po) - (1.0 + 7.0 * 0.25)) < 1e-15                                # halfway: (1/2)^2
    li = dict(kw, decay="linear", total_steps=14, end_lr=1.0)
    assert abs(lr(9, **li) - 4.5) < 1e-15 and abs(lr(13, **li) - 1.7) < 1e-12
    assert all(abs(lr(t, **li) - lr(t, **dict(po, power=1.0))) < 1e-15 for t in range(20))
    for sched in (st, po, li):                                                          # never rises after warm-up
        v = [lr(t, **sched) for t in range(4, 30)]
        assert all(a >= b for a, b in zip(v, v[1:]))
    tb = dict(base_lr=0.0, decay="table", table=[0.1, 0.4, 0.2])
    assert [lr(t, **tb) for t in range(5)] == [0.1, 0.4, 0.2, 0.2, 0.2]


def _lars_by_hand(w, g, v, lr, wd, eta=0.001, mu=0.9):
    w = w.astype(np.float64); g = g.astype(np.float64)
    wn, gn = np.sqrt((w * w).sum()), np.sqrt((g * g).sum())
    local = eta * wn / (gn + wd * wn) if wn > 0 and gn > 0 else 1.0
    v = mu * v + lr * local * (g + wd * w)
    return w - v, v


def test_train_loop_matches_torch_autograd_steps_with_handwritten_updates():
    """Three steps over two alternating batches: gradients from torch autograd, the LARS update and the
    moving averages written out here in numpy; the loop must land on the same weights, velocities, losses
    and BN moving averages."""
    table, params, images, labels = _small_setup(np.float64)
    images2 = synth.activation_nhwc(SEED + 1, "img", 2, 3, 32, 32, 1.0, np.float64)
    labels2 = synth.labels(SEED + 1, "lab", 2, 7)
    batches = [(images, labels), (images2, labels2)]
    sched = dict(base_lr=3.0, warmup_steps=2, warmup_start_lr=1.0, decay="linear", total_steps=6, end_lr=0.5)
    out = net.train_loop(batches, params, [np.zeros_like(p) for p in params], table, sched, 3,
                         widths=SMALL["widths"], blocks=SMALL["blocks"], label_smoothing=0.1)
    assert out["lrs"] == [1.0, 2.0, 3.0]
    wds = net.lars_hyper(table, 5e-5)
    n_bn = sum(k == "gamma" for _, _, k in table)
    w = [p.copy() for p in params]
    v = [np.zeros_like(p) for p in params]
    rm = [0.0] * n_bn
    rv = [1.0] * n_bn
    for t in range(3):
        ys = []
        tl, _, tg = _torch_forward(*batches[t % 2], w, table, SMALL["blocks"], 0.1, bn_inputs=ys)
        assert abs(out["losses"][t] - tl) < 1e-9
        assert len(ys) == n_bn
        for i, y in enumerate(ys):
            y2 = y.reshape(-1, y.shape[-1])
            rm[i] = 0.9 * rm[i] + 0.1 * y2.mean(0)
            rv[i] = 0.9 * rv[i] + 0.1 * y2.var(0)   # biased variance
        for i in range(len(w)):
            w[i], v[i] = _lars_by_hand(w[i], tg[i], v[i], out["lrs"][t], wds[i])
    for i, (name, _, _) in enumerate(table):
        assert orc.rel_l2(out["master"][i], w[i]) < 1e-7, name
        assert orc.rel_l2(out["velocity"][i], v[i]) < 1e-6, name
    for i in range(n_bn):
        np.testing.assert_allclose(out["running_mean"][i], rm[i], rtol=1e-7, atol=1e-9)
        np.testing.assert_allclose(out["running_var"][i], rv[i], rtol=1e-7, atol=1e-9)


def test_train_loop_lowers_the_loss_on_a_fixed_batch():
    table, params, images, labels = _small_setup(np.float32, N=4)
    sched = dict(base_lr=20.0, warmup_steps=2, warmup_start_lr=5.0)
    out = net.train_loop([(images, labels)], params, [np.zeros_like(p) for p in params], table, sched, 8,
                         round_model=synth.round_bf16, widths=SMALL["widths"], blocks=SMALL["blocks"])
    assert out["losses"][-1] < 0.7 * out["losses"][0], out["losses"]
    one = net.train_step(images, labels, params, [synth.round_bf16(p) for p in params],
                         [np.zeros_like(p) for p in params], table, lr=5.0, widths=SMALL["widths"], blocks=SMALL["blocks"])
    again = net.train_loop([(images, labels)], params, [np.zeros_like(p) for p in params], table, sched, 1,
                           round_model=synth.round_bf16, widths=SMALL["widths"], blocks=SMALL["blocks"])
    for a, b in zip(one["w_new"], again["master"]):   # one step of the loop is train_step
        np.testing.assert_array_equal(a, b)


# ------------------------------------------------------------------ seeded initialization, evaluation
def test_philox4x32_10_known_answers():
    """Known-answer vectors of Philox4x32-10 (Random123, Salmon et al. SC'11)."""
    kat = [((0, 0, 0, 0), (0, 0), (0x6627e8d5, 0xe169c58d, 0xbc57ac4c, 0x9b00dbd8)),
           ((0xffffffff,) * 4, (0xffffffff,) * 2, (0x408f276d, 0x41c83b0e, 0xa20bc7c6, 0x6d5451fd)),
           ((0x243f6a88, 0x85a308d3, 0x13198a2e, 0x03707344), (0xa4093822, 0x299f31d0),
            (0xd16cfe09, 0x94fdcceb, 0x5001e420, 0x24126ea1))]
    for ctr, key, want in kat:
        got = net.philox4x32_10(np.array(ctr, np.uint32), key)
        assert tuple(int(v) for v in got) == want, [hex(int(v)) for v in got]
    # vectorized = one at a time
    ctrs = np.array([k[0] for k in kat], np.uint32)
    keys = (np.array([k[1][0] for k in kat], np.uint32), np.array([k[1][1] for k in kat], np.uint32))
    assert np.array_equal(net.philox4x32_10(ctrs, keys), np.array([k[2] for k in kat], np.uint32))


def test_truncated_normal_stream_properties():
    from scipy import stats
    z = net.truncated_normal(100000, 3, 200_000)
    assert np.abs(z).max() <= 2.0 and np.abs(z).max() > 1.99
    assert abs(z.mean()) < 0.01
    assert abs(z.std() - 0.8796256610342398) < 0.005          # std of N(0,1) cut at +-2
    assert stats.kstest(z, stats.truncnorm(-2, 2).cdf).pvalue > 1e-3
    # pure function of (seed, tensor, element): any slice can be produced on its own, in any order
    assert np.array_equal(net.truncated_normal(100000, 3, 1000, first=50_000), z[50_000:51_000])
    # other tensors and other seeds are other streams
    for other in (net.truncated_normal(100000, 4, 200_000), net.truncated_normal(100001, 3, 200_000)):
        assert abs(np.corrcoef(z, other)[0, 1]) < 0.01
    big = net.truncated_normal(7, 0, 4, first=(1 << 32) - 2)   # the element index crosses 32 bits
    assert len(set(big.tolist())) == 4


def test_init_params_he_scaling_and_vector_tensors():
    table = net.param_table()
    params = net.init_params(table[:12], 100000)
    for (name, shape, kind), p in zip(table[:12], params):
        assert p.shape == tuple(shape) and p.dtype == np.float32
        if kind == "conv":
            fan_in = int(np.prod(shape[1:]))
            assert np.abs(p).max() <= 2.0 * np.sqrt(2.0 / fan_in) * (1 + 1e-6)
            if p.size >= 4096:
                assert abs(p.std() / (0.87962566 * np.sqrt(2.0 / fan_in)) - 1) < 0.05, name
        elif kind == "gamma":
            assert np.all(p == 1)
        else:
            assert np.all(p == 0)
    again = net.init_params(table[:12], 100000)
    assert all(np.array_equal(a, b) for a, b in zip(params, again))
    assert not np.array_equal(params[0], net.init_params(table[:1], 100001)[0])


def _torch_eval(images, params, rm, rv, blocks):
    import torch
    import torch.nn.functional as F
    it = iter([torch.tensor(p, dtype=torch.float64) for p in params])
    st = iter(range(len(rm)))

    def cbn(x, stride, pad, relu=True, res=None, wgb=None, i=None):
        w, g, b = wgb if wgb is not None else (next(it), next(it), next(it))
        i = next(st) if i is None else i
        y = F.conv2d(x, w.permute(0, 3, 1, 2), None, stride, pad)
        y = F.batch_norm(y, torch.tensor(rm[i], dtype=torch.float64), torch.tensor(rv[i], dtype=torch.float64), g, b, False, 0.1, 1e-5)
        if res is not None:
            y = y + res
        return F.relu(y) if relu else y

    x = torch.tensor(images, dtype=torch.float64).permute(0, 3, 1, 2)
    cur = F.max_pool2d(cbn(x, 2, 3), 3, 2, 1)
    for i, nb in enumerate(blocks):
        for j in range(nb):
            stride = 2 if (j == 0 and i > 0) else 1
            z1 = cbn(cur, 1, 0)
            z2 = cbn(z1, stride, 1)
            wgb3 = (next(it), next(it), next(it)); i3 = next(st)
            sc = cbn(cur, stride, 0, relu=False) if j == 0 else cur
            cur = cbn(z2, 1, 0, res=sc, wgb=wgb3, i=i3)
    fw, fb = next(it), next(it)
    return (cur.mean(dim=(2, 3)) @ fw.T + fb).numpy()


def test_eval_forward_matches_torch_eval_mode():
    table, params, images, labels = _small_setup(np.float64, N=5)
    rng = np.random.default_rng(3)
    n_bn = sum(k == "gamma" for _, _, k in table)
    chans = [s[0] for _, s, k in table if k == "gamma"]
    rm = [0.3 * rng.standard_normal(c) for c in chans]
    rv = [0.5 + rng.random(c) for c in chans]
    out = net.eval_forward(images, labels, params, rm, rv, SMALL["widths"], SMALL["blocks"])
    want = _torch_eval(images, params, rm, rv, SMALL["blocks"])
    np.testing.assert_allclose(out["logits"], want, rtol=1e-9, atol=1e-11)
    assert np.array_equal(out["pred"], want.argmax(1)) and out["correct"] == int((want.argmax(1) == labels).sum())
    assert n_bn == len(rm)
    # ties go to the first maximum
    pred, correct = orc.top1(np.array([[1.0, 3.0, 3.0], [2.0, 2.0, 1.0], [0.0, -1.0, 5.0]]), np.array([1, 1, 2]))
    assert pred.tolist() == [1, 0, 2] and correct == 2
