"""ResNet-50 (v1.5 bottleneck) training step wired from the oracle's operations.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Wiring (appendix log of the paper: stem convolution with stride 2, 64 filters
and no bias, batch normalization, max-pool 112 -> 56, bottleneck blocks;
He et al. for the rest):
  stem:   conv 7x7/2 pad 3 -> BN -> ReLU -> max-pool 3x3/2 pad 1
  block:  conv 1x1 -> BN -> ReLU -> conv 3x3 (stride s, pad 1) -> BN -> ReLU
          -> conv 1x1 -> BN -> (+ shortcut) -> ReLU
          shortcut = input, or conv 1x1 (stride s) -> BN in the first block of a stage
  stages: 3, 4, 6, 3 blocks of width 64, 128, 256, 512 (outputs 4x wider); s = 2
          in the first block of stages 2-4, on the 3x3 convolution
  head:   global average pool -> FC -> softmax cross-entropy (label smoothing)
  update: LARS + momentum on every parameter tensor (Sec. III-A1), weight decay
          only on convolution / FC weights.

Parameter order (the order of every params / grads list here): stem W, stem
gamma, stem beta; per block conv1 W, g, b, conv2 W, g, b, conv3 W, g, b and, if
the block has a projection shortcut, proj W, g, b; then FC W, FC b.
"""
import numpy as np

from . import (avgpool_bwd, avgpool_fwd, bn_infer, bn_relu_bwd, bn_relu_fwd, bn_running_update, conv_dgrad, conv_fwd,
               conv_wgrad, fc_bwd, fc_fwd, lars_update, maxpool_bwd, maxpool_fwd, top1, xent_fwd_bwd)


def param_table(widths=(64, 128, 256, 512), blocks=(3, 4, 6, 3), stem=64, classes=1000, in_ch=3,
                expansion=4):
    """List of (name, shape, kind); kind in conv|gamma|beta|fcw|fcb."""
    t = []

    def conv(name, k, r, c):
        t.append((name + ".w", (k, r, r, c), "conv"))
        t.append((name + ".gamma", (k,), "gamma"))
        t.append((name + ".beta", (k,), "beta"))

    conv("stem", stem, 7, in_ch)
    cin = stem
    for i, (wd, nb) in enumerate(zip(widths, blocks)):
        for j in range(nb):
            p = f"s{i}b{j}"
            conv(p + ".c1", wd, 1, cin)
            conv(p + ".c2", wd, 3, wd)
            conv(p + ".c3", wd * expansion, 1, wd)
            if j == 0:
                conv(p + ".proj", wd * expansion, 1, cin)
            cin = wd * expansion
    t.append(("fc.w", (classes, cin), "fcw"))
    t.append(("fc.b", (classes,), "fcb"))
    return t


def _conv_bn_fwd(x, w, gamma, beta, stride, pad, mode, eps, residual=None):
    y = conv_fwd(x, w, stride, pad)
    z, mean, rstd = bn_relu_fwd(y, gamma, beta, residual, eps, mode)
    return z, dict(x=x, w=w, y=y, z=z, gamma=gamma, mean=mean, rstd=rstd, stride=stride, pad=pad,
                   mode=mode)


def _conv_bn_bwd(dz, tp, need_dx=True):
    """Returns dx (or None), dresidual (or None), (dw, dgamma, dbeta)."""
    dy, dres, dgamma, dbeta = bn_relu_bwd(dz, tp["y"], tp["z"], tp["gamma"], tp["mean"],
                                          tp["rstd"], tp["mode"])
    dw = conv_wgrad(tp["x"], dy, tp["w"].shape, tp["stride"], tp["pad"])
    dx = conv_dgrad(dy, tp["w"], tp["x"].shape, tp["stride"], tp["pad"]) if need_dx else None
    return dx, dres, (dw, dgamma, dbeta)


def bottleneck_fwd(x, p, stride, has_proj, eps=1e-5):
    """p: list of 9 (or 12 with projection) arrays in parameter order."""
    z1, t1 = _conv_bn_fwd(x, p[0], p[1], p[2], 1, 0, 1, eps)
    z2, t2 = _conv_bn_fwd(z1, p[3], p[4], p[5], stride, 1, 1, eps)
    if has_proj:
        sc, tp = _conv_bn_fwd(x, p[9], p[10], p[11], stride, 0, 0, eps)
    else:
        sc, tp = x, None
    z3, t3 = _conv_bn_fwd(z2, p[6], p[7], p[8], 1, 0, 2, eps, residual=sc)
    return z3, (t1, t2, t3, tp)


def bottleneck_bwd(dout, tape):
    t1, t2, t3, tp = tape
    d2, dsc, g3 = _conv_bn_bwd(dout, t3)
    d1, _, g2 = _conv_bn_bwd(d2, t2)
    dx, _, g1 = _conv_bn_bwd(d1, t1)
    grads = list(g1) + list(g2) + list(g3)
    if tp is not None:
        dxp, _, gp = _conv_bn_bwd(dsc, tp)
        dx = (dx.astype(np.float64) + dxp.astype(np.float64)).astype(dx.dtype)
        grads += list(gp)
    else:
        dx = (dx.astype(np.float64) + dsc.astype(np.float64)).astype(dx.dtype)
    return dx, grads


def forward_backward(images, labels, params, widths=(64, 128, 256, 512), blocks=(3, 4, 6, 3),
                     eps=1e-5, label_smoothing=0.0, grad_scale=1.0, keep=False):
    """images NHWC, labels int32[N], params in parameter order (the values the
    forward pass uses).  Returns dict(loss, logits, grads[, acts])."""
    it = iter(range(len(params)))

    def take(n):
        return [params[next(it)] for _ in range(n)]

    acts = {}
    sp = take(3)
    z0, t0 = _conv_bn_fwd(images, sp[0], sp[1], sp[2], 2, 3, 1, eps)
    cur = maxpool_fwd(z0, 3, 2, 1)
    if keep:
        acts["stem.y"] = t0["y"]; acts["stem.z"] = z0; acts["pool"] = cur
    tapes = []
    bn_inputs = [t0["y"]]  # what every BN layer normalizes, in parameter order (for the moving averages)
    for i, nb in enumerate(blocks):
        for j in range(nb):
            has_proj = j == 0
            stride = 2 if (j == 0 and i > 0) else 1
            bp = take(12 if has_proj else 9)
            cur, tp = bottleneck_fwd(cur, bp, stride, has_proj, eps)
            tapes.append(tp)
            bn_inputs += [t["y"] for t in tp if t is not None]
            if keep:
                acts[f"s{i}b{j}.out"] = cur
    fw, fb = take(2)
    N, H, W, C = cur.shape
    a = avgpool_fwd(cur)
    logits = fc_fwd(a, fw, fb)
    loss, row_loss, dlogits = xent_fwd_bwd(logits, labels, label_smoothing, grad_scale)

    da, dfw, dfb = fc_bwd(a, fw, dlogits)
    d = avgpool_bwd(da, H, W)
    block_grads = []
    for tp in reversed(tapes):
        d, g = bottleneck_bwd(d, tp)
        block_grads.append(g)
    d = maxpool_bwd(z0, d, 3, 2, 1)
    _, _, g0 = _conv_bn_bwd(d, t0, need_dx=False)
    grads = list(g0)
    for g in reversed(block_grads):
        grads += g
    grads += [dfw, dfb]
    out = dict(loss=loss, row_loss=row_loss, logits=logits, dlogits=dlogits, grads=grads, bn_inputs=bn_inputs)
    if keep:
        out["acts"] = acts
    return out


def lars_hyper(table, weight_decay):
    """Per-tensor weight decay: on convolution / FC weights only."""
    return [weight_decay if kind in ("conv", "fcw") else 0.0 for (_, _, kind) in table]


def train_step(images, labels, master, model, velocity, table, *, eta=0.001, momentum=0.9, lr=1.0,
               weight_decay=5e-5, lars_eps=0.0, widths=(64, 128, 256, 512), blocks=(3, 4, 6, 3),
               eps=1e-5, label_smoothing=0.0, grad_scale=1.0):
    """One training step.  `model` are the values the forward/backward use (the
    master weights themselves, or their half-precision rounding, Sec. IV);
    LARS updates `master` (single precision) with the resulting gradients."""
    fb = forward_backward(images, labels, model, widths, blocks, eps, label_smoothing, grad_scale)
    wds = lars_hyper(table, weight_decay)
    w_new, v_new, norms = lars_update(master, fb["grads"], velocity, eta, momentum, lr, wds, lars_eps)
    fb.update(w_new=w_new, v_new=v_new, norms=norms)
    return fb


def learning_rate(t, base_lr, warmup_steps=0, warmup_start_lr=0.0, decay="none", total_steps=0, end_lr=0.0,
                  power=2.0, step_every=1, step_factor=0.1, table=None):
    """Learning rate of step t = 0, 1, ... (Sec. III-A1: gradual warm-up, then one of the decay patterns
    the paper lists -- step, polynomial, linear -- or any user-supplied table).  In double.

    t < warmup_steps:  start + (base - start) * t / warmup_steps   (reaches base at t = warmup_steps)
    afterwards, with u = t - warmup_steps and D = total_steps - warmup_steps:
      none        base
      step        base * step_factor ** floor(u / step_every)
      polynomial  end + (base - end) * (1 - min(u, D)/D) ** power
      linear      the polynomial with power 1
      table       table[min(t, len(table) - 1)]  (the table covers warm-up too: warmup_steps is ignored)
    """
    t = int(t)
    if decay == "table":
        return float(table[min(t, len(table) - 1)])
    if t < warmup_steps:
        return float(warmup_start_lr + (base_lr - warmup_start_lr) * (t / warmup_steps))
    u = t - warmup_steps
    if decay == "none":
        return float(base_lr)
    if decay == "step":
        return float(base_lr * step_factor ** (u // step_every))
    if decay in ("polynomial", "linear"):
        D = total_steps - warmup_steps
        frac = 1.0 - min(u, D) / D
        return float(end_lr + (base_lr - end_lr) * frac ** (power if decay == "polynomial" else 1.0))
    raise ValueError(decay)


def train_loop(batches, master, velocity, table, schedule, steps, *, first_step=0, round_model=None,
               bn_momentum=0.9, running_mean=None, running_var=None, **step_kw):
    """`steps` training steps (the inner loop of the paper's training: Sec. III-A).  Step t uses batch
    batches[t % len(batches)] = (images, labels) and the learning rate learning_rate(first_step + t,
    **schedule); the forward/backward passes read round_model(master) (the half-precision copy of
    Sec. IV; None: the master weights themselves); the moving averages of every BN layer's batch mean
    and biased variance follow with `bn_momentum` (appendix log: 0.9; start: mean 0, variance 1).
    Returns dict(losses, lrs, master, velocity, running_mean, running_var, last)."""
    master = [np.array(w, copy=True) for w in master]
    velocity = [np.array(v, copy=True) for v in velocity]
    n_bn = sum(1 for (_, _, kind) in table if kind == "gamma")
    gam = [w for w, (_, _, kind) in zip(master, table) if kind == "gamma"]
    rm = [np.zeros_like(g) for g in gam] if running_mean is None else [np.array(a, copy=True) for a in running_mean]
    rv = [np.ones_like(g) for g in gam] if running_var is None else [np.array(a, copy=True) for a in running_var]
    losses, lrs, fb = [], [], None
    for t in range(steps):
        images, labels = batches[t % len(batches)]
        lr = learning_rate(first_step + t, **schedule)
        model = master if round_model is None else [round_model(w) for w in master]
        fb = train_step(images, labels, master, model, velocity, table, lr=lr, **step_kw)
        assert len(fb["bn_inputs"]) == n_bn
        for i, y in enumerate(fb["bn_inputs"]):
            rm[i], rv[i] = bn_running_update(y, rm[i], rv[i], bn_momentum)
        master, velocity = fb["w_new"], fb["v_new"]
        losses.append(float(fb["loss"]))
        lrs.append(lr)
    return dict(losses=losses, lrs=lrs, master=master, velocity=velocity, running_mean=rm, running_var=rv, last=fb)


# ------------------------------------------------------------------ seeded parallel initialization
# Sec. III-B1: every process holds the same seed and initializes all weights itself, in parallel, instead
# of receiving them by broadcast.  For that each value must be a pure function of (seed, tensor, element):
# a counter-based generator.  Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
# as 1, 2, 3", SC'11) is used, written out below from its definition.
_PHILOX_M = (0xD2511F53, 0xCD9E8D57)   # round multipliers
_PHILOX_W = (0x9E3779B9, 0xBB67AE85)   # key increments (golden ratio, sqrt(3) - 1)
TRUNC = 2.0                            # the initializer's normal is cut at +-2 standard deviations


def philox4x32_10(counter, key):
    """counter: uint32 array [..., 4]; key: two uint32 (scalars or arrays broadcastable to counter[..., 0]).
    Ten rounds; per round (c0,c1,c2,c3) <- (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1, lo(M0*c0)),
    then the key is bumped by (W0, W1)."""
    c = [np.asarray(counter[..., i], np.uint64) for i in range(4)]
    k0 = np.asarray(key[0], np.uint64); k1 = np.asarray(key[1], np.uint64)
    mask = np.uint64(0xFFFFFFFF)
    for _ in range(10):
        p0 = np.uint64(_PHILOX_M[0]) * c[0]
        p1 = np.uint64(_PHILOX_M[1]) * c[2]
        c = [(p1 >> np.uint64(32)) ^ c[1] ^ k0, p1 & mask, (p0 >> np.uint64(32)) ^ c[3] ^ k1, p0 & mask]
        k0 = (k0 + np.uint64(_PHILOX_W[0])) & mask
        k1 = (k1 + np.uint64(_PHILOX_W[1])) & mask
    return np.stack([v.astype(np.uint32) for v in c], axis=-1)


def truncated_normal(seed, tensor_index, n, first=0):
    """Elements first .. first+n-1 of tensor `tensor_index`'s stream: standard normal restricted to
    [-TRUNC, TRUNC], by inversion -- u = (x0 + 1/2)/2^32 from the first Philox output for counter
    (element low word, element high word, tensor index, 0) and key (seed low, seed high);
    z = Phi^-1(Phi(-TRUNC) + u*(Phi(TRUNC) - Phi(-TRUNC))).  Double precision."""
    from scipy.special import ndtr, ndtri
    i = np.arange(first, first + n, dtype=np.uint64)
    ctr = np.zeros((n, 4), np.uint32)
    ctr[:, 0] = (i & np.uint64(0xFFFFFFFF)).astype(np.uint32)
    ctr[:, 1] = (i >> np.uint64(32)).astype(np.uint32)
    ctr[:, 2] = tensor_index
    x0 = philox4x32_10(ctr, (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF))[:, 0]
    u = (x0.astype(np.float64) + 0.5) / 4294967296.0
    lo, hi = ndtr(-TRUNC), ndtr(TRUNC)
    return ndtri(lo + u * (hi - lo))


def init_params(table, seed=100000):
    """Initial parameters (appendix log: truncated-normal initializer, seed 100000): convolution and FC
    weights std*z with std = sqrt(2/fan_in) (He) and z the truncated normal above, element index = the
    flat index in the tensor's own layout; BN gamma 1, beta 0, FC bias 0.  float32."""
    out = []
    for t, (_, shape, kind) in enumerate(table):
        n = int(np.prod(shape))
        if kind in ("conv", "fcw"):
            fan_in = int(np.prod(shape[1:]))
            z = truncated_normal(seed, t, n)
            out.append((np.sqrt(2.0 / fan_in) * z).astype(np.float32).reshape(shape))
        elif kind == "gamma":
            out.append(np.ones(shape, np.float32))
        else:
            out.append(np.zeros(shape, np.float32))
    return out


# ------------------------------------------------------------------ evaluation
def eval_forward(images, labels, params, running_mean, running_var, widths=(64, 128, 256, 512), blocks=(3, 4, 6, 3),
                 eps=1e-5):
    """The network in evaluation mode (appendix log: eval_accuracy): BN uses its moving averages.
    running_mean / running_var: one array per BN layer, parameter order.  Returns dict(logits, pred, correct)."""
    it = iter(range(len(params)))
    bn = iter(range(len(running_mean)))

    def cbn(x, stride, pad, mode, residual=None):
        w, g, b = (params[next(it)] for _ in range(3))
        i = next(bn)
        return bn_infer(conv_fwd(x, w, stride, pad), g, b, running_mean[i], running_var[i], residual, eps, mode)

    cur = maxpool_fwd(cbn(images, 2, 3, 1), 3, 2, 1)
    for i, nb in enumerate(blocks):
        for j in range(nb):
            stride = 2 if (j == 0 and i > 0) else 1
            z1 = cbn(cur, 1, 0, 1)
            z2 = cbn(z1, stride, 1, 1)
            if j == 0:  # parameter order: conv3 before the projection
                w3, g3, b3 = (params[next(it)] for _ in range(3))
                i3 = next(bn)
                sc = cbn(cur, stride, 0, 0)
                cur = bn_infer(conv_fwd(z2, w3, 1, 0), g3, b3, running_mean[i3], running_var[i3], sc, eps, 2)
            else:
                cur = cbn(z2, 1, 0, 2, residual=cur)
    fw, fb = params[next(it)], params[next(it)]
    logits = fc_fwd(avgpool_fwd(cur), fw, fb)
    pred, correct = top1(logits, labels)
    return dict(logits=logits, pred=pred, correct=correct)
