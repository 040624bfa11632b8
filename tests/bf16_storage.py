"""The forward pass of the network composed from the oracle's own operations, with the activations rounded to
bf16 wherever a bf16-storage implementation has to store them (every convolution output, every batch-norm output,
the pooled features).  Test-side code: the oracle's operations are called unchanged, only the tensors handed from
one to the next are rounded.  Two uses:
  * with and without the rounding, it measures how far bf16 storage alone moves the logits of a randomly
    initialised BN-ResNet on white-noise images (the reason the unrounded oracle is not an end-to-end reference at
    the bf16 bar);
  * with the rounding, it is the end-to-end reference for the GPU path's bf16 forward pass: both sides round at the
    same points.  What remains is float-vs-double accumulation, i.e. relative differences of ~1e-7 before a
    rounding -- and a network that re-rounds every layer amplifies those as well: a value that rounds the other way
    is off by a whole bf16 step, which makes more values downstream round the other way.  `jitter` measures that
    floor: every stored tensor is multiplied by 1 + jitter*N(0,1) before its rounding (1e-7 is the last bit of a
    float); the logits of ResNet-50 then move by about 5 %, half of what the rounding itself does.
"""
import numpy as np

import oracle as orc
import synth


def forward(images, model, vecs, blocks, rounded, eps=1e-5, keep=False, jitter=0.0, seed=1):
    """images NHWC (already bf16-representable), model[i]: the values the convolutions / FC read, vecs[i]: the float
    parameters (gamma, beta, FC bias are taken from these), both in parameter order.  Returns logits and, with keep,
    the block outputs."""
    rng = np.random.default_rng(seed)

    def R(a):
        if not rounded:
            return a
        if jitter:
            a = (a * (1.0 + jitter * rng.standard_normal(a.shape).astype(np.float32))).astype(np.float32)
        return synth.round_bf16(a)

    it = iter(range(len(model)))

    def cbn(x, stride, pad, mode, res=None):
        i, j, k = next(it), next(it), next(it)
        y = R(orc.conv_fwd(x, model[i], stride, pad))
        z, _, _ = orc.bn_relu_fwd(y, vecs[j], vecs[k], res, eps, mode)
        return R(z)

    cur = orc.maxpool_fwd(cbn(images, 2, 3, 1))
    outs = []
    for s, nb in enumerate(blocks):
        for b in range(nb):
            stride = 2 if (b == 0 and s > 0) else 1
            inp = cur
            z1 = cbn(inp, 1, 0, 1)
            z2 = cbn(z1, stride, 1, 1)
            i3 = (next(it), next(it), next(it))
            sc = cbn(inp, stride, 0, 0) if b == 0 else inp     # parameter order: conv3 before the projection
            y3 = R(orc.conv_fwd(z2, model[i3[0]], 1, 0))
            z3, _, _ = orc.bn_relu_fwd(y3, vecs[i3[1]], vecs[i3[2]], sc, eps, 2)
            cur = R(z3)
            if keep:
                outs.append(cur)
    a = R(orc.avgpool_fwd(cur))
    fw, fb = next(it), next(it)
    logits = orc.fc_fwd(a, model[fw], vecs[fb])
    return (logits, outs) if keep else logits


def loss_of(logits, labels, ls=0.0):
    return orc.xent_fwd_bwd(logits, labels, ls, 1.0)[0]
