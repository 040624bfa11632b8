"""Seeded synthetic inputs shared by the CPU oracle's tests and the GPU tests.

This module holds no arithmetic of the method: it only draws numbers.  Every
tensor is drawn from a counter-based generator (Philox) keyed by (seed, tag),
in the tensor's LOGICAL index order (N,C,H,W for activations, K,C,R,S for
convolution weights) and then permuted to the storage layout both sides use
(NHWC / KRSC), so the values do not depend on any layout choice.

Default seed 100000: the seed the paper's run logs (appendix,
run_set_random_seed).  Inputs stand in for ImageNet (Sec. I): 224x224x3
images, 1000 classes, values ~N(0,1) as after per-channel normalisation.
"""
import zlib

import numpy as np

DEFAULT_SEED = 100000


def _rng(seed, tag):
    return np.random.Generator(np.random.Philox(key=[int(seed), zlib.crc32(tag.encode())]))


def normal(seed, tag, shape, std=1.0, dtype=np.float32):
    """N(0, std^2) array of `shape`, drawn in C order of `shape`."""
    n = int(np.prod(shape)) if len(shape) else 1
    return (_rng(seed, tag).standard_normal(n) * std).reshape(shape).astype(dtype)


def activation_nhwc(seed, tag, N, C, H, W, std=1.0, dtype=np.float32):
    """Drawn as N,C,H,W; returned contiguous N,H,W,C."""
    a = normal(seed, tag, (N, C, H, W), std, dtype)
    return np.ascontiguousarray(a.transpose(0, 2, 3, 1))


def conv_weight_krsc(seed, tag, K, C, R, S, dtype=np.float32):
    """He-normal N(0, 2/(C*R*S)) drawn as K,C,R,S; returned contiguous K,R,S,C."""
    w = normal(seed, tag, (K, C, R, S), np.sqrt(2.0 / (C * R * S)), dtype)
    return np.ascontiguousarray(w.transpose(0, 2, 3, 1))


def labels(seed, tag, N, classes):
    return _rng(seed, tag).integers(0, classes, size=N, dtype=np.int64).astype(np.int32)


def round_bf16(a):
    """Round float32 values to the nearest bfloat16 (ties to even), returned as float32."""
    a = np.ascontiguousarray(a, np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    out = r.astype(np.uint32).view(np.float32).reshape(a.shape)
    return np.where(np.isfinite(a), out, a)


def bf16_bits(a):
    """The uint16 bit patterns of float32 values that are already bf16-representable."""
    a = np.ascontiguousarray(a, np.float32)
    u = a.view(np.uint32)
    assert np.all((u & 0xFFFF) == 0), "values are not bf16-representable"
    return (u >> 16).astype(np.uint16).reshape(a.shape)


def params_from_table(seed, table, dtype=np.float32):
    """Initial parameters for a list of (name, shape, kind):
    conv / FC weights He-normal, BN gamma = 1, BN beta = 0, FC bias = 0."""
    out = []
    for name, shape, kind in table:
        if kind == "conv":
            K, R, S, C = shape
            out.append(conv_weight_krsc(seed, name, K, C, R, S, dtype))
        elif kind == "fcw":
            out.append(normal(seed, name, shape, np.sqrt(2.0 / shape[1]), dtype))
        elif kind == "gamma":
            out.append(np.ones(shape, dtype))
        else:
            out.append(np.zeros(shape, dtype))
    return out


def grads_from_table(seed, table, std=1e-3, dtype=np.float32):
    """Synthetic gradients ~N(0, std^2) for every tensor of the table."""
    return [normal(seed, "grad:" + name, shape, std, dtype) for name, shape, _ in table]
