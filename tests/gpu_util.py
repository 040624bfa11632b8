"""Helpers of the GPU parity tests: host <-> device marshalling and the rel-L2 bar."""
import numpy as np
import torch

import oracle as orc
import synth

TOL = {"f32": 1e-4, "bf16": 2e-2, "lars": 1e-6}     # relative-L2 tolerances per tensor


def dev(a, bf16=False):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t.to(torch.bfloat16) if bf16 else t


def host(t):
    return t.detach().float().cpu().numpy() if t.dtype == torch.bfloat16 else t.detach().cpu().numpy()


def inputs(mode, *arrays):
    """In bf16 mode round the host arrays to bf16 once: both sides then get identical values."""
    if mode == "bf16":
        arrays = [synth.round_bf16(a) for a in arrays]
    return arrays


ELEMENT_REL = 2.0 ** -7     # per element: twice the largest relative error of one rounding to bf16


def elementwise_excess(got, want, rel=ELEMENT_REL):
    """max over elements of |got - want| - rel*|want|, in units of rel*rms(want): <= 1 means every element is within
    rel*|want| + rel*rms(want).  The per-tensor rel-L2 alone would let a few wrong rows of a large tensor pass (one
    wrong row of 125,440 moves it by 3e-3); this bound holds every element to what one bf16 rounding of the exact
    result (plus float accumulation noise relative to the tensor's scale) can produce."""
    g = np.asarray(got, dtype=np.float64).ravel()
    w = np.asarray(want, dtype=np.float64).ravel()
    rms = float(np.sqrt(np.mean(w * w))) if w.size else 0.0
    if w.size == 0:
        return 0.0
    worst = float(np.max(np.abs(g - w) - rel * np.abs(w)))
    if rms == 0.0:
        return 0.0 if worst <= 0.0 else np.inf
    return worst / (rel * rms)


def assert_close(got, want, tol, name="", elementwise=None):
    """rel-L2 <= tol; at the bf16 bar (tol == TOL["bf16"], or elementwise=True) every element is held as well."""
    g = host(got) if isinstance(got, torch.Tensor) else got
    err = orc.rel_l2(g, want)
    assert err <= tol, f"{name}: rel-L2 {err:.3e} > {tol:.1e}"
    if elementwise or (elementwise is None and tol == TOL["bf16"]):
        ex = elementwise_excess(g, want)
        assert ex <= 1.0, f"{name}: an element is off by more than 2^-7*|want| + {ex:.2f} * 2^-7*rms(want)"
    return err


def impose_relu_decisions(z_oracle, relu_bits, max_differing=8):
    """The oracle's BN+ReLU output with the ReLU decisions of the GPU pass imposed on it.

    relu_bits: the GPU forward pass's recorded decisions (one byte per 16-byte vector of its output, bit j = stored
    output j is positive).  A pre-activation within float rounding of zero may land on either side of the ReLU, and one
    differing decision moves a gradient by more than the float bar; both outcomes are valid.  So the decisions are
    checked to differ from the oracle's only where the oracle's value is within rounding of zero (and only in a
    handful of places), then the oracle's backward pass runs with the decisions of the pass under test: zero where
    the GPU decided "off", the oracle's value (or the smallest positive number) where it decided "on"."""
    z = np.asarray(z_oracle)
    bits = host(relu_bits) if isinstance(relu_bits, torch.Tensor) else np.asarray(relu_bits)
    V = z.size // bits.size
    on = ((bits.reshape(-1, 1) >> np.arange(V, dtype=np.uint8)) & 1).astype(bool).reshape(z.shape)
    differ = on != (z > 0)
    n = int(differ.sum())
    if n:
        rms = float(np.sqrt(np.mean(np.square(z, dtype=np.float64)))) or 1.0
        assert n <= max_differing and float(np.abs(z[differ]).max()) <= 1e-5 * rms, (n, float(np.abs(z[differ]).max()), rms)
    return np.where(on, np.maximum(z, np.finfo(np.float32).tiny), 0).astype(z.dtype), n
