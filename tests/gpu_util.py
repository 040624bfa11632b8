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
