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


def assert_close(got, want, tol, name=""):
    err = orc.rel_l2(host(got) if isinstance(got, torch.Tensor) else got, want)
    assert err <= tol, f"{name}: rel-L2 {err:.3e} > {tol:.1e}"
    return err
