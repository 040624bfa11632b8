"""The allocation-free LARS entry point (lars_update_noalloc, partial norms in the library's own device
array) against lars_update with a caller workspace: same kernels, so every output must be bit-equal, on
two calls in a row, the second with a smaller table (the shared array still holds the first call's sums)."""
import ctypes

import numpy as np
import pytest
import torch

import synth
from oracle import net

pytestmark = pytest.mark.gpu
SEED = synth.DEFAULT_SEED


@pytest.fixture(scope="module")
def rn():
    import paper_1903_12650_amd as rn
    return rn


def _arenas(table, seed_tag, grad_bf16):
    params = synth.params_from_table(SEED, table)
    grads = synth.grads_from_table(SEED, table, 1e-3)
    vel = [synth.normal(SEED, seed_tag + n, p.shape, 1e-3) for p, (n, _, _) in zip(params, table)]
    offs, tot = [], 0
    for p in params:
        offs.append(tot)
        tot += (p.size + 63) // 64 * 64

    def arena(arrs, bf=False):
        a = np.zeros(tot, np.float32)
        for o, p in zip(offs, arrs):
            a[o:o + p.size] = p.ravel()
        t = torch.from_numpy(a).cuda()
        return t.to(torch.bfloat16) if bf else t
    return params, offs, tot, arena(params), arena(grads, grad_bf16), arena(vel)


def _run_both(rn, table, grad_bf16, tag):
    params, offs, tot, W, G, V = _arenas(table, tag, grad_bf16)
    wds = net.lars_hyper(table, 5e-5)
    out = []
    for noalloc in (False, True):
        w, v = W.clone(), V.clone()
        low = torch.zeros(tot, dtype=torch.bfloat16, device="cuda")
        sl = lambda A: [A[o:o + p.size] for o, p in zip(offs, params)]
        tab = rn.LarsTable(sl(w), sl(G), sl(v), wds, None, sl(low))
        norms = torch.zeros(len(table) * 2, dtype=torch.float32, device="cuda")
        if noalloc:
            rn.lars_update_noalloc(tab, 0.001, 0.9, 1.0, 0.0, norms_out=norms)
        else:
            rn.lars_update(tab, 0.001, 0.9, 1.0, 0.0, norms_out=norms)
        torch.cuda.synchronize()
        out.append((w, v, low, norms))
    for a, b, what in zip(out[0], out[1], ("w", "v", "bf16 copy", "norms")):
        assert torch.equal(a, b), f"{tag}: {what} differs between lars_update and lars_update_noalloc"
    # and the update really happened (the weights moved)
    assert not torch.equal(out[1][0], W)


def test_noalloc_equals_workspace_form_twice_second_smaller(rn):
    full = net.param_table()                                   # 161 tensors, 25.56 M parameters, 3,200 chunks
    _run_both(rn, full, False, "first")
    small = [("a.w", (5, 3, 3, 7), "conv"), ("a.gamma", (5,), "gamma"), ("a.beta", (5,), "beta"),
             ("c.w", (17, 8193), "fcw"), ("c.b", (17,), "fcb")]
    _run_both(rn, small, False, "second")
    _run_both(rn, small, True, "third")                        # bf16 gradients


def test_noalloc_rejects_tables_beyond_the_scratch(rn):
    cap = int(rn.raw.lars_update_noalloc_max_chunks())
    assert cap == 32768
    n = (cap + 1) * 8192                                       # one tensor of cap+1 chunks: never touched
    one = torch.zeros(64, device="cuda")
    host = (rn.binding.LarsTensor * 1)()
    host[0] = rn.binding.LarsTensor(one.data_ptr(), one.data_ptr(), one.data_ptr(), 0, n, 0.0, 1)
    d = rn.binding.LarsDesc(1, 0.001, 0.9, 1.0, 0.0, rn.F32)
    rc = rn.raw.lars_update_noalloc(ctypes.byref(d), host, ctypes.c_void_p(one.data_ptr()), None, None)
    assert rc == -3 and b"built-in scratch" in rn.raw.rn50_last_error()
