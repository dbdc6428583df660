"""Helpers for the GPU parity tests: upload seeded layers and call the C ABI through the
Python binding.  The oracle side stays on the CPU (numpy in, numpy out)."""
import numpy as np


def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "a GPU test was collected without a GPU"
    return torch


def dev(a):
    torch = torch_cuda()
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def requant_dev(P, layer, window=None):
    lo, hi = window if window is not None else (layer.act_min, layer.act_max)
    return P.Requant(dev(layer.bias), dev(layer.mult), dev(layer.shift), lo, hi)


def run_pw(P, L, plan=None, window=None, residual=True, x=None):
    """Run prom_pw_conv(_ex) on a PwLayerInputs; returns the int8 numpy output."""
    torch = torch_cuda()
    xd = dev(L.x if x is None else x)
    wp = dev(P.prom_pack_ternary(L.weight))
    rq = requant_dev(P, L, window)
    res = dev(L.residual) if (residual and L.residual is not None) else None
    if plan is None:
        y = P.prom_pw_conv(xd, wp, L.cout, rq, res)
    else:
        y = P.prom_pw_conv_ex(xd, wp, L.cout, rq, res, plan=plan)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def oracle_pw(oracle, L, window=None, residual=True, x=None):
    lo, hi = window if window is not None else (L.act_min, L.act_max)
    return oracle.pw_conv(L.x if x is None else x, L.weight, L.bias, L.mult, L.shift, lo, hi,
                          L.residual if residual else None)


def assert_same(got, want, what=""):
    if not np.array_equal(got, want):
        bad = np.argwhere(got != want)
        i = tuple(bad[0])
        raise AssertionError(f"{what}: {len(bad)} of {got.size} outputs differ; first at {i}: "
                             f"got {int(got[i])} want {int(want[i])}")
