"""GPU test of lrnnx_lti_diag_scan_static, the entry point that takes no workspace and allocates nothing.

It runs the same kernels as lrnnx_lti_diag_scan on a scratch array inside the library's device image, so its
output must equal that entry point's bit for bit (and match the complex128 oracle to the fp32 bar of 1e-4).  The array
is shared by all calls on a GPU and keeps the previous call's contents: the second call here uses a smaller input, so
that stale chain slots of the first would be visible if the library did not re-arm them.
"""
import ctypes

import numpy as np
import pytest

from paper_2602_08810_amd import workloads
from _util import rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api():
    import torch
    assert torch.cuda.is_available()
    from paper_2602_08810_amd import api as _api
    _api.lib()
    return _api


def _one(api, oracle, B, P, L, seed, with_x0):
    import torch
    q = workloads.make_lti(B=B, P=P, L=L, seed=seed, with_x0=with_x0)
    lam, v = torch.from_numpy(q["lam"]).cuda(), torch.from_numpy(q["v"]).cuda()
    x0 = torch.from_numpy(q["x0"]).cuda() if with_x0 else None
    ref_x, ref_last = api.lrnnx_lti_diag_scan(lam, v, x0=x0, return_last_state=True, path="single_pass")
    out = torch.full_like(v, float("nan"))
    last = torch.full((B, P), float("nan"), dtype=torch.complex64, device="cuda")
    got = api.lrnnx_lti_diag_scan_static(lam, v, out, x0=x0, x_last_out=last)
    torch.cuda.synchronize()
    assert got.data_ptr() == out.data_ptr()
    assert torch.equal(torch.view_as_real(out), torch.view_as_real(ref_x)), (B, P, L)
    assert torch.equal(torch.view_as_real(last), torch.view_as_real(ref_last)), (B, P, L)
    xr = oracle.lti_diag_scan(q["lam"], q["v"], x0=q["x0"])
    xo = out.cpu().numpy()
    assert rel_err(xo.real, xr.real) <= 1e-4 and rel_err(xo.imag, xr.imag) <= 1e-4, (B, P, L)


def test_two_calls_in_a_row_second_smaller(api, oracle):
    _one(api, oracle, 4, 256, 4096, 1, True)      # the LTI benchmark configuration: 32 chained groups per row
    _one(api, oracle, 2, 100, 1000, 2, False)     # smaller: fewer groups, ragged P and L, the scratch holds stale slots
    _one(api, oracle, 1, 64, 33, 3, True)         # a single group


def test_limit_is_enforced_and_nothing_runs(api):
    import torch
    cap = int(api.lib().lrnnx_static_scratch_bytes())
    assert cap == 4 << 20
    B, P, L = 8, 1024, 8192                       # needs more chain slots than the array holds
    assert api.lrnnx_workspace_bytes(api.WS_LTI, B, P, 0, L, 0) > cap
    lam = torch.zeros(P, dtype=torch.complex64, device="cuda")
    v = torch.zeros((1, 8, P), dtype=torch.complex64, device="cuda")   # small buffers: the call must not touch them
    a = api.LtiArgs()
    a.struct_size = ctypes.sizeof(api.LtiArgs)
    a.B, a.P, a.L = B, P, L
    a.lambda_, a.v, a.x = lam.data_ptr(), v.data_ptr(), v.data_ptr()
    assert api.lib().lrnnx_lti_diag_scan_static(ctypes.byref(a)) == 3   # LRNNX_ERR_WORKSPACE
    a.B, a.L, a.path = 1, 8, 2                                           # the two-launch path is not offered
    assert api.lib().lrnnx_lti_diag_scan_static(ctypes.byref(a)) == 1
    torch.cuda.synchronize()
