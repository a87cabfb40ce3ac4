"""GPU parity: lrnnx_lti_diag_scan_bwd (through the C ABI) against the complex128 oracle.

The kernel takes the states its own forward call saved; the oracle recomputes them in fp64 from (lam, v, x0).
Tolerance: max-abs error over the tensor's max-abs value <= 1e-4 for fp32 storage (the bar of the forward scan) for
every output, dlam = sum conj(x_{k-1}) g_k included.  (dlam sums products of two fp32-scanned sequences and is the
output most sensitive to a systematic error in the powers lambda^len that carry states between wavefronts and
workgroups: those powers are formed in double precision and rounded once.)
"""
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


def _crel(got, ref):
    return max(rel_err(got.real, ref.real), rel_err(got.imag, ref.imag))


def _run(api, oracle, B, P, L, with_x0, seed, inplace=False):
    import torch
    q = workloads.make_lti(B=B, P=P, L=L, seed=seed, with_x0=with_x0, with_gx=True)
    lam, v, gx = (torch.from_numpy(q[k]).cuda() for k in ("lam", "v", "gx"))
    x0 = torch.from_numpy(q["x0"]).cuda() if with_x0 else None
    x = api.lrnnx_lti_diag_scan(lam, v, x0=x0)
    dv, dlam, dx0 = api.lrnnx_lti_diag_scan_bwd(lam, x, gx, x0=x0, out=gx if inplace else None)
    rdv, rdlam, rdx0 = oracle.lti_diag_scan_bwd(q["lam"], q["v"], q["gx"], x0=q["x0"])
    got = dv.cpu().numpy()
    assert _crel(got, rdv) <= 1e-4, "dv"
    assert _crel(dlam.cpu().numpy(), rdlam) <= 1e-4, "dlam"
    assert _crel(dx0.cpu().numpy(), rdx0) <= 1e-4, "dx0"
    return got, dlam.cpu().numpy()


def test_config1_backward(api, oracle):
    _run(api, oracle, 4, 256, 4096, False, 1)


@pytest.mark.parametrize("B,P,L", [(1, 1, 1), (2, 5, 17), (3, 300, 1000), (1, 64, 33), (2, 257, 4099), (1, 2048, 64),
                                   (1, 64, 8192), (1, 70, 5000), (2, 2053, 700), (16, 300, 1000), (2, 64, 128), (1, 64, 129)])
@pytest.mark.parametrize("with_x0", [False, True])
def test_shapes(api, oracle, B, P, L, with_x0):
    _run(api, oracle, B, P, L, with_x0, seed=B * 1000 + P + L)


def test_long_sequence_many_groups(api, oracle):
    """L = 65536: 512 time groups chained by look-back, 32 anchors."""
    _run(api, oracle, 1, 96, 65536, True, seed=9)


def test_in_place_and_dv_deterministic(api, oracle):
    got, _ = _run(api, oracle, 2, 128, 2048, True, 77, inplace=True)
    got2, _ = _run(api, oracle, 2, 128, 2048, True, 77, inplace=False)
    assert np.array_equal(got, got2)


def test_without_dx0_and_rejects_small_workspace(api):
    import torch
    q = workloads.make_lti(B=1, P=64, L=300, seed=3, with_gx=True)
    lam, v, gx = (torch.from_numpy(q[k]).cuda() for k in ("lam", "v", "gx"))
    x = api.lrnnx_lti_diag_scan(lam, v)
    dv, dlam, dx0 = api.lrnnx_lti_diag_scan_bwd(lam, x, gx, want_dx0=False)
    assert dx0 is None and bool(dv.isfinite().all()) and bool(dlam.isfinite().all())
    with pytest.raises(api.LrnnxError):
        api.lrnnx_lti_diag_scan_bwd(lam, x, gx, workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))
