"""GPU parity: lrnnx_diag_scan_bwd (through the C ABI) against the fp64 oracle.  The kernel takes the states its own
forward call saved; the oracle recomputes them in fp64.  Tolerance 1e-4 of each tensor's max-abs value."""
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


def _err(got, ref):
    if np.iscomplexobj(ref):
        return max(rel_err(got.real, ref.real), rel_err(got.imag, ref.imag))
    return rel_err(got, ref)


def _run(api, oracle, B, P, L, cplx, with_x0, seed):
    import torch
    q = workloads.make_diag(B=B, P=P, L=L, cplx=cplx, seed=seed, with_x0=with_x0, with_gx=True)
    a, b, gx = (torch.from_numpy(q[k]).cuda() for k in ("a", "b", "gx"))
    x0 = torch.from_numpy(q["x0"]).cuda() if with_x0 else None
    x = api.lrnnx_diag_scan(a, b, x0=x0)
    da, db, dx0 = api.lrnnx_diag_scan_bwd(a, x, gx, x0=x0)
    rda, rdb, rdx0 = oracle.diag_scan_bwd(q["a"], q["b"], q["gx"], x0=q["x0"])
    assert _err(db.cpu().numpy(), rdb) <= 1e-4, "db"
    assert _err(da.cpu().numpy(), rda) <= 1e-4, "da"
    assert _err(dx0.cpu().numpy(), rdx0) <= 1e-4, "dx0"
    return da, db


@pytest.mark.parametrize("B,P,L", [(1, 1, 1), (2, 5, 17), (3, 300, 1000), (1, 64, 33), (2, 257, 4099), (1, 2048, 64),
                                   (1, 64, 8192), (1, 70, 5000), (2, 64, 128), (1, 64, 129), (16, 300, 1000),
                                   (4, 256, 4096)])
@pytest.mark.parametrize("cplx", [False, True])
@pytest.mark.parametrize("with_x0", [False, True])
def test_shapes(api, oracle, B, P, L, cplx, with_x0):
    _run(api, oracle, B, P, L, cplx, with_x0, seed=B * 1000 + P + L)


@pytest.mark.parametrize("cplx", [False, True])
def test_long_sequence_and_determinism(api, oracle, cplx):
    import torch
    da1, db1 = _run(api, oracle, 1, 96, 65536, cplx, True, seed=9)
    da2, db2 = _run(api, oracle, 1, 96, 65536, cplx, True, seed=9)
    assert torch.equal(da1, da2) and torch.equal(db1, db2)


def test_constant_coefficient_agrees_with_the_lti_backward(api):
    import torch
    q = workloads.make_lti(B=2, P=130, L=3000, seed=5, with_x0=True, with_gx=True)
    lam, v, x0, gx = (torch.from_numpy(q[k]).cuda() for k in ("lam", "v", "x0", "gx"))
    x = api.lrnnx_lti_diag_scan(lam, v, x0=x0)
    dv, dlam, dx0 = api.lrnnx_lti_diag_scan_bwd(lam, x, gx, x0=x0)
    da, db, dx0b = api.lrnnx_diag_scan_bwd(lam.expand_as(v).contiguous(), x, gx, x0=x0)
    assert float((db - dv).abs().max()) <= 1e-4 * float(dv.abs().max())
    assert float((dx0b - dx0).abs().max()) <= 1e-4 * float(dx0.abs().max())
    assert float((da.sum(dim=(0, 1)) - dlam).abs().max()) <= 1e-3 * float(dlam.abs().max())


def test_without_dx0_and_bad_arguments(api):
    import torch
    a = torch.rand(1, 40, 8, device="cuda")
    x = api.lrnnx_diag_scan(a, torch.randn_like(a))
    da, db, dx0 = api.lrnnx_diag_scan_bwd(a, x, torch.randn_like(a), want_dx0=False)
    assert dx0 is None and bool(da.isfinite().all()) and bool(db.isfinite().all())
    with pytest.raises(api.LrnnxError):
        api.lrnnx_diag_scan_bwd(a, x, torch.randn_like(a), workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))
