"""GPU parity: lrnnx_diag_scan (caller-supplied a_k, b_k; through the C ABI) against the fp64 oracle.

Tolerance: max-abs error over the tensor's max-abs value <= 1e-4 (fp32 storage and arithmetic, the bar of the LTI scan).
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


def _err(got, ref):
    if np.iscomplexobj(ref):
        return max(rel_err(got.real, ref.real), rel_err(got.imag, ref.imag))
    return rel_err(got, ref)


def _run(api, oracle, B, P, L, cplx, with_x0, seed, inplace=False):
    import torch
    q = workloads.make_diag(B=B, P=P, L=L, cplx=cplx, seed=seed, with_x0=with_x0)
    a, b = torch.from_numpy(q["a"]).cuda(), torch.from_numpy(q["b"]).cuda()
    x0 = torch.from_numpy(q["x0"]).cuda() if with_x0 else None
    x, x_last = api.lrnnx_diag_scan(a, b, x0=x0, return_last_state=True, out=b if inplace else None)
    ref = oracle.diag_scan(q["a"], q["b"], x0=q["x0"])
    got = x.cpu().numpy()
    assert _err(got, ref) <= 1e-4
    assert np.max(np.abs(x_last.cpu().numpy() - ref[:, -1, :])) <= 1e-4 * np.max(np.abs(ref))
    return got


@pytest.mark.parametrize("B,P,L", [(1, 1, 1), (2, 5, 17), (3, 300, 1000), (1, 64, 33), (2, 257, 4099), (1, 2048, 64),
                                   (1, 64, 8192), (1, 70, 5000), (2, 2053, 700), (16, 300, 1000), (4, 256, 4096)])
@pytest.mark.parametrize("cplx", [False, True])
@pytest.mark.parametrize("with_x0", [False, True])
def test_shapes(api, oracle, B, P, L, cplx, with_x0):
    _run(api, oracle, B, P, L, cplx, with_x0, seed=B * 1000 + P + L)


@pytest.mark.parametrize("cplx", [False, True])
def test_long_sequence_many_groups(api, oracle, cplx):
    _run(api, oracle, 1, 96, 65536, cplx, True, seed=9)


@pytest.mark.parametrize("cplx", [False, True])
def test_in_place_and_deterministic(api, oracle, cplx):
    got = _run(api, oracle, 2, 128, 2048, cplx, True, 77, inplace=True)
    got2 = _run(api, oracle, 2, 128, 2048, cplx, True, 77, inplace=False)
    assert np.array_equal(got, got2)


def test_constant_coefficient_agrees_with_the_lti_scan(api):
    """With a_k = lambda for every k the two entry points compute the same recurrence (different arithmetic order)."""
    import torch
    q = workloads.make_lti(B=2, P=130, L=3000, seed=5, with_x0=True)
    lam, v, x0 = (torch.from_numpy(q[k]).cuda() for k in ("lam", "v", "x0"))
    x1 = api.lrnnx_lti_diag_scan(lam, v, x0=x0)
    x2 = api.lrnnx_diag_scan(lam.expand_as(v).contiguous(), v, x0=x0)
    assert float((x1 - x2).abs().max()) <= 1e-4 * float(x1.abs().max())


def test_gates_reset_and_hold(api):
    """a_k = 0 forgets everything before k (exactly); a_k = 1 with b_k = 0 carries the state across a chunk border
    (to rounding: the state entering a chunk is rebuilt from aggregates, not stepped)."""
    import torch
    g = torch.Generator(device="cuda").manual_seed(3)
    a = torch.rand(1, 1000, 64, device="cuda", generator=g) * 0.5 + 0.5
    b = torch.randn(1, 1000, 64, device="cuda", generator=g)
    a[:, 300], a[:, 511:515], b[:, 511:515] = 0.0, 1.0, 0.0
    x = api.lrnnx_diag_scan(a, b)
    assert torch.equal(x[:, 300], b[:, 300])
    assert float((x[:, 514] - x[:, 510]).abs().max()) <= 1e-6 * float(x.abs().max())
    x_tail = api.lrnnx_diag_scan(a[:, 300:].contiguous(), b[:, 300:].contiguous())
    assert float((x_tail - x[:, 300:]).abs().max()) <= 1e-5 * float(x.abs().max())


def test_rejects_bad_arguments(api):
    import torch
    a = torch.rand(1, 8, 4, device="cuda")
    with pytest.raises(TypeError):
        api.lrnnx_diag_scan(a, a.to(torch.complex64))
    with pytest.raises(api.LrnnxError):
        api.lrnnx_diag_scan(a, a.clone(), workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))
