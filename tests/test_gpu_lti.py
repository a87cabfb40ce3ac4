"""GPU parity: lrnnx_lti_diag_scan (through the C ABI) against the complex128 oracle."""
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


def _run(api, oracle, B, P, L, with_x0, seed, inplace=False, path="auto"):
    import torch
    q = workloads.make_lti(B=B, P=P, L=L, seed=seed, with_x0=with_x0)
    lam, v = torch.from_numpy(q["lam"]).cuda(), torch.from_numpy(q["v"]).cuda()
    x0 = torch.from_numpy(q["x0"]).cuda() if with_x0 else None
    x, x_last = api.lrnnx_lti_diag_scan(lam, v, x0=x0, return_last_state=True, out=v if inplace else None, path=path)
    ref = oracle.lti_diag_scan(q["lam"], q["v"], x0=q["x0"])
    got = x.cpu().numpy()
    assert rel_err(got.real, ref.real) <= 1e-4 and rel_err(got.imag, ref.imag) <= 1e-4
    assert np.max(np.abs(x_last.cpu().numpy() - ref[:, -1, :])) <= 1e-4 * np.max(np.abs(ref))
    return got, ref


@pytest.mark.parametrize("path", ["single_pass", "chunk_carry"])
def test_config1(api, oracle, path):
    """Benchmark configuration 1: B=4, P=256, L=4096, complex64; one-launch look-back path and two-launch path."""
    _run(api, oracle, 4, 256, 4096, False, 1, path=path)


@pytest.mark.parametrize("B,P,L", [(1, 1, 1), (2, 5, 17), (3, 300, 1000), (1, 64, 33), (2, 257, 4099), (1, 2048, 64),
                                   (1, 64, 8192), (1, 70, 5000), (2, 2053, 700), (16, 300, 1000)])
@pytest.mark.parametrize("with_x0", [False, True])
@pytest.mark.parametrize("path", ["single_pass", "chunk_carry"])
def test_shapes(api, oracle, B, P, L, with_x0, path):
    _run(api, oracle, B, P, L, with_x0, seed=B * 1000 + P + L, path=path)


def test_long_sequence_many_groups(api, oracle):
    """L = 65536: 256 time groups chained by look-back in the single-pass kernel."""
    _run(api, oracle, 1, 96, 65536, True, seed=9, path="single_pass")
    _run(api, oracle, 1, 96, 65536, True, seed=9, path="chunk_carry")


def test_in_place_and_deterministic(api, oracle):
    import torch
    got, _ = _run(api, oracle, 2, 128, 2048, True, 77, inplace=True)
    got2, _ = _run(api, oracle, 2, 128, 2048, True, 77, inplace=False)
    assert np.array_equal(got, got2)


def test_impulse_gives_powers_of_lambda(api):
    import torch
    P, L = 96, 512
    q = workloads.make_lti(B=1, P=P, L=L, seed=5)
    v = torch.zeros((1, L, P), dtype=torch.complex64, device="cuda")
    v[0, 0] = 1.0
    x = api.lrnnx_lti_diag_scan(torch.from_numpy(q["lam"]).cuda(), v).cpu().numpy()
    ref = q["lam"].astype(np.complex128)[None, :] ** np.arange(L)[:, None]
    assert np.max(np.abs(x[0] - ref)) <= 1e-4


def test_error_codes(api):
    import torch
    lam = torch.ones(4, dtype=torch.complex64, device="cuda")
    v = torch.zeros((1, 4096, 4), dtype=torch.complex64, device="cuda")
    with pytest.raises(api.LrnnxError) as e:
        api.lrnnx_lti_diag_scan(lam, v, workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert e.value.code == 3


def test_chain_status_word_stays_clear(api, oracle):
    """The optional status word reports a bounded wait between workgroups that ran out; on a healthy run of many
    chained groups (here 512 per row, and the adjoint and the caller-coefficient scans over the same shape) the library
    must leave it at the caller's zero."""
    import torch
    q = workloads.make_lti(B=2, P=70, L=65536 // 2, seed=11, with_gx=True)
    lam, v, gx = (torch.from_numpy(q[k]).cuda() for k in ("lam", "v", "gx"))
    st = torch.zeros(1, dtype=torch.int32, device="cuda")
    x = api.lrnnx_lti_diag_scan(lam, v, path="single_pass", chain_status=st)
    api.lrnnx_lti_diag_scan_bwd(lam, x, gx, chain_status=st)
    a = torch.from_numpy(np.abs(q["v"]).astype(np.float32) * 0.5).cuda().contiguous()
    xs = api.lrnnx_diag_scan(a, gx.real.contiguous(), chain_status=st)
    api.lrnnx_diag_scan_bwd(a, xs, gx.imag.contiguous(), chain_status=st)
    torch.cuda.synchronize()
    assert int(st.item()) == 0
    ref = oracle.lti_diag_scan(q["lam"], q["v"])
    got = x.cpu().numpy()
    assert rel_err(got.real, ref.real) <= 1e-4 and rel_err(got.imag, ref.imag) <= 1e-4
    with pytest.raises(ValueError):
        api.lrnnx_lti_diag_scan(lam, v, chain_status=torch.zeros(2, dtype=torch.int32, device="cuda"))
