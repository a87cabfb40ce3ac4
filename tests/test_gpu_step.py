"""GPU parity: single-token step kernels against the oracle, and the paper's mode-equivalence check
(Sec. 3: parallel scan vs step-wise execution) between the scan kernel and the step kernel."""
import numpy as np
import pytest

from paper_2602_08810_amd import workloads
from _util import TOL, dev, host, rel_err, sel_inputs_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api():
    import torch
    assert torch.cuda.is_available()
    from paper_2602_08810_amd import api as _api
    _api.lib()
    return _api


@pytest.mark.parametrize("io", ["f32", "bf16"])
@pytest.mark.parametrize("N", [1, 2, 4, 8, 16, 32])
@pytest.mark.parametrize("disc", ["zoh_s6", "zoh", "bilinear", "dirac"])
def test_selective_step_matches_oracle_over_several_tokens(api, oracle, io, N, disc):
    B, D, L = 3, 300, 5
    p = workloads.make_selective(B=B, D=D, N=N, L=L, io=io, gate=True, with_x0=True, with_dy=False, seed=90 + N,
                                 bias=("uniform", -4.0, -2.0))
    t = sel_inputs_dev(p, io)
    x = t["x0"].clone()
    xr = p["x0"].astype(np.float64)
    for l in range(L):
        # time slices of the [B,D,L] tensors: stride_d = L
        y = api.lrnnx_selective_step(x, t["u"][:, :, l], t["delta"][:, :, l], t["A"], t["Bm"][:, l].contiguous(),
                                     t["Cm"][:, l].contiguous(), Dskip=t["Dskip"], delta_bias=t["delta_bias"],
                                     z=t["z"][:, :, l], disc=disc)
        yr, xr = oracle.selective_step(xr, p["u"][:, :, l], p["delta"][:, :, l], p["A"], p["Bm"][:, l], p["Cm"][:, l],
                                       Dskip=p["Dskip"], delta_bias=p["delta_bias"], z=p["z"][:, :, l], disc=disc)
        assert rel_err(host(y), yr) <= TOL[io], f"y at token {l}"
        assert rel_err(host(x), xr) <= 1e-4, f"state at token {l}"


def test_step_by_step_equals_the_scan_kernel(api, oracle):
    """L step launches reproduce one scan launch (state and outputs), the paper's mode-equivalence test."""
    B, D, N, L = 2, 70, 16, 600
    p = workloads.make_selective(B=B, D=D, N=N, L=L, io="f32", gate=True, with_x0=True, with_dy=False, seed=97)
    t = sel_inputs_dev(p, "f32")
    y_scan, x_last = api.lrnnx_selective_scan_fwd(**t, return_last_state=True)
    import torch
    x = t["x0"].clone()
    ys = torch.empty_like(y_scan)
    Bt, Ct = t["Bm"].transpose(0, 1).contiguous(), t["Cm"].transpose(0, 1).contiguous()     # [L,B,N]
    for l in range(L):
        api.lrnnx_selective_step(x, t["u"][:, :, l], t["delta"][:, :, l], t["A"], Bt[l], Ct[l], Dskip=t["Dskip"],
                                 delta_bias=t["delta_bias"], z=t["z"][:, :, l], out=ys[:, :, l])
    assert rel_err(host(ys), host(y_scan)) <= 1e-4
    assert rel_err(host(x), host(x_last)) <= 1e-4


def test_lti_step(api, oracle):
    import torch
    B, P, L = 3, 500, 6
    q = workloads.make_lti(B=B, P=P, L=L, seed=98, with_x0=True)
    lam = torch.from_numpy(q["lam"]).cuda()
    v = torch.from_numpy(q["v"]).cuda()
    x = torch.from_numpy(q["x0"]).cuda().clone()
    xr = q["x0"].astype(np.complex128)
    for k in range(L):
        api.lrnnx_lti_step(lam, x, v[:, k].contiguous())
        xr = oracle.lti_step(q["lam"], xr, q["v"][:, k])
        got = x.cpu().numpy()
        assert rel_err(got.real, xr.real) <= 1e-4 and rel_err(got.imag, xr.imag) <= 1e-4
    x_scan = api.lrnnx_lti_diag_scan(lam, v, x0=torch.from_numpy(q["x0"]).cuda())
    assert rel_err(np.abs(x.cpu().numpy() - x_scan[:, -1].cpu().numpy()), np.abs(xr)) <= 1e-4 or \
        np.max(np.abs(x.cpu().numpy() - x_scan[:, -1].cpu().numpy())) <= 1e-4 * np.max(np.abs(xr))


def test_error_codes(api):
    import torch
    x = torch.zeros((1, 4, 3), device="cuda")
    u = torch.zeros((1, 4), device="cuda")
    with pytest.raises(api.LrnnxError) as e:
        api.lrnnx_selective_step(x, u, u, torch.zeros((4, 3), device="cuda"), torch.zeros((1, 3), device="cuda"),
                                 torch.zeros((1, 3), device="cuda"))
    assert e.value.code == 2


@pytest.mark.parametrize("io", ["f32", "bf16"])
@pytest.mark.parametrize("N,D,G", [(16, 24, 3), (4, 10, 5), (2, 6, 6), (8, 64, 2)])
def test_selective_step_with_grouped_maps(api, oracle, io, N, D, G):
    """Bm, Cm [B,G,N] per token: against the oracle, and step by step against the grouped scan kernel."""
    import torch
    B, L = 3, 6
    p = workloads.make_selective(B=B, D=D, N=N, L=L, io=io, gate=True, with_x0=True, with_dy=False, seed=50 + G,
                                 bias=("uniform", -4.0, -2.0), bc_groups=G)
    t = sel_inputs_dev(p, io)
    y_scan, x_last = api.lrnnx_selective_scan_fwd(**t, return_last_state=True)
    x = t["x0"].clone()
    xr = p["x0"].astype(np.float64)
    for l in range(L):
        y = api.lrnnx_selective_step(x, t["u"][:, :, l], t["delta"][:, :, l], t["A"], t["Bm"][:, :, l].contiguous(),
                                     t["Cm"][:, :, l].contiguous(), Dskip=t["Dskip"], delta_bias=t["delta_bias"],
                                     z=t["z"][:, :, l])
        yr, xr = oracle.selective_step(xr, p["u"][:, :, l], p["delta"][:, :, l], p["A"], p["Bm"][:, :, l],
                                       p["Cm"][:, :, l], Dskip=p["Dskip"], delta_bias=p["delta_bias"], z=p["z"][:, :, l])
        assert rel_err(host(y), yr) <= TOL[io], f"y at token {l}"
        assert rel_err(host(x), xr) <= 1e-4, f"state at token {l}"
        assert rel_err(host(y), host(y_scan[:, :, l])) <= TOL[io]
    assert rel_err(host(x), host(x_last)) <= 1e-4


def _cmaps(a, io):
    """[..., 2] float32 (re, im), already rounded -> complex64 (float32 I/O) or bfloat16 pairs."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t.to(torch.bfloat16) if io == "bf16" else torch.view_as_complex(t)


@pytest.mark.parametrize("io", ["f32", "bf16"])
@pytest.mark.parametrize("N", [1, 2, 4, 8, 16])
@pytest.mark.parametrize("disc", ["zoh_s6", "zoh", "bilinear", "dirac"])
def test_complex_step_matches_oracle_over_several_tokens(api, oracle, io, N, disc):
    import torch
    B, D, L = 3, 300, 5
    p = workloads.make_selective_complex(B=B, D=D, N=N, L=L, io=io, gate=True, seed=190 + N, with_x0=True)
    cplx = lambda a: a[..., 0].astype(np.float64) + 1j * a[..., 1].astype(np.float64)
    u, dl, z = dev(p["u"], io), dev(p["delta"], io), dev(p["z"], io)
    A = torch.from_numpy(p["A"]).cuda()
    x = torch.from_numpy(p["x0"]).cuda().clone()
    xr = p["x0"].astype(np.complex128)
    for l in range(L):
        y = api.lrnnx_selective_step_complex(x, u[:, :, l], dl[:, :, l], A, _cmaps(p["Bm"][:, l], io), _cmaps(p["Cm"][:, l], io),
                                             Dskip=dev(p["Dskip"]), delta_bias=dev(p["delta_bias"]), z=z[:, :, l], disc=disc)
        yr, xr = oracle.selective_step_complex(xr, p["u"][:, :, l], p["delta"][:, :, l], p["A"], cplx(p["Bm"][:, l]),
                                               cplx(p["Cm"][:, l]), Dskip=p["Dskip"], delta_bias=p["delta_bias"],
                                               z=p["z"][:, :, l], disc=disc)
        assert rel_err(host(y), yr) <= TOL[io], f"y at token {l}"
        xg = x.cpu().numpy()
        assert float(np.abs(xg - xr).max() / np.abs(xr).max()) <= 1e-4, f"state at token {l}"


def test_complex_step_by_step_equals_the_complex_scan_kernel(api):
    """L complex step launches reproduce one launch of the complex scan (state and outputs)."""
    import torch
    B, D, N, L = 2, 40, 16, 300
    p = workloads.make_selective_complex(B=B, D=D, N=N, L=L, io="f32", gate=True, seed=197, with_x0=True)
    u, dl, z = dev(p["u"]), dev(p["delta"]), dev(p["z"])
    A, x0 = torch.from_numpy(p["A"]).cuda(), torch.from_numpy(p["x0"]).cuda()
    Bm, Cm = _cmaps(p["Bm"], "f32"), _cmaps(p["Cm"], "f32")
    kw = dict(Dskip=dev(p["Dskip"]), delta_bias=dev(p["delta_bias"]))
    y_scan, x_last = api.lrnnx_selective_scan_fwd_complex(u, dl, A, Bm, Cm, z=z, x0=x0, return_last_state=True, **kw)
    x = x0.clone()
    ys = torch.empty_like(y_scan)
    Bt, Ct = Bm.transpose(0, 1).contiguous(), Cm.transpose(0, 1).contiguous()     # [L,B,N]
    for l in range(L):
        api.lrnnx_selective_step_complex(x, u[:, :, l], dl[:, :, l], A, Bt[l], Ct[l], z=z[:, :, l], out=ys[:, :, l], **kw)
    assert rel_err(host(ys), host(y_scan)) <= 1e-4
    assert float((x - x_last).abs().max() / x_last.abs().max()) <= 1e-4
