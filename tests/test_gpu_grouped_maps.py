"""GPU parity of the selective scan with grouped maps Bm, Cm [B,G,L,N] (channel d reads group d // (D/G)),
forward and backward through the C ABI, against the fp64 oracle; same tolerances as the ungrouped tests."""
import numpy as np
import pytest

from paper_2602_08810_amd import workloads
from _util import TOL, dev, host, rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api():
    import torch
    assert torch.cuda.is_available()
    from paper_2602_08810_amd import api as _api
    _api.lib()
    return _api


def _check(api, oracle, B, D, N, L, G, io, seed, disc="zoh_s6", with_ckpt=True):
    p = workloads.make_selective(B=B, D=D, N=N, L=L, io=io, gate=True, seed=seed, with_x0=True, bc_groups=G,
                                 bias=("uniform", -4.0, -2.0))
    t = dict(u=dev(p["u"], io), delta=dev(p["delta"], io), A=dev(p["A"]), Bm=dev(p["Bm"], io), Cm=dev(p["Cm"], io),
             Dskip=dev(p["Dskip"]), delta_bias=dev(p["delta_bias"]), z=dev(p["z"], io), x0=dev(p["x0"]))
    y, x_last, ckpt = api.lrnnx_selective_scan_fwd(**t, disc=disc, return_last_state=True, return_ckpt=True)
    g = api.lrnnx_selective_scan_bwd(**t, dy=dev(p["dy"], io), disc=disc, ckpt=ckpt if with_ckpt else None,
                                     want_dx0=True)
    ref = {k: p[k] for k in ("u", "delta", "A", "Bm", "Cm", "Dskip", "delta_bias", "z", "x0")}
    yr, xr = oracle.selective_scan_fwd(**ref, disc=disc)
    r = oracle.selective_scan_bwd(dy=p["dy"], **ref, disc=disc)
    assert rel_err(host(y), yr) <= TOL[io]
    assert rel_err(host(x_last), xr) <= 1e-4
    assert tuple(g["dBm"].shape) == p["Bm"].shape
    tol = {"du": TOL[io], "ddelta": TOL[io], "dz": TOL[io], "dA": 1e-4, "dBm": 1e-4, "dCm": 1e-4, "dD": 1e-4,
           "dbias": 1e-4, "dx0": 1e-4}
    errs = {k: rel_err(host(g[k]), r[k]) for k in tol}
    bad = {k: v for k, v in errs.items() if not v <= tol[k]}
    assert not bad, f"{bad} (all {errs})"


@pytest.mark.parametrize("B,D,N,L,G", [(2, 16, 16, 300, 2), (1, 24, 16, 1000, 3), (2, 20, 8, 257, 4), (1, 6, 16, 700, 6),
                                       (3, 26, 4, 130, 2), (1, 256, 16, 600, 2), (2, 9, 2, 64, 9)])
@pytest.mark.parametrize("io", ["f32", "bf16"])
def test_grouped_shapes(api, oracle, B, D, N, L, G, io):
    """Channels per group that are multiples of the workgroup's 8 channels, smaller than it, and ragged against it."""
    _check(api, oracle, B, D, N, L, G, io, seed=D * 10 + G)


@pytest.mark.parametrize("disc", ["zoh", "bilinear", "dirac"])
def test_grouped_other_discretisations(api, oracle, disc):
    _check(api, oracle, 2, 12, 16, 400, 3, "f32", seed=3, disc=disc)


def test_grouped_backward_without_checkpoints(api, oracle):
    _check(api, oracle, 2, 24, 16, 900, 4, "bf16", seed=5, with_ckpt=False)


def test_one_group_in_4d_layout_equals_the_plain_call(api):
    import torch
    p = workloads.make_selective(B=2, D=16, N=16, L=500, io="bf16", gate=True, seed=8)
    t = dict(u=dev(p["u"], "bf16"), delta=dev(p["delta"], "bf16"), A=dev(p["A"]), Dskip=dev(p["Dskip"]),
             delta_bias=dev(p["delta_bias"]), z=dev(p["z"], "bf16"))
    Bm, Cm = dev(p["Bm"], "bf16"), dev(p["Cm"], "bf16")
    y1 = api.lrnnx_selective_scan_fwd(**t, Bm=Bm, Cm=Cm)
    y2 = api.lrnnx_selective_scan_fwd(**t, Bm=Bm[:, None].contiguous(), Cm=Cm[:, None].contiguous())
    assert torch.equal(y1, y2)


def test_rejects_groups_that_do_not_divide_the_channels(api):
    p = workloads.make_selective(B=1, D=10, N=4, L=32, seed=1, bc_groups=3)
    with pytest.raises(ValueError):
        api.lrnnx_selective_scan_fwd(dev(p["u"]), dev(p["delta"]), dev(p["A"]), dev(p["Bm"]), dev(p["Cm"]))


def test_grouped_chunk_carry_path_equals_single_pass(api, oracle):
    p = workloads.make_selective(B=1, D=24, N=16, L=6000, io="bf16", gate=True, seed=12, bc_groups=3)
    t = dict(u=dev(p["u"], "bf16"), delta=dev(p["delta"], "bf16"), A=dev(p["A"]), Bm=dev(p["Bm"], "bf16"),
             Cm=dev(p["Cm"], "bf16"), Dskip=dev(p["Dskip"]), delta_bias=dev(p["delta_bias"]), z=dev(p["z"], "bf16"))
    yr, _ = oracle.selective_scan_fwd(**{k: p[k] for k in ("u", "delta", "A", "Bm", "Cm", "Dskip", "delta_bias", "z")})
    for path in ("single_pass", "chunk_carry"):
        assert rel_err(host(api.lrnnx_selective_scan_fwd(**t, path=path)), yr) <= TOL["bf16"], path


# ----------------------------------------------------------------------------- complex-A scan with grouped maps
def _cmaps(a, io):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t.to(torch.bfloat16) if io == "bf16" else torch.view_as_complex(t)


def _cplx(a):
    return a[..., 0].astype(np.float64) + 1j * a[..., 1].astype(np.float64)


def _crel(got, ref):
    den = np.abs(ref).max()
    return float(np.abs(np.asarray(got, dtype=np.complex128) - ref).max() / (den if den > 0 else 1.0))


@pytest.mark.parametrize("B,D,N,L,G", [(2, 16, 16, 300, 2), (1, 24, 16, 1000, 3), (2, 20, 8, 257, 4), (1, 6, 16, 700, 6),
                                       (3, 26, 4, 130, 2), (1, 192, 16, 520, 2), (2, 9, 2, 64, 9)])
@pytest.mark.parametrize("io", ["f32", "bf16"])
def test_complex_grouped_shapes(api, oracle, B, D, N, L, G, io):
    import torch
    p = workloads.make_selective_complex(B=B, D=D, N=N, L=L, io=io, gate=True, seed=D * 7 + G, with_x0=True, bc_groups=G)
    dy = workloads._io_round(np.random.Generator(np.random.PCG64(D + G)).standard_normal((B, D, L), dtype=np.float32), io)
    t = dict(u=dev(p["u"], io), delta=dev(p["delta"], io), A=torch.from_numpy(p["A"]).cuda(), Bm=_cmaps(p["Bm"], io),
             Cm=_cmaps(p["Cm"], io), Dskip=dev(p["Dskip"]), delta_bias=dev(p["delta_bias"]), z=dev(p["z"], io),
             x0=torch.from_numpy(p["x0"]).cuda())
    y, x_last, ckpt = api.lrnnx_selective_scan_fwd_complex(**t, disc="zoh", return_last_state=True, return_ckpt=True)
    g = api.lrnnx_selective_scan_bwd_complex(**t, dy=dev(dy, io), disc="zoh", ckpt=ckpt if L % 2 else None, want_dx0=True)
    ref = dict(u=p["u"], delta=p["delta"], A=p["A"], Bm=_cplx(p["Bm"]), Cm=_cplx(p["Cm"]), Dskip=p["Dskip"],
               delta_bias=p["delta_bias"], z=p["z"], x0=p["x0"])
    yr, xr = oracle.selective_scan_fwd_complex(**ref, disc="zoh")
    r = oracle.selective_scan_bwd_complex(dy=dy, **ref, disc="zoh")
    assert rel_err(host(y), yr) <= TOL[io]
    assert _crel(x_last.cpu().numpy(), xr) <= 1e-4
    assert tuple(g["dBm"].shape) == ref["Bm"].shape
    errs = {k: (rel_err(host(g[k]), r[k]), TOL[io]) for k in ("du", "ddelta", "dz")}
    errs.update({k: (rel_err(host(g[k]), r[k]), 1e-4) for k in ("dD", "dbias")})
    errs.update({k: (_crel(g[k].cpu().numpy(), r[k]), 1e-4) for k in ("dA", "dBm", "dCm", "dx0")})
    bad = {k: v for k, v in errs.items() if not v[0] <= v[1]}
    assert not bad, f"{bad} (all {errs})"
    # single-token step with the first step's maps [B,G,N] reproduces the scan's first output
    x = t["x0"].clone()
    y1 = api.lrnnx_selective_step_complex(x, t["u"][:, :, 0], t["delta"][:, :, 0], t["A"], t["Bm"][:, :, 0].contiguous(),
                                          t["Cm"][:, :, 0].contiguous(), Dskip=t["Dskip"], delta_bias=t["delta_bias"],
                                          z=t["z"][:, :, 0], disc="zoh")
    assert rel_err(host(y1), yr[:, :, 0]) <= TOL[io]
