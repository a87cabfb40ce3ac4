"""GPU parity: lrnnx_selective_scan_fwd_complex (complex diagonal A, complex maps, y = Re(C x) + D u; through the
C ABI) against the fp64 oracle.  Tolerances as for the real scan: 1e-4 (fp32 I/O), 2e-2 (bf16 I/O) of max|y|."""
import numpy as np
import pytest

from paper_2602_08810_amd import workloads
from _util import TOL, dev, host, rel_err

pytestmark = pytest.mark.gpu

DISCS = ["zoh_s6", "zoh", "bilinear", "dirac"]


@pytest.fixture(scope="module")
def api():
    import torch
    assert torch.cuda.is_available()
    from paper_2602_08810_amd import api as _api
    _api.lib()
    return _api


def _cplx(a):
    return a[..., 0].astype(np.float64) + 1j * a[..., 1].astype(np.float64)


def _maps_dev(a, io):
    """[B,L,N,2] float32 (already rounded) -> the tensor the binding wants for this I/O type."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t.to(torch.bfloat16) if io == "bf16" else torch.view_as_complex(t)


def _run(api, oracle, B, D, N, L, io, disc, gate, x0, seed, softplus=True, path="auto", groups=1):
    import torch
    p = workloads.make_selective_complex(B=B, D=D, N=N, L=L, io=io, gate=gate, seed=seed, with_x0=x0, bc_groups=groups)
    if not softplus:
        p["delta"] = workloads._io_round(np.abs(p["delta"]) * 0.1 + 0.01, io)
        p["delta_bias"] = None
    t = dict(u=dev(p["u"], io), delta=dev(p["delta"], io), A=torch.from_numpy(p["A"]).cuda(), Bm=_maps_dev(p["Bm"], io),
             Cm=_maps_dev(p["Cm"], io), Dskip=dev(p["Dskip"]), delta_bias=dev(p["delta_bias"]), z=dev(p["z"], io),
             x0=None if p["x0"] is None else torch.from_numpy(p["x0"]).cuda())
    y, x_last = api.lrnnx_selective_scan_fwd_complex(**t, disc=disc, delta_softplus=softplus, return_last_state=True,
                                                     path=path)
    yr, xr = oracle.selective_scan_fwd_complex(p["u"], p["delta"], p["A"], _cplx(p["Bm"]), _cplx(p["Cm"]), Dskip=p["Dskip"],
                                               delta_bias=p["delta_bias"], z=p["z"], x0=p["x0"], disc=disc,
                                               delta_softplus=softplus)
    assert rel_err(host(y), yr) <= TOL[io], "y"
    xl = x_last.cpu().numpy()
    assert max(rel_err(xl.real, xr.real), rel_err(xl.imag, xr.imag)) <= 1e-4, "x_last"


@pytest.mark.parametrize("io", ["f32", "bf16"])
@pytest.mark.parametrize("disc", DISCS)
def test_all_discretisations(api, oracle, io, disc):
    _run(api, oracle, 2, 10, 16, 1300, io, disc, gate=True, x0=True, seed=1)


@pytest.mark.parametrize("io", ["f32", "bf16"])
@pytest.mark.parametrize("B,D,N,L", [(1, 1, 1, 1), (2, 3, 2, 7), (1, 13, 4, 511), (3, 8, 8, 513), (1, 9, 16, 1025),
                                     (2, 24, 16, 2048)])
def test_shapes(api, oracle, io, B, D, N, L):
    _run(api, oracle, B, D, N, L, io, "zoh_s6", gate=bool(L % 2), x0=bool(D % 2), seed=B + D + N + L)


@pytest.mark.parametrize("io", ["f32", "bf16"])
@pytest.mark.parametrize("N", [1, 2, 4, 8, 16])
def test_state_sizes_on_short_tiles(api, oracle, io, N):
    """Row lengths the launch walks in 256-step tiles (four channels per workgroup): three tiles with a ragged tail,
    and one tile not even half full; D not a multiple of four."""
    _run(api, oracle, 2, 13, N, 700, io, "zoh_s6", gate=True, x0=True, seed=70 + N)
    _run(api, oracle, 3, 6, N, 100, io, "bilinear", gate=False, x0=False, seed=90 + N)


def test_caller_supplied_step_sizes(api, oracle):
    _run(api, oracle, 2, 6, 16, 700, "f32", "zoh", gate=False, x0=True, seed=5, softplus=False)


def test_long_sequence(api, oracle):
    _run(api, oracle, 1, 8, 16, 20000, "bf16", "zoh_s6", gate=True, x0=False, seed=6)


def test_real_data_reproduces_the_real_kernel(api):
    """With zero imaginary parts the complex entry point computes what the real one does."""
    import torch
    p = workloads.make_selective(B=2, D=12, N=16, L=900, io="f32", gate=True, seed=7, with_dy=False)
    t = dict(u=dev(p["u"]), delta=dev(p["delta"]), Dskip=dev(p["Dskip"]), delta_bias=dev(p["delta_bias"]), z=dev(p["z"]))
    y = api.lrnnx_selective_scan_fwd(**t, A=dev(p["A"]), Bm=dev(p["Bm"]), Cm=dev(p["Cm"]))
    yc = api.lrnnx_selective_scan_fwd_complex(**t, A=dev(p["A"]).to(torch.complex64), Bm=dev(p["Bm"]).to(torch.complex64),
                                              Cm=dev(p["Cm"]).to(torch.complex64))
    assert float((y - yc).abs().max()) <= 2e-5 * float(y.abs().max())


def test_two_calls_chained_through_the_state_equal_one_call(api, oracle):
    """Chunked prefill: the second call starts from the first call's x_last (x0); y of both calls is what one call
    over the whole sequence gives, on the GPU and against the oracle."""
    import torch
    B, D, N, L, cut, io = 2, 12, 16, 1400, 777, "f32"
    p = workloads.make_selective_complex(B=B, D=D, N=N, L=L, io=io, gate=True, seed=11, with_x0=True)
    full = dict(u=dev(p["u"]), delta=dev(p["delta"]), A=torch.from_numpy(p["A"]).cuda(), Bm=_maps_dev(p["Bm"], io),
                Cm=_maps_dev(p["Cm"], io), Dskip=dev(p["Dskip"]), delta_bias=dev(p["delta_bias"]), z=dev(p["z"]))
    x0 = torch.from_numpy(p["x0"]).cuda()
    y, xl = api.lrnnx_selective_scan_fwd_complex(**full, x0=x0, return_last_state=True)
    part = lambda lo, hi: dict(full, u=full["u"][:, :, lo:hi], delta=full["delta"][:, :, lo:hi], z=full["z"][:, :, lo:hi],
                               Bm=full["Bm"][:, lo:hi].contiguous(), Cm=full["Cm"][:, lo:hi].contiguous())
    y1, xl1 = api.lrnnx_selective_scan_fwd_complex(**part(0, cut), x0=x0, return_last_state=True)
    y2, xl2 = api.lrnnx_selective_scan_fwd_complex(**part(cut, L), x0=xl1, return_last_state=True)
    yy = torch.cat([y1, y2], dim=2)
    assert float((yy - y).abs().max()) <= 2e-6 * float(y.abs().max())
    assert float((xl2 - xl).abs().max()) <= 2e-6 * float(xl.abs().max())
    yr, xr = oracle.selective_scan_fwd_complex(p["u"], p["delta"], p["A"], _cplx(p["Bm"]), _cplx(p["Cm"]), Dskip=p["Dskip"],
                                               delta_bias=p["delta_bias"], z=p["z"], x0=p["x0"])
    assert rel_err(host(yy), yr) <= TOL[io]


@pytest.mark.parametrize("io", ["f32", "bf16"])
@pytest.mark.parametrize("disc", DISCS)
def test_chunk_carry_path(api, oracle, io, disc):
    """Aggregate per chunk, chain, rerun from the true carry-in: ragged last chunk, initial state, every scheme."""
    _run(api, oracle, 1, 5, 16, 2100, io, disc, gate=True, x0=True, seed=400, path="chunk_carry")
    _run(api, oracle, 2, 9, 4, 1300, io, disc, gate=False, x0=False, seed=401, path="chunk_carry", groups=3)


def test_chunk_carry_checkpoints_feed_the_backward_pass(api, oracle):
    """The checkpoints written by the chunked forward are those of the single pass (the backward restarts from them)."""
    import torch
    p = workloads.make_selective_complex(B=1, D=6, N=8, L=4096, io="bf16", gate=True, seed=402, with_x0=True)
    t = dict(u=dev(p["u"], "bf16"), delta=dev(p["delta"], "bf16"), A=torch.from_numpy(p["A"]).cuda(),
             Bm=_maps_dev(p["Bm"], "bf16"), Cm=_maps_dev(p["Cm"], "bf16"), Dskip=dev(p["Dskip"]),
             delta_bias=dev(p["delta_bias"]), z=dev(p["z"], "bf16"), x0=torch.from_numpy(p["x0"]).cuda())
    assert api.lib().lrnnx_selective_scan_fwd_complex_chunks(1, 6, 8, 4096, 1, 0) > 1      # the automatic choice chunks
    y1, x1, c1 = api.lrnnx_selective_scan_fwd_complex(**t, return_last_state=True, return_ckpt=True, path="single_pass")
    y2, x2, c2 = api.lrnnx_selective_scan_fwd_complex(**t, return_last_state=True, return_ckpt=True, path="auto")
    scale = float(torch.view_as_real(c1).abs().max())
    assert float(torch.view_as_real(c1 - c2).abs().max()) <= 1e-5 * scale
    assert float(torch.view_as_real(x1 - x2).abs().max()) <= 1e-5 * float(torch.view_as_real(x1).abs().max())
    assert float((y1.float() - y2.float()).abs().max()) <= 2e-2 * float(y1.float().abs().max())
    with pytest.raises(api.LrnnxError) as e:
        api.lrnnx_selective_scan_fwd_complex(**t, path="chunk_carry", workspace=torch.empty(64, dtype=torch.uint8, device="cuda"))
    assert e.value.code == 3
