"""GPU parity: lrnnx_selective_scan_bwd_complex (backward of the selective scan with a complex diagonal A, through
the C ABI) against the fp64 oracle.  Every gradient is compared relative to the largest magnitude of the oracle's
array, as for the real scan: du, ddelta, dz within 1e-4 (float32 I/O) or 2e-2 (bfloat16 I/O); the float32 outputs
dA, dBm, dCm, dD, dbias, dx0 within 1e-4."""
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
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t.to(torch.bfloat16) if io == "bf16" else torch.view_as_complex(t)


GRAD_TOL_F32 = 1e-4      # the float32 outputs (reduced gradients), whatever the I/O type


def _crel(got, ref):
    """max |got - ref| / max |ref| over a complex array."""
    den = np.abs(ref).max()
    return float(np.abs(np.asarray(got, dtype=np.complex128) - ref).max() / (den if den > 0 else 1.0))


def _run(api, oracle, B, D, N, L, io, disc, gate, x0, seed, softplus=True, use_ckpt=False, bias=True, skip=True,
         path="auto", groups=1):
    import torch
    p = workloads.make_selective_complex(B=B, D=D, N=N, L=L, io=io, gate=gate, seed=seed, with_x0=x0, bc_groups=groups)
    rng = np.random.Generator(np.random.PCG64(seed + 77))
    dy = workloads._io_round(rng.standard_normal((B, D, L), dtype=np.float32), io)
    if not softplus:
        p["delta"] = workloads._io_round(np.abs(p["delta"]) * 0.1 + 0.01, io)
        p["delta_bias"] = None
    if not bias:
        p["delta_bias"] = None
    if not skip:
        p["Dskip"] = None
    t = dict(u=dev(p["u"], io), delta=dev(p["delta"], io), A=torch.from_numpy(p["A"]).cuda(), Bm=_maps_dev(p["Bm"], io),
             Cm=_maps_dev(p["Cm"], io), Dskip=dev(p["Dskip"]), delta_bias=dev(p["delta_bias"]), z=dev(p["z"], io),
             x0=None if p["x0"] is None else torch.from_numpy(p["x0"]).cuda())
    ckpt = None
    if use_ckpt:
        _, ckpt = api.lrnnx_selective_scan_fwd_complex(**t, disc=disc, delta_softplus=softplus, return_ckpt=True)
    g = api.lrnnx_selective_scan_bwd_complex(**t, dy=dev(dy, io), ckpt=ckpt, disc=disc, delta_softplus=softplus,
                                             want_dx0=True, path=path)
    torch.cuda.synchronize()
    r = oracle.selective_scan_bwd_complex(p["u"], p["delta"], p["A"], _cplx(p["Bm"]), _cplx(p["Cm"]), dy, Dskip=p["Dskip"],
                                          delta_bias=p["delta_bias"], z=p["z"], x0=p["x0"], disc=disc,
                                          delta_softplus=softplus)
    errs = {}
    for k in ("du", "ddelta", "dz"):
        if r[k] is not None:
            errs[k] = (rel_err(host(g[k]), r[k]), TOL[io])
    for k in ("dD", "dbias"):
        if r[k] is not None:
            errs[k] = (rel_err(host(g[k]), r[k]), GRAD_TOL_F32)
    for k in ("dA", "dBm", "dCm", "dx0"):
        errs[k] = (_crel(g[k].cpu().numpy(), r[k]), GRAD_TOL_F32)
    bad = {k: v for k, v in errs.items() if not v[0] <= v[1]}
    assert not bad, f"rel errors over tolerance: {bad}  (all: {errs})"
    return g


@pytest.mark.parametrize("io", ["f32", "bf16"])
@pytest.mark.parametrize("disc", DISCS)
def test_all_discretisations(api, oracle, io, disc):
    _run(api, oracle, 2, 10, 16, 700, io, disc, gate=True, x0=True, seed=1)


@pytest.mark.parametrize("io", ["f32", "bf16"])
@pytest.mark.parametrize("B,D,N,L", [(1, 1, 1, 1), (2, 3, 2, 7), (1, 13, 4, 511), (3, 8, 8, 513), (1, 9, 16, 1025),
                                     (2, 70, 16, 600)])
def test_shapes(api, oracle, io, B, D, N, L):
    _run(api, oracle, B, D, N, L, io, "zoh_s6", gate=bool(L % 2), x0=bool(D % 2), seed=B + D + N + L)


@pytest.mark.parametrize("disc", ["zoh_s6", "bilinear"])
def test_checkpoints_from_the_forward_call(api, oracle, disc):
    _run(api, oracle, 2, 12, 16, 1500, "f32", disc, gate=True, x0=True, seed=3, use_ckpt=True)


def test_caller_supplied_step_sizes_no_bias_no_skip(api, oracle):
    _run(api, oracle, 2, 6, 16, 700, "f32", "zoh", gate=False, x0=True, seed=5, softplus=False, skip=False)


def test_long_sequence(api, oracle):
    _run(api, oracle, 1, 8, 16, 9000, "bf16", "zoh_s6", gate=True, x0=False, seed=6)


def test_mamba_block_shape_full(api, oracle):
    """The shape bench.py times for the complex-A scan (B=8, D=1536, N=16, L=2048, bf16 I/O, gate), in the same launch
    configuration (checkpoints from the forward call): every output of both passes against the oracle."""
    import torch
    B, D, N, L, io = 8, 1536, 16, 2048, "bf16"
    p = workloads.make_selective_complex(B=B, D=D, N=N, L=L, io=io, gate=True, seed=2)
    dy = workloads._io_round(np.random.Generator(np.random.PCG64(99)).standard_normal((B, D, L), dtype=np.float32), io)
    t = dict(u=dev(p["u"], io), delta=dev(p["delta"], io), A=torch.from_numpy(p["A"]).cuda(), Bm=_maps_dev(p["Bm"], io),
             Cm=_maps_dev(p["Cm"], io), Dskip=dev(p["Dskip"]), delta_bias=dev(p["delta_bias"]), z=dev(p["z"], io))
    y, ckpt = api.lrnnx_selective_scan_fwd_complex(**t, return_ckpt=True)
    g = api.lrnnx_selective_scan_bwd_complex(**t, dy=dev(dy, io), ckpt=ckpt)
    torch.cuda.synchronize()
    kw = dict(Dskip=p["Dskip"], delta_bias=p["delta_bias"], z=p["z"])
    Bc, Cc = _cplx(p["Bm"]), _cplx(p["Cm"])
    yr, _ = oracle.selective_scan_fwd_complex(p["u"], p["delta"], p["A"], Bc, Cc, **kw)
    assert rel_err(host(y), yr) <= TOL[io], "y"
    del yr
    r = oracle.selective_scan_bwd_complex(p["u"], p["delta"], p["A"], Bc, Cc, dy, **kw)
    errs = {k: (rel_err(host(g[k]), r[k]), TOL[io]) for k in ("du", "ddelta", "dz")}
    errs.update({k: (rel_err(host(g[k]), r[k]), GRAD_TOL_F32) for k in ("dD", "dbias")})
    errs.update({k: (_crel(g[k].cpu().numpy(), r[k]), GRAD_TOL_F32) for k in ("dA", "dBm", "dCm")})
    bad = {k: v for k, v in errs.items() if not v[0] <= v[1]}
    assert not bad, f"rel errors over tolerance: {bad}  (all: {errs})"


def test_real_data_reproduces_the_real_backward(api):
    """With zero imaginary parts the complex entry point returns the real kernel's gradients (real parts) and no
    imaginary gradient for Cm; the other complex gradients' real parts agree too."""
    import torch
    p = workloads.make_selective(B=2, D=12, N=16, L=900, io="f32", gate=True, seed=7)
    t = dict(u=dev(p["u"]), delta=dev(p["delta"]), Dskip=dev(p["Dskip"]), delta_bias=dev(p["delta_bias"]), z=dev(p["z"]),
             dy=dev(p["dy"]))
    g = api.lrnnx_selective_scan_bwd(**t, A=dev(p["A"]), Bm=dev(p["Bm"]), Cm=dev(p["Cm"]))
    c64 = torch.complex64
    gc = api.lrnnx_selective_scan_bwd_complex(**t, A=dev(p["A"]).to(c64), Bm=dev(p["Bm"]).to(c64), Cm=dev(p["Cm"]).to(c64))
    for k in ("du", "ddelta", "dz", "dD", "dbias"):
        assert rel_err(host(gc[k]), host(g[k]).astype(np.float64)) <= 2e-5, k
    for k in ("dA", "dBm", "dCm"):
        assert rel_err(gc[k].real.cpu().numpy(), host(g[k]).astype(np.float64)) <= 2e-5, k


def test_bad_arguments_are_rejected(api):
    import torch
    p = workloads.make_selective_complex(B=1, D=4, N=16, L=64, io="f32", gate=False, seed=9)
    t = dict(u=dev(p["u"]), delta=dev(p["delta"]), A=torch.from_numpy(p["A"]).cuda(), Bm=_maps_dev(p["Bm"], "f32"),
             Cm=_maps_dev(p["Cm"], "f32"), dy=dev(p["u"]))
    with pytest.raises(ValueError):
        api.lrnnx_selective_scan_bwd_complex(**dict(t, A=t["A"].real.contiguous()))
    with pytest.raises(ValueError):
        api.lrnnx_selective_scan_bwd_complex(**t, ckpt=torch.zeros((1, 4, 2, 16), dtype=torch.complex64, device="cuda"))
    with pytest.raises(RuntimeError):                    # workspace too small for the checkpoints
        api.lrnnx_selective_scan_bwd_complex(**t, workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))


@pytest.mark.parametrize("io", ["f32", "bf16"])
@pytest.mark.parametrize("disc", DISCS)
def test_chunked_over_time(api, oracle, io, disc):
    """path = chunk_carry: chunks of the time axis side by side, each started from the adjoint carried in from the
    later chunks (ragged last chunk, with and without the forward pass's checkpoints)."""
    _run(api, oracle, 1, 5, 16, 2100, io, disc, True, True, seed=300, use_ckpt=True, path="chunk_carry")
    _run(api, oracle, 2, 9, 4, 1300, io, disc, False, True, seed=301, use_ckpt=False, path="chunk_carry")


@pytest.mark.parametrize("N", [1, 2, 8])
def test_chunked_over_time_state_sizes_and_groups(api, oracle, N):
    _run(api, oracle, 2, 12, N, 1800, "bf16", "zoh_s6", True, False, seed=310 + N, use_ckpt=True, path="chunk_carry", groups=3)
    _run(api, oracle, 1, 3, N, 257, "f32", "zoh_s6", True, True, seed=320 + N, softplus=False, use_ckpt=True, path="chunk_carry")


def test_auto_path_chunks_long_sequences_with_few_rows(api, oracle):
    assert api.lib().lrnnx_selective_scan_bwd_chunks(1, 8, 16, 8192, 1, 0, 1) > 1
    _run(api, oracle, 1, 8, 16, 8192, "bf16", "zoh_s6", True, True, seed=330, use_ckpt=True, path="auto")
    _run(api, oracle, 1, 8, 16, 8192, "bf16", "zoh_s6", True, True, seed=330, use_ckpt=True, path="single_pass")
