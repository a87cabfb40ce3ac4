"""GPU parity on inputs chosen to reach the branches the random workloads never take.

The kernels evaluate softplus, the exact zero-order hold and its A-derivative piecewise (saturation above s = 20, the
series of log(1 + e^s) below e^s = 1/64, the series of (e^x - 1)/x below |x| = 1/64 and of its derivative below
|x| = 1/8, the A = 0 limit); asynchronous mode may hand in a step size of exactly zero; and the complex scan must
take any phase Delta * Im(A).  Each case places values on both sides of a switch point (or at the special value) on
purpose and compares forward and backward with the fp64 oracle at the float32 bar (1e-4 of max|output|).
"""
import numpy as np
import pytest

from paper_2602_08810_amd import workloads
from _util import check_outputs, dev, host

pytestmark = pytest.mark.gpu

BWD_OUTS = ("du", "ddelta", "dA", "dBm", "dCm", "dD", "dbias", "dz", "dx0")


@pytest.fixture(scope="module")
def api():
    import torch
    assert torch.cuda.is_available()
    from paper_2602_08810_amd import api as _api
    _api.lib()
    return _api


def _fwd_bwd(api, oracle, p, disc, softplus, where, tol=1e-4, io="f32"):
    """Forward and backward through the C ABI against the oracle, every output."""
    t = dict(u=dev(p["u"], io), delta=dev(p["delta"], io), A=dev(p["A"]), Bm=dev(p["Bm"], io), Cm=dev(p["Cm"], io),
             Dskip=dev(p["Dskip"]), delta_bias=dev(p["delta_bias"]), z=dev(p["z"], io), x0=dev(p["x0"]))
    y, x_last, ckpt = api.lrnnx_selective_scan_fwd(**t, disc=disc, delta_softplus=softplus, return_last_state=True,
                                                   return_ckpt=True)
    g = api.lrnnx_selective_scan_bwd(**t, dy=dev(p["dy"], io), ckpt=ckpt, disc=disc, delta_softplus=softplus,
                                     want_dx0=True)
    kw = dict(Dskip=p["Dskip"], delta_bias=p["delta_bias"], z=p["z"], x0=p["x0"], disc=disc, delta_softplus=softplus)
    yr, xr = oracle.selective_scan_fwd(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], **kw)
    r = oracle.selective_scan_bwd(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], p["dy"], **kw)
    io_tol = tol if io == "f32" else 2e-2
    pairs = {"y": (host(y), yr, io_tol), "x_last": (host(x_last), xr, tol)}
    for k in BWD_OUTS:
        if r[k] is not None:
            pairs[k] = (host(g[k]), r[k], io_tol if k in ("du", "ddelta", "dz") else tol)
    return check_outputs(pairs, where=where)


def _base(B, D, N, L, seed, gate=True):
    return workloads.make_selective(B=B, D=D, N=N, L=L, io="f32", gate=gate, bias=None, seed=seed, with_x0=True)


@pytest.mark.parametrize("disc,io", [("zoh_s6", "f32"), ("zoh", "f32"), ("zoh_s6", "bf16")])
def test_softplus_series_log_and_saturation_branches(api, oracle, disc, io):
    """s = delta + bias placed at -30 and -4.2 (series of log1p), -4.1 and 19.9 (logarithm), 20.1 and 40 (saturated:
    softplus(s) = s, derivative 1); the switch points are e^s = 1/64 (s = -4.1589) and s = 20.  With bfloat16 I/O the
    kernels take the logarithm throughout (absolute error 2^-24 in the step size) and the values are the nearest
    bfloat16 numbers, still on both sides of the switch points."""
    p = workloads.make_selective(B=2, D=6, N=16, L=700, io=io, gate=True, bias=None, seed=501, with_x0=True)
    s_values = np.array([-30.0, -4.2, -4.1, 19.9, 20.1, 40.0, -4.1589, 20.0, 0.3, -1.0], dtype=np.float32)
    L = p["delta"].shape[2]
    pattern = s_values[(np.arange(L)[None, None, :] + np.arange(6)[None, :, None] * 3) % len(s_values)]
    p["delta"] = workloads._io_round(np.ascontiguousarray(np.broadcast_to(pattern, p["delta"].shape)), io)
    p["delta_bias"] = np.zeros(6, dtype=np.float32)
    # steps of size 20-40 with A of order -1 wipe the state; keep A small so that the large steps still matter
    p["A"] = (p["A"] * 0.02).astype(np.float32)
    _fwd_bwd(api, oracle, p, disc, True, f"softplus branches, {disc}, {io}", io=io)


def test_softplus_bias_moves_values_across_the_switch_points(api, oracle):
    """The same switch points reached through delta_bias (the kernels add it before the transform)."""
    p = _base(1, 4, 8, 300, seed=502, gate=False)
    p["delta"] = np.tile(np.array([0.0, 0.1, -0.1, 0.05], dtype=np.float32), (1, 4, 75))
    p["delta_bias"] = np.array([-4.1589, 20.0, -30.0, 40.0], dtype=np.float32)
    p["A"] = (p["A"] * 0.02).astype(np.float32)
    _fwd_bwd(api, oracle, p, "zoh_s6", True, "softplus branches through delta_bias")


@pytest.mark.parametrize("io", ["f32", "bf16"])
def test_exact_zoh_A_zero_and_series_switch_points(api, oracle, io):
    """Exact zero-order hold with A = 0 (gain Delta, dg/dA = Delta^2 / 2) and with Delta*A just either side of the
    switch points of the gain series (|x| = 1/64) and of its A-derivative (|x| = 1/8)."""
    B, D, N, L = 2, 5, 16, 600
    p = workloads.make_selective(B=B, D=D, N=N, L=L, io=io, gate=True, bias=None, seed=503, with_x0=True)
    dt = np.float32(0.5)
    x_targets = np.array([0.0, -1 / 64 * 0.98, -1 / 64 * 1.02, -1 / 8 * 0.98, -1 / 8 * 1.02, -1 / 64, -1 / 8, -1e-4,
                          -1e-7, -1 / 64 * 0.999, -1 / 64 * 1.001, -1 / 8 * 0.999, -0.5, -2.0, 0.0, -1 / 100], dtype=np.float64)
    A = np.tile((x_targets / dt).astype(np.float32), (D, 1))
    A[1] = A[1][::-1]
    A[2, :] = 0.0                                   # a channel whose every state has A = 0: a pure integrator
    p["A"] = np.ascontiguousarray(A)
    # Delta = 0.5 (1 +- a few per cent), exactly representable in both I/O types, so Delta*A straddles the targets
    steps = np.array([0.5, 0.5078125, 0.4921875, 0.5], dtype=np.float32)
    p["delta"] = np.ascontiguousarray(np.broadcast_to(steps[np.arange(L) % 4], (B, D, L))).astype(np.float32)
    p["delta_bias"] = None
    # integrators accumulate: keep the drive small so that the outputs stay of order one
    p["u"] = workloads._io_round(p["u"] * 0.05, io)
    _fwd_bwd(api, oracle, p, "zoh", False, f"exact ZOH switch points, {io}", io=io)


@pytest.mark.parametrize("disc", ["zoh_s6", "zoh", "bilinear", "dirac"])
def test_zero_step_size_in_asynchronous_mode(api, oracle, disc):
    """delta_softplus = 0 with Delta = 0 on many steps (events with no time gap): a = 1, and g = 0 (1 for dirac)."""
    p = _base(2, 5, 8, 530, seed=504)
    rng = np.random.Generator(np.random.PCG64(7))
    gaps = rng.uniform(0.01, 0.3, size=p["delta"].shape).astype(np.float32)
    gaps[rng.uniform(size=gaps.shape) < 0.4] = 0.0
    gaps[:, 0, :] = 0.0                             # one channel never advances: x stays x0, y = C x0 + D u
    gaps[:, 1, :64] = 0.0                           # a whole leading lane tile of zeros
    p["delta"] = gaps
    p["delta_bias"] = None
    _fwd_bwd(api, oracle, p, disc, False, f"zero step size, {disc}")


@pytest.mark.parametrize("revs", [0.4, 40.0, 300.0])
def test_complex_scan_takes_any_phase(api, oracle, revs):
    """Complex A with Delta*Im(A) of `revs` revolutions per step (asynchronous mode, so Delta is the caller's).  The
    hardware sine and cosine are valid within +-256 revolutions; the kernels drop whole revolutions first, so neither
    a single step (300) nor the product of a lane's eight steps (8 x 40) may leave that range unnoticed.  The phase of
    a step carries the rounding of the fp32 product Delta*Im(A)/(2 pi), revs * 2^-24 revolutions, and a state with a
    memory of M steps sums M such errors: the bar is max(1e-4, 2 pi * revs * 2^-24 * 4 M) with M = 8 here."""
    import torch
    B, D, N, L = 2, 6, 8, 777
    p = workloads.make_selective_complex(B=B, D=D, N=N, L=L, io="f32", gate=True, seed=505, with_x0=True)
    rng = np.random.Generator(np.random.PCG64(8))
    dt = rng.uniform(0.09, 0.11, size=(B, D, L)).astype(np.float32)
    p["delta"] = dt
    p["delta_bias"] = None
    im = (2 * np.pi * revs / 0.1) * rng.uniform(0.9, 1.1, size=(D, N)) * rng.choice([-1.0, 1.0], size=(D, N))
    p["A"] = (-np.exp(rng.uniform(0.0, 0.5, size=(D, N))) + 1j * im).astype(np.complex64)   # memory 1/(0.1 |Re A|) <= 10 steps
    tol = max(1e-4, 2 * np.pi * revs * 2.0 ** -24 * 32)
    cplx = lambda a: torch.view_as_complex(torch.from_numpy(np.ascontiguousarray(a)).cuda())
    t = dict(u=dev(p["u"]), delta=dev(p["delta"]), A=torch.from_numpy(p["A"]).cuda(), Bm=cplx(p["Bm"]), Cm=cplx(p["Cm"]),
             Dskip=dev(p["Dskip"]), z=dev(p["z"]), x0=torch.from_numpy(p["x0"]).cuda())
    y, x_last, ckpt = api.lrnnx_selective_scan_fwd_complex(**t, delta_softplus=False, return_last_state=True, return_ckpt=True)
    dy = workloads.make_selective(B=B, D=D, N=1, L=L, io="f32", seed=506)["dy"]
    g = api.lrnnx_selective_scan_bwd_complex(**t, dy=dev(dy), ckpt=ckpt, delta_softplus=False, want_dx0=True)
    Bc = p["Bm"][..., 0] + 1j * p["Bm"][..., 1]
    Cc = p["Cm"][..., 0] + 1j * p["Cm"][..., 1]
    kw = dict(Dskip=p["Dskip"], z=p["z"], x0=p["x0"], delta_softplus=False)
    yr, xr = oracle.selective_scan_fwd_complex(p["u"], p["delta"], p["A"], Bc, Cc, **kw)
    r = oracle.selective_scan_bwd_complex(p["u"], p["delta"], p["A"], Bc, Cc, dy, **kw)
    pairs = {"y": (host(y), yr, tol), "x_last.re": (x_last.cpu().numpy().real, xr.real, tol),
             "x_last.im": (x_last.cpu().numpy().imag, xr.imag, tol)}
    for k in ("du", "ddelta", "dz", "dD"):
        pairs[k] = (host(g[k]), r[k], tol)
    for k in ("dA", "dBm", "dCm", "dx0"):
        got = g[k].cpu().numpy()
        pairs[k + ".re"] = (got.real, r[k].real, tol)
        pairs[k + ".im"] = (got.imag, r[k].imag, tol)
    check_outputs(pairs, where=f"complex scan at {revs} revolutions per step")
