"""The library calls can be captured in a HIP graph and replayed (Sec. 4.2 of the paper runs generation under
graph capture to remove per-token launch overhead): every call only enqueues kernels on the caller's stream, and
buffers are cleared by fill kernels.  Each graph is replayed several times with eager work in between and every
replay is checked against the eager result."""
import pytest

from paper_2602_08810_amd import workloads
from _util import dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api():
    import torch
    assert torch.cuda.is_available()
    from paper_2602_08810_amd import api as _api
    _api.lib()
    return _api


def _eager_noise(torch):
    """Unrelated eager work and a synchronisation between replays."""
    a = torch.randn(512, 512, device="cuda")
    (a @ a).sum().item()


def test_generation_loop_of_step_calls_replays(api):
    import torch
    T, B, D, N = 12, 4, 64, 16
    g = torch.Generator(device="cuda").manual_seed(1)
    bf = torch.bfloat16
    r = lambda *s: torch.randn(*s, device="cuda", generator=g)
    u, dl, z = r(T, B, D).to(bf), r(T, B, D).to(bf), r(T, B, D).to(bf)
    Bm, Cm = r(T, B, N).to(bf), r(T, B, N).to(bf)
    A, Dk, bias = -torch.exp(r(D, N) * 0.5), r(D), r(D) - 3
    x_init = r(B, D, N)

    def loop(x, y):
        for t in range(T):
            api.lrnnx_selective_step(x, u[t], dl[t], A, Bm[t], Cm[t], Dskip=Dk, delta_bias=bias, z=z[t], out=y[t])

    x_ref, y_ref = x_init.clone(), torch.empty(T, B, D, dtype=bf, device="cuda")
    loop(x_ref, y_ref)
    torch.cuda.synchronize()

    x, y = x_init.clone(), torch.empty(T, B, D, dtype=bf, device="cuda")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        loop(x, y)
    for _ in range(3):
        x.copy_(x_init)
        y.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, y_ref) and torch.equal(x, x_ref)
        _eager_noise(torch)


@pytest.mark.parametrize("path", ["single_pass", "chunk_carry"])
def test_forward_backward_pair_replays(api, path):
    """Forward + backward captured in one graph; the chunked backward path (three more launches, its aggregates in
    the workspace) replays like the single pass."""
    import torch
    p = workloads.make_selective(B=2, D=32, N=16, L=1500, io="bf16", gate=True, seed=4, bias=("uniform", -4.0, -2.0))
    t = dict(u=dev(p["u"], "bf16"), delta=dev(p["delta"], "bf16"), A=dev(p["A"]), Bm=dev(p["Bm"], "bf16"),
             Cm=dev(p["Cm"], "bf16"), Dskip=dev(p["Dskip"]), delta_bias=dev(p["delta_bias"]), z=dev(p["z"], "bf16"))
    dy = dev(p["dy"], "bf16")
    y_ref, ck_ref = api.lrnnx_selective_scan_fwd(**t, return_ckpt=True)
    g_ref = api.lrnnx_selective_scan_bwd(**t, dy=dy, ckpt=ck_ref, path=path)
    torch.cuda.synchronize()

    y, ck = torch.empty_like(y_ref), torch.empty_like(ck_ref)
    outs = {k: torch.empty_like(v) for k, v in g_ref.items() if v is not None}
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        api.lrnnx_selective_scan_fwd(**t, out=y, ckpt_out=ck, workspace=ws)
        api.lrnnx_selective_scan_bwd(**t, dy=dy, ckpt=ck, outs=outs, workspace=ws, path=path)
    for _ in range(3):
        for v in (y, ck, *outs.values()):
            v.fill_(7.0)                                   # stale contents must not survive a replay
        ws.fill_(255)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, y_ref) and torch.equal(ck, ck_ref)
        for k in ("du", "ddelta", "dz"):
            assert torch.equal(outs[k], g_ref[k]), k
        for k in ("dA", "dBm", "dCm", "dD", "dbias"):    # float atomics: equal up to summation order
            scale = float(g_ref[k].abs().max())
            assert float((outs[k] - g_ref[k]).abs().max()) <= 1e-5 * scale, k
        _eager_noise(torch)


def test_complex_forward_backward_pair_replays(api):
    import numpy as np
    import torch
    p = workloads.make_selective_complex(B=2, D=40, N=16, L=1100, io="bf16", gate=True, seed=8, with_x0=True)
    bf = torch.bfloat16
    maps = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda().to(bf)
    t = dict(u=dev(p["u"], "bf16"), delta=dev(p["delta"], "bf16"), A=torch.from_numpy(p["A"]).cuda(), Bm=maps(p["Bm"]),
             Cm=maps(p["Cm"]), Dskip=dev(p["Dskip"]), delta_bias=dev(p["delta_bias"]), z=dev(p["z"], "bf16"),
             x0=torch.from_numpy(p["x0"]).cuda())
    dy = dev(p["u"][:, :, ::-1].copy(), "bf16")
    y_ref, ck_ref = api.lrnnx_selective_scan_fwd_complex(**t, return_ckpt=True)
    g_ref = api.lrnnx_selective_scan_bwd_complex(**t, dy=dy, ckpt=ck_ref, want_dx0=True)
    torch.cuda.synchronize()

    y, ck = torch.empty_like(y_ref), torch.empty_like(ck_ref)
    outs = {k: torch.empty_like(v) for k, v in g_ref.items() if v is not None}
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        api.lrnnx_selective_scan_fwd_complex(**t, out=y, ckpt_out=ck)
        api.lrnnx_selective_scan_bwd_complex(**t, dy=dy, ckpt=ck, outs=outs, want_dx0=True)
    for _ in range(3):
        for v in (y, ck, *outs.values()):
            v.fill_(7.0)                                   # stale contents must not survive a replay
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, y_ref) and torch.equal(torch.view_as_real(ck), torch.view_as_real(ck_ref))
        for k in ("du", "ddelta", "dz"):
            assert torch.equal(outs[k], g_ref[k]), k
        assert torch.equal(torch.view_as_real(outs["dx0"]), torch.view_as_real(g_ref["dx0"]))
        for k in ("dA", "dBm", "dCm", "dD", "dbias"):    # float atomics: equal up to summation order
            scale = float(g_ref[k].abs().max())
            assert float((outs[k] - g_ref[k]).abs().max()) <= 1e-5 * scale, k
        _eager_noise(torch)


def test_chained_scans_replay(api):
    """The single-launch LTI scan, its adjoint and the caller-coefficient scan re-arm their workspace on every replay."""
    import torch
    q = workloads.make_lti(B=2, P=192, L=5000, seed=6, with_x0=True, with_gx=True)
    lam, v, x0, gx = (torch.from_numpy(q[k]).cuda() for k in ("lam", "v", "x0", "gx"))
    x_ref = api.lrnnx_lti_diag_scan(lam, v, x0=x0)
    dv_ref, dlam_ref, _ = api.lrnnx_lti_diag_scan_bwd(lam, x_ref, gx, x0=x0)
    a = lam.expand_as(v).contiguous()
    xd_ref = api.lrnnx_diag_scan(a, v, x0=x0)
    torch.cuda.synchronize()

    x, dv, xd = torch.empty_like(v), torch.empty_like(v), torch.empty_like(v)
    ws = [torch.empty(4 << 20, dtype=torch.uint8, device="cuda") for _ in range(3)]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        api.lrnnx_lti_diag_scan(lam, v, x0=x0, out=x, workspace=ws[0])
        _, dlam, _ = api.lrnnx_lti_diag_scan_bwd(lam, x, gx, x0=x0, out=dv, workspace=ws[1])
        api.lrnnx_diag_scan(a, v, x0=x0, out=xd, workspace=ws[2])
    for _ in range(3):
        for t_ in (x, dv, xd):
            t_.fill_(0)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(x, x_ref) and torch.equal(dv, dv_ref) and torch.equal(xd, xd_ref)
        assert float((dlam - dlam_ref).abs().max()) <= 1e-5 * float(dlam_ref.abs().max())
        assert bool(x.isfinite().all())
        _eager_noise(torch)
