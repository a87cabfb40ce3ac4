"""GPU parity at the FULL sizes of the benchmark configurations 1-4, in the launch configuration bench.py times.

Every output of every configuration is compared with the oracle element by element.  Configs 3 and 4 are too large
for one oracle call in host memory, so the oracle runs on blocks of channels (config 3) or one batch entry at a time
(config 4): rows (b,d) are independent recurrences and the shared-parameter gradients dBm, dCm of a batch entry need
only that entry's rows.  Config 4 also keeps the identities that hold at any size:
    <dBm, Bm> = <dCm, Cm> = <du, u> - sum_d Dskip[d] dD[d]        (ypre - Dskip*u is bilinear in (Bm, Cm), linear in u)
"""
import numpy as np
import pytest

from paper_2602_08810_amd import workloads
from _util import TOL, check_outputs, dev, host, rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api():
    import torch
    assert torch.cuda.is_available()
    from paper_2602_08810_amd import api as _api
    _api.lib()
    return _api


def _upload(p, io):
    return dict(u=dev(p["u"], io), delta=dev(p["delta"], io), A=dev(p["A"]), Bm=dev(p["Bm"], io), Cm=dev(p["Cm"], io),
                Dskip=dev(p["Dskip"]), delta_bias=dev(p["delta_bias"]), z=dev(p["z"], io))


def _rows(p, b, ds):
    """Sub-problem of batch entry b (or all if None) and channels ds, for the oracle."""
    bs = slice(None) if b is None else slice(b, b + 1)
    q = dict(u=p["u"][bs][:, ds], delta=p["delta"][bs][:, ds], A=p["A"][ds], Bm=p["Bm"][bs], Cm=p["Cm"][bs],
             Dskip=p["Dskip"][ds], delta_bias=p["delta_bias"][ds])
    q["z"] = p["z"][bs][:, ds] if p["z"] is not None else None
    return q


def test_config1_lti_full(api, oracle):
    import torch
    q, cfg = workloads.make("c1")
    x = api.lrnnx_lti_diag_scan(torch.from_numpy(q["lam"]).cuda(), torch.from_numpy(q["v"]).cuda()).cpu().numpy()
    ref = oracle.lti_diag_scan(q["lam"], q["v"])
    assert rel_err(x.real, ref.real) <= 1e-4 and rel_err(x.imag, ref.imag) <= 1e-4


def test_config2_fwd_bwd_full(api, oracle):
    """Every output of the forward and the backward pass against the oracle on the whole config-2 workload."""
    p, cfg = workloads.make("c2")
    t = _upload(p, "bf16")
    y, ckpt = api.lrnnx_selective_scan_fwd(**t, return_ckpt=True)
    g = api.lrnnx_selective_scan_bwd(**t, dy=dev(p["dy"], "bf16"), ckpt=ckpt)
    yr, _ = oracle.selective_scan_fwd(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], Dskip=p["Dskip"],
                                      delta_bias=p["delta_bias"], z=p["z"])
    assert rel_err(host(y), yr) <= TOL["bf16"]
    del yr
    r = oracle.selective_scan_bwd(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], p["dy"], Dskip=p["Dskip"],
                                  delta_bias=p["delta_bias"], z=p["z"])
    errs = {k: rel_err(host(g[k]), r[k]) for k in ("du", "ddelta", "dz", "dA", "dBm", "dCm", "dD", "dbias")}
    tol = {"du": 2e-2, "ddelta": 2e-2, "dz": 2e-2, "dA": 1e-4, "dBm": 1e-4, "dCm": 1e-4, "dD": 1e-4, "dbias": 1e-4}
    bad = {k: v for k, v in errs.items() if not v <= tol[k]}
    assert not bad, f"{bad} (all {errs})"


def test_config3_long_forward_all_rows(api, oracle):
    """L = 65536: both forward paths (in-kernel carry over 128 tiles; three-launch chunk carry), every one of the
    2048 channels against the oracle (run in blocks of channels to bound host memory)."""
    p, cfg = workloads.make("c3", with_dy=False)
    D = cfg["D"]
    t = _upload(p, "bf16")
    outs = {path: api.lrnnx_selective_scan_fwd(**t, path=path, return_last_state=True)
            for path in ("single_pass", "chunk_carry")}
    got = {path: (host(y), host(xl)) for path, (y, xl) in outs.items()}
    del outs, t
    worst = {}
    for d0 in range(0, D, 256):
        ds = np.arange(d0, min(D, d0 + 256))
        q = _rows(p, 0, ds)
        yr, xr = oracle.selective_scan_fwd(q["u"], q["delta"], q["A"], q["Bm"], q["Cm"], Dskip=q["Dskip"],
                                           delta_bias=q["delta_bias"])
        for path, (y, xl) in got.items():
            rep = check_outputs({"y": (y[:, ds], yr, TOL["bf16"]), "x_last": (xl[:, ds], xr, 1e-4)},
                                where=f"config 3 {path} channels {d0}..{ds[-1]}")
            worst[(path, d0)] = rep
    assert len(worst) == 2 * ((D + 255) // 256)


def test_config4_backward_all_rows(api, oracle):
    """Every output of config 4's backward pass, element by element, in the launch shape bench.py times (80 channels
    per workgroup, 16 tiles): the oracle runs one batch entry at a time (rows are independent; dA, dD, dbias are sums
    over batch entries and are accumulated here in fp64), which bounds host memory."""
    import torch
    p, cfg = workloads.make("c4")
    B, D, N, L = cfg["B"], cfg["D"], cfg["N"], cfg["L"]
    t = _upload(p, "bf16")
    dy = dev(p["dy"], "bf16")
    y, ckpt = api.lrnnx_selective_scan_fwd(**t, return_ckpt=True)
    g = api.lrnnx_selective_scan_bwd(**t, dy=dy, ckpt=ckpt)
    torch.cuda.synchronize()
    gh = {k: host(v) for k, v in g.items()}
    yh = host(y)
    del y, ckpt, dy

    sums = {k: np.zeros_like(gh[k], dtype=np.float64) for k in ("dA", "dD", "dbias")}
    allc = np.arange(D)
    for b in range(B):
        q = _rows(p, b, allc)
        r = oracle.selective_scan_bwd(q["u"], q["delta"], q["A"], q["Bm"], q["Cm"], p["dy"][b:b + 1], Dskip=q["Dskip"],
                                      delta_bias=q["delta_bias"], z=q["z"])
        yr, _ = oracle.selective_scan_fwd(q["u"], q["delta"], q["A"], q["Bm"], q["Cm"], Dskip=q["Dskip"],
                                          delta_bias=q["delta_bias"], z=q["z"])
        check_outputs({"y": (yh[b:b + 1], yr, TOL["bf16"]),
                       "du": (gh["du"][b:b + 1], r["du"], TOL["bf16"]),
                       "ddelta": (gh["ddelta"][b:b + 1], r["ddelta"], TOL["bf16"]),
                       "dz": (gh["dz"][b:b + 1], r["dz"], TOL["bf16"]),
                       "dBm": (gh["dBm"][b:b + 1], r["dBm"], 1e-4),
                       "dCm": (gh["dCm"][b:b + 1], r["dCm"], 1e-4)}, where=f"config 4 batch entry {b}")
        for k in sums:
            sums[k] += r[k]
    check_outputs({k: (gh[k], sums[k], 1e-4) for k in sums}, where="config 4 sums over the batch")

    # identities that hold at any size, kept as a second line of defence (fp64 sums on the device):
    #   <dBm, Bm> = <dCm, Cm> = <du, u> - sum_d Dskip[d] dD[d]
    f64 = torch.float64
    ib = float((g["dBm"].to(f64) * t["Bm"].to(f64)).sum())
    ic = float((g["dCm"].to(f64) * t["Cm"].to(f64)).sum())
    iu = float((g["du"].to(f64) * t["u"].to(f64)).sum()) - float((g["dD"].to(f64) * t["Dskip"].to(f64)).sum())
    scale = float((g["dBm"].to(f64).abs() * t["Bm"].to(f64).abs()).sum())
    assert abs(ib - ic) <= 1e-5 * scale, (ib, ic, scale)
    assert abs(ib - iu) <= 2e-3 * scale, (ib, iu, scale)       # du is rounded to bf16 element by element


def test_long_sequence_backward(api, oracle):
    """Backward over 256 tiles (L = 65536) for a handful of channels: adjoint and checkpoint carries across many tiles
    in one workgroup (single pass), and the same sequence cut into 64 chunks (the automatic choice for so few rows)."""
    p = workloads.make_selective(B=1, D=12, N=16, L=65536, io="bf16", gate=True, seed=33, bias=("uniform", -4.0, -2.0))
    t = _upload(p, "bf16")
    y, ckpt = api.lrnnx_selective_scan_fwd(**t, return_ckpt=True)
    r = oracle.selective_scan_bwd(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], p["dy"], Dskip=p["Dskip"],
                                  delta_bias=p["delta_bias"], z=p["z"])
    assert api.lib().lrnnx_selective_scan_bwd_chunks(1, 12, 16, 65536, 1, 0, 0) == 64
    for path in ("single_pass", "auto"):
        g = api.lrnnx_selective_scan_bwd(**t, dy=dev(p["dy"], "bf16"), ckpt=ckpt, want_dx0=True, path=path)
        errs = {k: rel_err(host(g[k]), r[k]) for k in ("du", "ddelta", "dz", "dA", "dBm", "dCm", "dD", "dbias", "dx0")}
        tol = {"du": 2e-2, "ddelta": 2e-2, "dz": 2e-2, "dA": 1e-4, "dBm": 1e-4, "dCm": 1e-4, "dD": 1e-4, "dbias": 1e-4,
               "dx0": 1e-4}
        bad = {k: v for k, v in errs.items() if not v <= tol[k]}
        assert not bad, f"{path}: {bad} (all {errs})"
