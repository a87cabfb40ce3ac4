"""GPU parity of the complex-A selective scan on packed variable-length batches (cu_seqlens), forward and backward
through the C ABI, against the fp64 oracle (every sequence scanned on its own slice); same tolerances as the
batched complex tests."""
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


def _cplx(a):
    return a[..., 0].astype(np.float64) + 1j * a[..., 1].astype(np.float64)


def _maps_dev(a, io):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t.to(torch.bfloat16) if io == "bf16" else torch.view_as_complex(t)


def _crel(got, ref):
    den = np.abs(ref).max()
    return float(np.abs(np.asarray(got, dtype=np.complex128) - ref).max() / (den if den > 0 else 1.0))


def _check(api, oracle, D, N, lengths, io, seed, G=1, gap=0, with_ckpt=True, disc="zoh_s6", max_seqlen=None,
           path="auto"):
    import torch
    p = workloads.make_packed_complex(D=D, N=N, lengths=lengths, io=io, seed=seed, bc_groups=G, gap=gap)
    cu = torch.from_numpy(p["cu_seqlens"]).cuda()
    t = dict(u=dev(p["u"], io), delta=dev(p["delta"], io), A=torch.from_numpy(p["A"]).cuda(), Bm=_maps_dev(p["Bm"], io),
             Cm=_maps_dev(p["Cm"], io), Dskip=dev(p["Dskip"]), delta_bias=dev(p["delta_bias"]), z=dev(p["z"], io),
             x0=torch.from_numpy(p["x0"]).cuda())
    sentinel = 3.0
    y0 = torch.full_like(t["u"], sentinel)
    y, x_last, ckpt = api.lrnnx_selective_scan_fwd_complex(**t, disc=disc, cu_seqlens=cu, return_last_state=True,
                                                           return_ckpt=True, out=y0)
    g = api.lrnnx_selective_scan_bwd_complex(**t, dy=dev(p["dy"], io), disc=disc, cu_seqlens=cu, want_dx0=True,
                                             ckpt=ckpt if with_ckpt else None, max_seqlen=max_seqlen, path=path)
    if max_seqlen is not None and path == "auto":
        # the hint only moves channels between workgroups: what one channel computes on its own is bit for bit the same
        g0 = api.lrnnx_selective_scan_bwd_complex(**t, dy=dev(p["dy"], io), disc=disc, cu_seqlens=cu, want_dx0=True,
                                                  ckpt=ckpt)
        for k in ("du", "ddelta", "dz"):
            assert torch.equal(g[k], g0[k]), k
    torch.cuda.synchronize()
    ref = dict(u=p["u"], delta=p["delta"], A=p["A"], Bm=_cplx(p["Bm"]), Cm=_cplx(p["Cm"]), Dskip=p["Dskip"],
               delta_bias=p["delta_bias"], z=p["z"], x0=p["x0"])
    yr, xr = oracle.selective_scan_fwd_complex_packed(cu_seqlens=p["cu_seqlens"], disc=disc, **ref)
    r = oracle.selective_scan_bwd_complex_packed(dy=p["dy"], cu_seqlens=p["cu_seqlens"], disc=disc, **ref)
    inside = np.zeros(p["u"].shape[1], bool)
    for o, e in zip(p["cu_seqlens"][:-1], p["cu_seqlens"][1:]):
        inside[o:e] = True
    yh = host(y)
    assert rel_err(yh[:, inside], yr[:, inside]) <= TOL[io]
    assert np.all(yh[:, ~inside] == sentinel), "steps outside every sequence must not be written"
    assert _crel(x_last.cpu().numpy(), xr) <= 1e-4
    errs = {}
    for k in ("du", "ddelta", "dz"):
        errs[k] = (rel_err(host(g[k])[:, inside], r[k][:, inside]), TOL[io])
    for k in ("dD", "dbias"):
        errs[k] = (rel_err(host(g[k]), r[k]), 1e-4)
    for k in ("dA", "dBm", "dCm", "dx0"):
        errs[k] = (_crel(g[k].cpu().numpy(), r[k]), 1e-4)
    bad = {k: v for k, v in errs.items() if not v[0] <= v[1]}
    assert not bad, f"rel errors over tolerance: {bad}  (all: {errs})"
    assert tuple(g["dBm"].shape) == p["Bm"].shape[:-1]


@pytest.mark.parametrize("io", ["f32", "bf16"])
@pytest.mark.parametrize("lengths", [(700, 1, 256, 513, 2000), (8, 16, 24, 512), (300,), (1, 1, 1, 1, 5), (1030, 0, 77)])
def test_packed_complex_lengths(api, oracle, lengths, io):
    """Ragged mixes: starts that are and are not 16-byte aligned, one-step and empty sequences, several tiles."""
    _check(api, oracle, 16, 16, lengths, io, seed=len(lengths))


def test_packed_complex_with_grouped_maps_and_unused_steps_around(api, oracle):
    _check(api, oracle, 24, 8, (333, 900, 40), "bf16", seed=7, G=3, gap=5)


def test_packed_complex_small_state_and_ragged_channels(api, oracle):
    _check(api, oracle, 13, 4, (100, 600, 257), "f32", seed=8)
    _check(api, oracle, 5, 1, (100, 300, 257), "bf16", seed=12)


@pytest.mark.parametrize("disc", ["zoh", "bilinear", "dirac"])
def test_packed_complex_other_discretisations(api, oracle, disc):
    _check(api, oracle, 8, 16, (129, 511, 64), "f32", seed=9, disc=disc)


def test_packed_complex_backward_without_checkpoints(api, oracle):
    _check(api, oracle, 16, 16, (700, 300, 1500), "bf16", seed=10, with_ckpt=False)


@pytest.mark.parametrize("hint", [1500, 10**9])
def test_packed_complex_one_long_sequence_with_max_seqlen(api, oracle, hint):
    """One sequence of six tiles among 32 of one tile each: with the longest length known its workgroups take 8
    channels and those of the short sequences 24, instead of 33 each."""
    lengths = (20,) * 11 + (1500,) + (20,) * 21
    _check(api, oracle, 256, 16, lengths, "bf16", seed=42, max_seqlen=hint)


@pytest.mark.parametrize("hint", [None, 5000, 1000])
def test_packed_complex_backward_in_chunks(api, oracle, hint):
    """The chunked backward on a packed batch, chunks planned for the longest length the caller names, for the whole
    axis, or for a length that is too small (the last chunk of a longer sequence takes what is left)."""
    lengths = (3000, 700, 5000, 10)
    planned = min(hint or sum(lengths), sum(lengths))
    assert api.lib().lrnnx_selective_scan_bwd_chunks(len(lengths), 16, 16, planned, 1, 2, 1) > 1
    _check(api, oracle, 16, 16, lengths, "bf16", seed=61, max_seqlen=hint, path="chunk_carry")


def test_packed_complex_backward_in_chunks_variants(api, oracle):
    _check(api, oracle, 24, 8, (2100, 900, 40), "f32", seed=62, G=3, gap=5, path="chunk_carry")
    _check(api, oracle, 16, 16, (700, 300, 1500), "bf16", seed=63, with_ckpt=False, path="chunk_carry", max_seqlen=1500)
    _check(api, oracle, 16, 16, (1030, 0, 77), "f32", seed=64, path="chunk_carry")      # an empty sequence: its dx0 is zero


def test_packed_complex_boundaries_are_clamped(api):
    """Boundaries beyond the packed axis are clamped on the device (no fault, same results as the clamped list)."""
    import torch
    p = workloads.make_packed_complex(D=8, N=16, lengths=(100, 200), io="f32", seed=11)
    t = dict(u=dev(p["u"]), delta=dev(p["delta"]), A=torch.from_numpy(p["A"]).cuda(), Bm=_maps_dev(p["Bm"], "f32"),
             Cm=_maps_dev(p["Cm"], "f32"))
    i64 = dict(dtype=torch.int64, device="cuda")
    y = api.lrnnx_selective_scan_fwd_complex(**t, cu_seqlens=torch.tensor([-5, 100, 10_000], **i64))
    good = api.lrnnx_selective_scan_fwd_complex(**t, cu_seqlens=torch.tensor([0, 100, 300], **i64))
    assert torch.equal(y, good)
    dy = dev(p["dy"])
    g = api.lrnnx_selective_scan_bwd_complex(**t, dy=dy, cu_seqlens=torch.tensor([-5, 100, 10_000], **i64))
    gg = api.lrnnx_selective_scan_bwd_complex(**t, dy=dy, cu_seqlens=torch.tensor([0, 100, 300], **i64))
    assert torch.equal(g["du"], gg["du"]) and torch.equal(g["ddelta"], gg["ddelta"])
