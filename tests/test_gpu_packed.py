"""GPU parity of the selective scan on packed variable-length batches (cu_seqlens), forward and backward through the
C ABI, against the fp64 oracle (every sequence scanned on its own slice); same tolerances as the batched tests."""
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


def _check(api, oracle, D, N, lengths, io, seed, G=1, gap=0, with_ckpt=True, disc="zoh_s6", max_seqlen=None,
           path="auto", same_bits=True):
    import torch
    p = workloads.make_packed(D=D, N=N, lengths=lengths, io=io, seed=seed, bc_groups=G, gap=gap)
    cu = torch.from_numpy(p["cu_seqlens"]).cuda()
    t = dict(u=dev(p["u"], io), delta=dev(p["delta"], io), A=dev(p["A"]), Bm=dev(p["Bm"], io), Cm=dev(p["Cm"], io),
             Dskip=dev(p["Dskip"]), delta_bias=dev(p["delta_bias"]), z=dev(p["z"], io), x0=dev(p["x0"]))
    sentinel = 3.0
    y0 = torch.full_like(t["u"], sentinel)
    y, x_last, ckpt = api.lrnnx_selective_scan_fwd(**t, disc=disc, cu_seqlens=cu, return_last_state=True,
                                                   return_ckpt=True, out=y0)
    g = api.lrnnx_selective_scan_bwd(**t, dy=dev(p["dy"], io), disc=disc, cu_seqlens=cu, want_dx0=True,
                                     ckpt=ckpt if with_ckpt else None, max_seqlen=max_seqlen, path=path)
    if max_seqlen is not None and path == "auto" and same_bits:
        # the hint only moves channels between workgroups: what one channel computes on its own is bit for bit the same
        g0 = api.lrnnx_selective_scan_bwd(**t, dy=dev(p["dy"], io), disc=disc, cu_seqlens=cu, want_dx0=True, ckpt=ckpt)
        for k in ("du", "ddelta", "dz", "dx0"):
            assert torch.equal(g[k], g0[k]), k
    ref = {k: p[k] for k in ("u", "delta", "A", "Bm", "Cm", "Dskip", "delta_bias", "z", "x0")}
    yr, xr = oracle.selective_scan_fwd_packed(cu_seqlens=p["cu_seqlens"], disc=disc, **ref)
    r = oracle.selective_scan_bwd_packed(dy=p["dy"], cu_seqlens=p["cu_seqlens"], disc=disc, **ref)
    inside = np.zeros(p["u"].shape[1], bool)
    for o, e in zip(p["cu_seqlens"][:-1], p["cu_seqlens"][1:]):
        inside[o:e] = True
    yh = host(y)
    assert rel_err(yh[:, inside], yr[:, inside]) <= TOL[io]
    assert np.all(yh[:, ~inside] == sentinel), "steps outside every sequence must not be written"
    assert rel_err(host(x_last), xr) <= 1e-4
    tol = {"du": TOL[io], "ddelta": TOL[io], "dz": TOL[io], "dA": 1e-4, "dBm": 1e-4, "dCm": 1e-4, "dD": 1e-4,
           "dbias": 1e-4, "dx0": 1e-4}
    errs = {}
    for k in tol:
        got, want = host(g[k]), r[k]
        if k in ("du", "ddelta", "dz"):
            got, want = got[:, inside], want[:, inside]
        errs[k] = rel_err(got, want)
    bad = {k: v for k, v in errs.items() if not v <= tol[k]}
    assert not bad, f"{bad} (all {errs})"
    assert tuple(g["dBm"].shape) == p["Bm"].shape


@pytest.mark.parametrize("io", ["f32", "bf16"])
@pytest.mark.parametrize("lengths", [(700, 1, 256, 513, 2000), (8, 16, 24, 512), (300,), (1, 1, 1, 1, 5), (1030, 0, 77)])
def test_packed_lengths(api, oracle, lengths, io):
    """Ragged mixes: starts that are and are not 16-byte aligned, one-step and empty sequences, several tiles."""
    _check(api, oracle, 16, 16, lengths, io, seed=len(lengths))


@pytest.mark.parametrize("io", ["f32", "bf16"])
def test_packed_starts_at_every_residue_mod_8(api, oracle, io):
    """Sequence starts at 0, 513, 522, 532, 543, 555, 568, 582, 597: every residue mod 8, i.e. every misalignment of a
    row against the 16-byte vector accesses (which only need element alignment), with sequences of more than one
    vector and two of more than one tile."""
    lengths = (513, 9, 10, 11, 12, 13, 14, 15, 600)
    starts = np.concatenate([[0], np.cumsum(lengths)[:-1]])
    assert set(int(v) % 8 for v in starts) == set(range(8))
    _check(api, oracle, 12, 16, lengths, io, seed=31)


def test_packed_with_grouped_maps_and_unused_steps_around(api, oracle):
    _check(api, oracle, 24, 16, (333, 900, 40), "bf16", seed=7, G=3, gap=5)


def test_packed_small_state_and_ragged_channels(api, oracle):
    _check(api, oracle, 13, 4, (100, 600, 257), "f32", seed=8)


@pytest.mark.parametrize("disc", ["zoh", "bilinear", "dirac"])
def test_packed_other_discretisations(api, oracle, disc):
    _check(api, oracle, 8, 16, (129, 511, 64), "f32", seed=9, disc=disc)


def test_packed_backward_without_checkpoints(api, oracle):
    _check(api, oracle, 16, 16, (700, 300, 1500), "bf16", seed=10, with_ckpt=False)


@pytest.mark.parametrize("hint", [1500, 1000, 100, 10**9])
def test_packed_one_long_sequence_with_max_seqlen(api, oracle, hint):
    """One sequence of six tiles among 32 of one tile each, on enough channels that a workgroup takes 16 of them: with
    the longest length known (1500) the workgroups of the long sequence take 8 channels, those of the short ones 16,
    and the workgroups of the launch the short ones do not need leave at once.  A hint that is too small (1000: the
    long sequence still gets fewer channels than the others; 100: no effect) or far too large is as correct."""
    lengths = (20,) * 11 + (1500,) + (20,) * 21
    _check(api, oracle, 1024, 16, lengths, "bf16", seed=41, max_seqlen=hint)


def test_packed_one_long_sequence_with_max_seqlen_and_grouped_maps(api, oracle):
    """The same batch with four groups of maps (256 channels each): the channel blocks of a workgroup stay within one
    group whatever number of channels its sequence's length gives it."""
    lengths = (20,) * 11 + (1500,) + (20,) * 21
    _check(api, oracle, 1024, 16, lengths, "f32", seed=43, G=4, max_seqlen=1500)


@pytest.mark.parametrize("io", ["f32", "bf16"])
@pytest.mark.parametrize("hint", [None, 5000, 1000])
def test_packed_backward_in_chunks(api, oracle, hint, io):
    """The chunked backward on a packed batch: every sequence cut into chunks counted from its own start, planned for
    the longest length the caller names (5000), for the whole axis (no hint), or for a length that is too small (1000:
    the last chunk of the longer sequences then takes what is left).  Sequences of 10 and 700 steps end before most
    chunks start; 3000 and 5000 are not multiples of the chunk."""
    lengths = (3000, 700, 5000, 10)
    planned = min(hint or sum(lengths), sum(lengths))
    assert api.lib().lrnnx_selective_scan_bwd_chunks(len(lengths), 16, 16, planned, 1, 2, 0) > 1
    _check(api, oracle, 16, 16, lengths, io, seed=51, max_seqlen=hint, path="chunk_carry")


def test_packed_backward_in_chunks_variants(api, oracle):
    """Grouped maps with unused steps around the sequences, no checkpoints from the forward call, a small state, and
    the automatic choice (which cuts a packed batch into chunks only when it is told the longest length)."""
    _check(api, oracle, 24, 16, (2100, 900, 40), "bf16", seed=52, G=3, gap=5, path="chunk_carry")
    _check(api, oracle, 16, 16, (700, 300, 1500), "bf16", seed=53, with_ckpt=False, path="chunk_carry", max_seqlen=1500)
    _check(api, oracle, 13, 4, (100, 2600, 257), "f32", seed=54, path="chunk_carry")
    _check(api, oracle, 16, 16, (1030, 0, 77), "f32", seed=56, path="chunk_carry")      # an empty sequence: its dx0 is zero
    assert api.lib().lrnnx_selective_scan_bwd_chunks(2, 32, 16, 6000, 1, 0, 0) > 1
    _check(api, oracle, 32, 16, (6000, 5000), "bf16", seed=55, max_seqlen=6000, same_bits=False)


@pytest.mark.parametrize("lengths", [
    (3000, 1500, 1000, 2048, 512, 512, 700, 324, 100, 100, 60, 40, 2200, 1800, 32, 8, 448, 900, 300, 300, 200, 100, 100, 100),
    (2048,) * 8], ids=["24_mixed", "8x2048"])
def test_packed_batches_of_the_benchmark_at_full_size(api, oracle, lengths):
    """The two packed batches bench.py times (16384 steps on 1536 channels, N = 16, bf16; the backward call with
    max_seqlen), every output against the oracle.  The second is config 2 itself as a packed batch: its launch takes
    the shape of the batch [8,1536,2048]."""
    assert sum(lengths) == 16384
    _check(api, oracle, 1536, 16, lengths, "bf16", seed=71, max_seqlen=max(lengths))


def test_packed_backward_in_chunks_with_a_small_workspace(api, oracle):
    """A workspace with room for fewer chunks than planned: the call cuts the sequences into fewer, longer chunks
    (same results); with room for less than two chunks an explicit request is refused."""
    import torch
    lengths = (3000, 700, 5000, 10)
    B, D, N = len(lengths), 16, 16
    nch = api.lib().lrnnx_selective_scan_bwd_chunks(B, D, N, 5000, 1, 2, 0)
    assert nch >= 4
    per_chunk = 2 * B * D * N * 4
    p = workloads.make_packed(D=D, N=N, lengths=lengths, io="f32", seed=57)
    cu = torch.from_numpy(p["cu_seqlens"]).cuda()
    t = dict(u=dev(p["u"]), delta=dev(p["delta"]), A=dev(p["A"]), Bm=dev(p["Bm"]), Cm=dev(p["Cm"]),
             Dskip=dev(p["Dskip"]), delta_bias=dev(p["delta_bias"]), z=dev(p["z"]), x0=dev(p["x0"]))
    _, ckpt = api.lrnnx_selective_scan_fwd(**t, cu_seqlens=cu, return_ckpt=True)
    kw = dict(dy=dev(p["dy"]), cu_seqlens=cu, want_dx0=True, ckpt=ckpt, path="chunk_carry", max_seqlen=5000)
    full = api.lrnnx_selective_scan_bwd(**t, **kw)
    small = api.lrnnx_selective_scan_bwd(**t, **kw, workspace=torch.empty(per_chunk * 2 + 100, dtype=torch.uint8, device="cuda"))
    for k in ("du", "ddelta", "dz", "dA", "dBm", "dCm", "dD", "dbias", "dx0"):
        assert rel_err(host(small[k]), host(full[k])) <= 1e-5, k
    with pytest.raises(api.LrnnxError):
        api.lrnnx_selective_scan_bwd(**t, **kw, workspace=torch.empty(per_chunk + 100, dtype=torch.uint8, device="cuda"))


def test_packed_max_seqlen_is_validated(api):
    p = workloads.make_packed(D=8, N=16, lengths=(100, 200), io="f32", seed=11)
    import torch
    t = dict(u=dev(p["u"]), delta=dev(p["delta"]), A=dev(p["A"]), Bm=dev(p["Bm"]), Cm=dev(p["Cm"]))
    cu = torch.from_numpy(p["cu_seqlens"]).cuda()
    with pytest.raises(api.LrnnxError):
        api.lrnnx_selective_scan_bwd(**t, dy=dev(p["dy"]), cu_seqlens=cu, max_seqlen=-1)
    # without cu_seqlens the hint is ignored
    b = workloads.make_selective(B=2, D=8, N=16, L=300, io="f32", seed=12)
    tb = dict(u=dev(b["u"]), delta=dev(b["delta"]), A=dev(b["A"]), Bm=dev(b["Bm"]), Cm=dev(b["Cm"]))
    g0 = api.lrnnx_selective_scan_bwd(**tb, dy=dev(b["dy"]))
    g1 = api.lrnnx_selective_scan_bwd(**tb, dy=dev(b["dy"]), max_seqlen=5)
    assert torch.equal(g0["du"], g1["du"]) and torch.equal(g0["ddelta"], g1["ddelta"])


def test_packed_boundaries_are_clamped_and_chunk_carry_is_refused(api):
    """Boundaries beyond the packed axis are clamped on the device (no fault, finite results)."""
    import torch
    p = workloads.make_packed(D=8, N=16, lengths=(100, 200), io="f32", seed=11)
    t = dict(u=dev(p["u"]), delta=dev(p["delta"]), A=dev(p["A"]), Bm=dev(p["Bm"]), Cm=dev(p["Cm"]))
    cu = torch.tensor([-5, 100, 10_000], dtype=torch.int64, device="cuda")
    y = api.lrnnx_selective_scan_fwd(**t, cu_seqlens=cu)
    good = api.lrnnx_selective_scan_fwd(**t, cu_seqlens=torch.tensor([0, 100, 300], dtype=torch.int64, device="cuda"))
    assert torch.equal(y, good)
    with pytest.raises(api.LrnnxError):
        api.lrnnx_selective_scan_fwd(**t, cu_seqlens=cu, path="chunk_carry")
