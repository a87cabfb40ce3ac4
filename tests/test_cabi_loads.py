"""CPU check: the built C-ABI library loads and exports every symbol include/lrnnx.h declares; host-only queries work."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2602_08810_amd", "liblrnnx.so")


def _declared():
    text = open(os.path.join(ROOT, "include", "lrnnx.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lrnnx_[a-z_0-9]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        pytest.skip("liblrnnx.so not built (run python -m paper_2602_08810_amd.build)")
    return ctypes.CDLL(LIB)


def test_every_declared_symbol_is_exported(lib):
    names = _declared()
    assert {"lrnnx_selective_scan_fwd", "lrnnx_selective_scan_bwd", "lrnnx_lti_diag_scan"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in lrnnx.h but not exported"


def test_host_queries(lib):
    lib.lrnnx_workspace_bytes.argtypes = [ctypes.c_int] + [ctypes.c_int64] * 4 + [ctypes.c_int] * 3
    lib.lrnnx_workspace_bytes.restype = ctypes.c_size_t
    lib.lrnnx_ckpt_interval.restype = ctypes.c_int64
    lib.lrnnx_status_string.restype = ctypes.c_char_p
    I = lib.lrnnx_ckpt_interval()
    assert I > 0
    # backward: the checkpoints of the recompute sweep (rounded up to 256 bytes), then the chunk aggregates
    ck = 2 * 3 * ((1000 + I - 1) // I) * 16 * 4
    carry = lib.lrnnx_workspace_bytes(7, 2, 3, 16, 1000, 1, 1, 0)
    assert carry > 0 and carry % (2 * 2 * 3 * 16 * 4) == 0            # two arrays [B,D,chunks,N] of floats
    assert lib.lrnnx_workspace_bytes(1, 2, 3, 16, 1000, 1, 1, 0) == (ck + 255) // 256 * 256 + carry
    assert lib.lrnnx_workspace_bytes(7, 1, 8, 16, 200, 1, 1, 0) == 0        # a single tile: nothing to cut
    chunks = lib.lrnnx_selective_scan_bwd_chunks
    chunks.argtypes = [ctypes.c_int64] * 4 + [ctypes.c_int] * 3
    assert chunks(16, 2560, 16, 4096, 1, 0, 0) == 1                   # enough rows to fill the chip: one pass
    assert chunks(16, 2560, 16, 4096, 1, 2, 0) == 2                   # ... unless the chunked path is asked for
    assert chunks(1, 2048, 16, 65536, 1, 0, 0) == 32 and chunks(1, 1024, 16, 32768, 1, 0, 0) == 32   # 512 workgroups each
    assert chunks(2, 768, 16, 8192, 1, 0, 0) == 8 and chunks(8, 1536, 16, 2048, 1, 0, 0) == 1
    assert chunks(1, 1024, 16, 32768, 1, 1, 0) == 1 and chunks(1, 8, 16, 200, 1, 2, 0) == 1
    assert chunks(1, 8, 3, 200, 1, 0, 0) == 0 and chunks(1, 9, 16, 200, 2, 0, 0) == 0
    assert chunks(1, 512, 16, 65536, 1, 0, 1) > 1 and chunks(8, 1536, 16, 2048, 1, 0, 1) == 1    # the complex-A scan
    assert chunks(1, 64, 32, 4096, 1, 0, 1) == 0                      # ... takes N <= 16
    assert lib.lrnnx_workspace_bytes(0, 1, 2048, 16, 65536, 1, 1, 0) > 0
    assert lib.lrnnx_workspace_bytes(0, 1, 8, 3, 64, 1, 1, 0) == 0          # unsupported N
    assert lib.lrnnx_workspace_bytes(2, 4, 256, 0, 4096, 0, 1, 0) > 0
    assert lib.lrnnx_workspace_bytes(3, 4, 256, 0, 4096, 0, 1, 0) > 0
    assert lib.lrnnx_workspace_bytes(4, 4, 256, 0, 4096, 2, 1, 0) > lib.lrnnx_workspace_bytes(4, 4, 256, 0, 4096, 0, 1, 0) > 0
    assert lib.lrnnx_workspace_bytes(4, 4, 256, 0, 4096, 1, 1, 0) == 0      # bf16 is not a dtype of the raw scan
    assert lib.lrnnx_workspace_bytes(5, 4, 256, 0, 4096, 2, 1, 0) > lib.lrnnx_workspace_bytes(5, 4, 256, 0, 4096, 0, 1, 0) > 0
    ckc = 2 * 3 * ((1000 + I - 1) // I) * 16 * 8                      # the complex backward: float pairs
    wsc = lib.lrnnx_workspace_bytes(6, 2, 3, 16, 1000, 1, 1, 0)
    assert wsc > (ckc + 255) // 256 * 256 and (wsc - (ckc + 255) // 256 * 256) % (2 * 2 * 3 * 16 * 8) == 0
    assert lib.lrnnx_workspace_bytes(8, 1, 64, 16, 8192, 1, 1, 0) > 0 and lib.lrnnx_workspace_bytes(8, 1, 64, 32, 8192, 1, 1, 0) == 0
    assert lib.lrnnx_status_string(0) == b"ok" and lib.lrnnx_status_string(3).startswith(b"workspace")
    assert lib.lrnnx_version() >= 300
    # grouped maps plan with (B * groups) row groups of D / groups channels: the aggregates of the chunked backward
    # are sized for that plan (a multiple of two arrays [B,D,chunks,N]), and D must be a multiple of the groups
    g4 = lib.lrnnx_workspace_bytes(7, 1, 512, 16, 16384, 1, 4, 0)
    assert g4 > 0 and g4 % (2 * 512 * 16 * 4) == 0 and lib.lrnnx_workspace_bytes(7, 1, 510, 16, 16384, 1, 4, 0) == 0
    # packed batches: checkpoints [D, L / interval + B, N] of the recompute sweep, then the larger of the B ints of
    # launch order and the chunk aggregates [B,D,chunks,N] x 2 as planned for sequences of L steps; the forward call
    # needs none (single pass only)
    slots = 1024 // I + 3
    nch = chunks(3, 8, 16, 1024, 1, 2, 0)
    assert nch > 1 and chunks(3, 8, 16, 1024, 1, 0, 0) <= nch
    assert lib.lrnnx_workspace_bytes(1, 3, 8, 16, 1024, 1, 1, 1) == (8 * slots * 16 * 4 + 255) // 256 * 256 + 2 * 3 * 8 * nch * 16 * 4
    assert lib.lrnnx_workspace_bytes(7, 3, 8, 16, 1024, 1, 1, 1) == 2 * 3 * 8 * nch * 16 * 4
    nchc = chunks(3, 8, 16, 1024, 1, 2, 1)
    assert lib.lrnnx_workspace_bytes(6, 3, 8, 16, 1024, 1, 1, 1) == (8 * slots * 16 * 8 + 255) // 256 * 256 + 2 * 3 * 8 * nchc * 16 * 8
    assert lib.lrnnx_workspace_bytes(7, 300, 8, 16, 256, 1, 1, 1) == 4 * 300     # one tile: no chunks, the launch order
    assert lib.lrnnx_workspace_bytes(0, 3, 8, 16, 1024, 1, 1, 1) == 0
    assert lib.lrnnx_static_scratch_bytes() == 4 << 20


def test_null_and_bad_struct_are_rejected_without_a_gpu(lib):
    """Argument errors are detected on the host before anything touches the device."""
    lib.lrnnx_selective_scan_fwd.argtypes = [ctypes.c_void_p]
    lib.lrnnx_selective_scan_bwd.argtypes = [ctypes.c_void_p]
    lib.lrnnx_lti_diag_scan.argtypes = [ctypes.c_void_p]
    assert lib.lrnnx_selective_scan_fwd(None) == 1
    assert lib.lrnnx_selective_scan_bwd(None) == 1
    assert lib.lrnnx_lti_diag_scan(None) == 1
    lib.lrnnx_lti_diag_scan_bwd.argtypes = [ctypes.c_void_p]
    assert lib.lrnnx_lti_diag_scan_bwd(None) == 1
    lib.lrnnx_selective_scan_fwd_complex.argtypes = [ctypes.c_void_p]
    assert lib.lrnnx_selective_scan_fwd_complex(None) == 1
    lib.lrnnx_selective_step_complex.argtypes = [ctypes.c_void_p]
    assert lib.lrnnx_selective_step_complex(None) == 1
    lib.lrnnx_selective_scan_bwd_complex.argtypes = [ctypes.c_void_p]
    assert lib.lrnnx_selective_scan_bwd_complex(None) == 1
    lib.lrnnx_diag_scan_bwd.argtypes = [ctypes.c_void_p]
    assert lib.lrnnx_diag_scan_bwd(None) == 1
    lib.lrnnx_diag_scan.argtypes = [ctypes.c_void_p]
    assert lib.lrnnx_diag_scan(None) == 1
    buf = (ctypes.c_char * 512)()                                       # struct_size = 0
    assert lib.lrnnx_selective_scan_fwd(ctypes.addressof(buf)) == 1
    assert lib.lrnnx_lti_diag_scan(ctypes.addressof(buf)) == 1
    lib.lrnnx_lti_diag_scan_static.argtypes = [ctypes.c_void_p]
    assert lib.lrnnx_lti_diag_scan_static(None) == 1 and lib.lrnnx_lti_diag_scan_static(ctypes.addressof(buf)) == 1


def test_bench_refuses_more_than_one_gpu():
    """bench.py is a one-GPU benchmark: --gpus 2 ends with a message and a non-zero status before touching a GPU."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stdout + r.stderr)


def test_binding_refuses_host_tensors():
    """The Python binding passes device pointers to the library; a CPU tensor is refused before any launch."""
    torch = pytest.importorskip("torch")
    from paper_2602_08810_amd import api
    u = torch.zeros(1, 2, 8)
    A = -torch.ones(2, 4)
    Bm = torch.zeros(1, 8, 4)
    with pytest.raises(TypeError, match="GPU tensors"):
        api.lrnnx_selective_scan_fwd(u, u, A, Bm, Bm)
    with pytest.raises(TypeError, match="GPU tensors"):
        api.lrnnx_selective_scan_bwd(u, u, A, Bm, Bm, dy=u)
    lam = torch.zeros(4, dtype=torch.complex64)
    v = torch.zeros(1, 8, 4, dtype=torch.complex64)
    with pytest.raises(TypeError, match="GPU tensors"):
        api.lrnnx_lti_diag_scan(lam, v)
    with pytest.raises(TypeError, match="GPU tensors"):
        api.lrnnx_selective_step(torch.zeros(1, 2, 4), u[:, :, 0], u[:, :, 0], A, Bm[:, 0], Bm[:, 0])


def _fwd_args(**over):
    """A syntactically valid forward argument block with fake (aligned, non-null, never dereferenced) pointers."""
    from paper_2602_08810_amd import api
    a = api.FwdArgs()
    a.struct_size = ctypes.sizeof(api.FwdArgs)
    a.B, a.D, a.N, a.L = 2, 8, 16, 100
    a.io_dtype, a.disc, a.delta_softplus, a.path = api.BF16, 0, 1, 0
    fake = 0x10000
    a.u = a.delta = a.A = a.Bm = a.Cm = a.y = fake
    a.u_stride_b = a.delta_stride_b = a.y_stride_b = 800
    a.u_stride_d = a.delta_stride_d = a.y_stride_d = 100
    for k, v in over.items():
        setattr(a, k, v)
    return a


def test_host_side_validation_of_the_forward_call(lib):
    """Every refusal below is decided on the host, before any HIP call: status codes as documented in lrnnx.h.
    The pointers are fake, so the test only runs where no GPU could ever be handed them."""
    torch = pytest.importorskip("torch")
    if torch.cuda.device_count() > 0:
        pytest.skip("host-only test: not run on a machine with a GPU")
    from paper_2602_08810_amd import api
    lib.lrnnx_selective_scan_fwd.argtypes = [ctypes.POINTER(api.FwdArgs)]
    call = lambda **over: lib.lrnnx_selective_scan_fwd(ctypes.byref(_fwd_args(**over)))
    assert call(B=65536) == 2                      # more batch entries than a launch grid holds: unsupported
    assert call(N=3) == 2 and call(N=64) == 2      # state sizes without a kernel
    assert call(L=0) == 1 and call(B=0) == 1 and call(D=0) == 1
    assert call(io_dtype=7) == 1 and call(disc=4) == 1 and call(path=9) == 1
    assert call(Bm=0x10004) == 1                   # maps must be 16-byte aligned
    assert call(u=0) == 1 and call(y=0) == 1       # required pointers
    assert call(u_stride_d=-1) == 1                # negative stride
    assert call(y_stride_d=50) == 1                # output rows would overlap
    assert call(bc_groups=3) == 1                  # D = 8 is not a multiple of 3 groups
    assert call(path=2) == 3                       # the chunk-carry path needs a workspace
    assert call(struct_size=ctypes.sizeof(api.FwdArgs) - 8) == 1 and call(struct_size=ctypes.sizeof(api.FwdArgs) + 8) == 1


def test_host_side_validation_of_the_backward_and_lti_calls(lib):
    """As above for lrnnx_selective_scan_bwd, lrnnx_lti_diag_scan and lrnnx_diag_scan (fake pointers, no GPU)."""
    torch = pytest.importorskip("torch")
    if torch.cuda.device_count() > 0:
        pytest.skip("host-only test: not run on a machine with a GPU")
    from paper_2602_08810_amd import api
    fake = 0x10000

    def bwd(**over):
        a = api.BwdArgs()
        a.struct_size = ctypes.sizeof(api.BwdArgs)
        a.B, a.D, a.N, a.L = 2, 8, 16, 100
        a.io_dtype, a.disc, a.delta_softplus = api.BF16, 0, 1
        for f in ("u", "delta", "A", "Bm", "Cm", "dy", "du", "ddelta", "dA", "dBm", "dCm", "ckpt"):
            setattr(a, f, fake)
        for f in ("u", "delta", "dy", "du", "ddelta"):
            setattr(a, f + "_stride_b", 800)
            setattr(a, f + "_stride_d", 100)
        for k, v in over.items():
            setattr(a, k, v)
        return lib.lrnnx_selective_scan_bwd(ctypes.byref(a))
    lib.lrnnx_selective_scan_bwd.argtypes = [ctypes.POINTER(api.BwdArgs)]
    assert bwd(ckpt=0) == 3                                   # no checkpoints and no workspace to recompute them into
    assert bwd(ckpt=0, workspace=fake, workspace_bytes=16) == 3
    assert bwd(dz=fake) == 1                                  # dz without z
    assert bwd(dD=fake) == 1 and bwd(dbias=fake) == 1         # dD without Dskip, dbias without delta_bias
    assert bwd(dBm=0x10008) == 1 and bwd(du=0) == 1 and bwd(dA=0) == 1
    assert bwd(du_stride_d=99) == 1 and bwd(dy_stride_b=-1) == 1
    assert bwd(N=5) == 2 and bwd(B=70000) == 2
    assert bwd(bc_groups=3) == 1 and bwd(bc_groups=-1) == 1
    assert bwd(path=9) == 1 and bwd(path=-1) == 1
    assert bwd(path=2, L=2000, du_stride_d=2000, ddelta_stride_d=2000) == 3   # the chunked path keeps its aggregates in the workspace
    # ... also for a packed batch (du, ddelta [D,L]), where max_seqlen is a hint that must not be negative
    assert bwd(path=2, cu_seqlens=fake, L=2000, du_stride_d=2000, ddelta_stride_d=2000) == 3
    assert bwd(cu_seqlens=fake, max_seqlen=-1) == 1

    def lti(**over):
        a = api.LtiArgs()
        a.struct_size = ctypes.sizeof(api.LtiArgs)
        a.B, a.P, a.L = 2, 64, 100
        a.lambda_ = a.v = a.x = fake
        for k, v in over.items():
            setattr(a, k, v)
        return lib.lrnnx_lti_diag_scan(ctypes.byref(a))
    lib.lrnnx_lti_diag_scan.argtypes = [ctypes.POINTER(api.LtiArgs)]
    assert lti(P=0) == 1 and lti(L=0) == 1 and lti(B=0) == 1
    assert lti(v=0x10004) == 1 and lti(x=0) == 1 and lti(path=7) == 1
    assert lti(B=70000) == 2
    assert lti() == 3                                         # every path of this call needs its workspace
    assert lti(chain_status=0x10002) == 1                     # a 4-byte word
    lib.lrnnx_lti_diag_scan_static.argtypes = [ctypes.POINTER(api.LtiArgs)]
    a = api.LtiArgs()
    a.struct_size = ctypes.sizeof(api.LtiArgs)
    a.B, a.P, a.L = 8, 1024, 8192
    a.lambda_ = a.v = a.x = fake
    assert lib.lrnnx_lti_diag_scan_static(ctypes.byref(a)) == 3   # needs more chain slots than the static array has
    a.path = 2
    assert lib.lrnnx_lti_diag_scan_static(ctypes.byref(a)) == 1   # the two-launch path is not offered there


def test_host_side_validation_of_the_complex_calls(lib):
    """As above for the complex-A forward and backward entry points (fake pointers, no GPU: only refusals are
    exercised)."""
    torch = pytest.importorskip("torch")
    if torch.cuda.device_count() > 0:
        pytest.skip("host-only test: not run on a machine with a GPU")
    from paper_2602_08810_amd import api
    fake = 0x10000

    def fwd(size=None, **over):
        a = api.FwdComplexArgs()
        a.struct_size = ctypes.sizeof(api.FwdComplexArgs) if size is None else size
        a.B, a.D, a.N, a.L = 2, 8, 16, 100
        a.io_dtype, a.disc, a.delta_softplus = api.BF16, 0, 1
        a.u = a.delta = a.A = a.Bm = a.Cm = a.y = fake
        a.u_stride_b = a.delta_stride_b = a.y_stride_b = 800
        a.u_stride_d = a.delta_stride_d = a.y_stride_d = 100
        for k, v in over.items():
            setattr(a, k, v)
        return lib.lrnnx_selective_scan_fwd_complex(ctypes.byref(a))
    lib.lrnnx_selective_scan_fwd_complex.argtypes = [ctypes.POINTER(api.FwdComplexArgs)]
    assert fwd(N=32) == 2 and fwd(N=3) == 2 and fwd(B=65536) == 2      # complex states: N <= 16
    assert fwd(L=0) == 1 and fwd(io_dtype=5) == 1 and fwd(disc=-1) == 1
    assert fwd(y=0) == 1                                               # nothing to compute: no y, ckpt or x_last
    assert fwd(A=0x10004) == 1 and fwd(x0=0x10004) == 1 and fwd(ckpt=0x10004) == 1 and fwd(Cm=0x10008) == 1
    assert fwd(bc_groups=3) == 1 and fwd(bc_groups=-2) == 1
    assert fwd(cu_seqlens=0x10004) == 1                                # boundaries are 8-byte integers
    assert fwd(path=5) == 1 and fwd(path=2, cu_seqlens=fake) == 2
    assert fwd(path=2, L=4000, y_stride_d=4000) == 3                   # the chunk-carry path needs its workspace
    assert fwd(path=2, L=4000, y_stride_d=4000, workspace=0x10004, workspace_bytes=1 << 30) == 1
    assert fwd(size=ctypes.sizeof(api.FwdComplexArgs) - 8) == 1        # any size but the struct's own is refused

    def bwd(size=None, **over):
        a = api.BwdComplexArgs()
        a.struct_size = ctypes.sizeof(api.BwdComplexArgs) if size is None else size
        a.B, a.D, a.N, a.L = 2, 8, 16, 100
        a.io_dtype, a.disc, a.delta_softplus = api.BF16, 0, 1
        for f in ("u", "delta", "A", "Bm", "Cm", "dy", "du", "ddelta", "dA", "dBm", "dCm", "ckpt"):
            setattr(a, f, fake)
        for f in ("u", "delta", "dy", "du", "ddelta"):
            setattr(a, f + "_stride_b", 800)
            setattr(a, f + "_stride_d", 100)
        for k, v in over.items():
            setattr(a, k, v)
        return lib.lrnnx_selective_scan_bwd_complex(ctypes.byref(a))
    lib.lrnnx_selective_scan_bwd_complex.argtypes = [ctypes.POINTER(api.BwdComplexArgs)]
    assert bwd(ckpt=0) == 3 and bwd(ckpt=0, workspace=fake, workspace_bytes=64) == 3
    assert bwd(N=32) == 2 and bwd(B=70000) == 2
    assert bwd(dz=fake) == 1 and bwd(dD=fake) == 1 and bwd(dbias=fake) == 1
    assert bwd(dA=0x10004) == 1 and bwd(dx0=0x10004) == 1 and bwd(dCm=0x10008) == 1
    assert bwd(cu_seqlens=0x10004) == 1 and bwd(bc_groups=5) == 1
    assert bwd(path=4) == 1 and bwd(cu_seqlens=fake, max_seqlen=-1) == 1
    assert bwd(path=2, cu_seqlens=fake, L=2000, du_stride_d=2000, ddelta_stride_d=2000) == 3
    assert bwd(path=2, L=2000, du_stride_d=2000, ddelta_stride_d=2000) == 3
    assert bwd(size=ctypes.sizeof(api.BwdComplexArgs) + 16) == 1
    # packed mode sizes the recompute workspace by D * (L / interval + B) * N float pairs
    need = 8 * (100 // int(lib.lrnnx_ckpt_interval()) + 2) * 16 * 8
    assert bwd(ckpt=0, cu_seqlens=fake, workspace=fake, workspace_bytes=need - 1) == 3
