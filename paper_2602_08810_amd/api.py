"""Thin ctypes binding of liblrnnx.so: argument marshalling only.

Every function here has the name of the C entry point it calls (include/lrnnx.h) and
does nothing but check tensor dtypes/devices, allocate the outputs and the workspace
with torch, fill the args struct with data pointers, strides and the current HIP
stream, and call into the library.  There is no CPU or PyTorch fallback: if the
library has not been built, importing the entry points raises.
"""
from __future__ import annotations

import ctypes
import functools
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblrnnx.so")

F32, BF16, C64 = 0, 1, 2
DISC = {"zoh_s6": 0, "zoh": 1, "bilinear": 2, "dirac": 3}
PATH = {"auto": 0, "single_pass": 1, "chunk_carry": 2}
WS_FWD, WS_BWD, WS_LTI, WS_LTI_BWD, WS_DIAG, WS_DIAG_BWD, WS_BWD_COMPLEX, WS_BWD_CARRY, WS_FWD_COMPLEX = 0, 1, 2, 3, 4, 5, 6, 7, 8
STATUS = {0: "ok", 1: "invalid argument", 2: "unsupported", 3: "workspace", 4: "launch"}

_vp, _i32, _i64, _sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t


_SEL_HEAD = [("struct_size", _sz), ("B", _i32), ("D", _i32), ("N", _i32), ("bc_groups", _i32), ("L", _i64),
             ("io_dtype", _i32), ("disc", _i32), ("delta_softplus", _i32), ("path", _i32), ("cu_seqlens", _vp)]
_SEL_INPUTS = [("u", _vp), ("u_stride_b", _i64), ("u_stride_d", _i64),
               ("delta", _vp), ("delta_stride_b", _i64), ("delta_stride_d", _i64),
               ("A", _vp), ("Bm", _vp), ("Cm", _vp), ("Dskip", _vp), ("delta_bias", _vp),
               ("z", _vp), ("z_stride_b", _i64), ("z_stride_d", _i64),
               ("x0", _vp)]
_SEL_FWD_TAIL = [("y", _vp), ("y_stride_b", _i64), ("y_stride_d", _i64), ("x_last", _vp), ("ckpt", _vp),
                 ("workspace", _vp), ("workspace_bytes", _sz), ("stream", _vp)]
_SEL_BWD_TAIL = [("dy", _vp), ("dy_stride_b", _i64), ("dy_stride_d", _i64), ("ckpt", _vp),
                 ("du", _vp), ("du_stride_b", _i64), ("du_stride_d", _i64),
                 ("ddelta", _vp), ("ddelta_stride_b", _i64), ("ddelta_stride_d", _i64),
                 ("dz", _vp), ("dz_stride_b", _i64), ("dz_stride_d", _i64),
                 ("dA", _vp), ("dBm", _vp), ("dCm", _vp), ("dD", _vp), ("dbias", _vp), ("dx0", _vp),
                 ("workspace", _vp), ("workspace_bytes", _sz), ("stream", _vp)]


class FwdArgs(ctypes.Structure):                  # lrnnx_ss_fwd_args
    _fields_ = _SEL_HEAD + _SEL_INPUTS + _SEL_FWD_TAIL


class FwdComplexArgs(ctypes.Structure):           # lrnnx_ss_fwd_complex_args (same layout, complex pointers)
    _fields_ = _SEL_HEAD + _SEL_INPUTS + _SEL_FWD_TAIL


class BwdArgs(ctypes.Structure):                  # lrnnx_ss_bwd_args
    _fields_ = _SEL_HEAD + [("max_seqlen", _i64)] + _SEL_INPUTS + _SEL_BWD_TAIL


class BwdComplexArgs(ctypes.Structure):           # lrnnx_ss_bwd_complex_args
    _fields_ = _SEL_HEAD + [("max_seqlen", _i64)] + _SEL_INPUTS + _SEL_BWD_TAIL


class LtiArgs(ctypes.Structure):
    _fields_ = [
        ("struct_size", _sz), ("B", _i32), ("P", _i32), ("L", _i64), ("path", _i32), ("reserved", _i32),
        ("lambda_", _vp), ("v", _vp), ("x0", _vp), ("x", _vp), ("x_last", _vp), ("chain_status", _vp),
        ("workspace", _vp), ("workspace_bytes", _sz), ("stream", _vp),
    ]


class LtiBwdArgs(ctypes.Structure):
    _fields_ = [
        ("struct_size", _sz), ("B", _i32), ("P", _i32), ("L", _i64),
        ("lambda_", _vp), ("x", _vp), ("x0", _vp), ("gx", _vp), ("dv", _vp), ("dlambda", _vp), ("dx0", _vp),
        ("chain_status", _vp), ("workspace", _vp), ("workspace_bytes", _sz), ("stream", _vp),
    ]


class DiagScanArgs(ctypes.Structure):
    _fields_ = [
        ("struct_size", _sz), ("B", _i32), ("P", _i32), ("L", _i64), ("dtype", _i32), ("reserved", _i32),
        ("a", _vp), ("b", _vp), ("x0", _vp), ("x", _vp), ("x_last", _vp), ("chain_status", _vp),
        ("workspace", _vp), ("workspace_bytes", _sz), ("stream", _vp),
    ]


class DiagScanBwdArgs(ctypes.Structure):
    _fields_ = [
        ("struct_size", _sz), ("B", _i32), ("P", _i32), ("L", _i64), ("dtype", _i32), ("reserved", _i32),
        ("a", _vp), ("x", _vp), ("x0", _vp), ("gx", _vp), ("da", _vp), ("db", _vp), ("dx0", _vp),
        ("chain_status", _vp), ("workspace", _vp), ("workspace_bytes", _sz), ("stream", _vp),
    ]


_STEP_FIELDS = [
    ("struct_size", _sz), ("B", _i32), ("D", _i32), ("N", _i32), ("bc_groups", _i32),
    ("io_dtype", _i32), ("disc", _i32), ("delta_softplus", _i32), ("reserved", _i32),
    ("x", _vp),
    ("u", _vp), ("u_stride_b", _i64), ("u_stride_d", _i64),
    ("delta", _vp), ("delta_stride_b", _i64), ("delta_stride_d", _i64),
    ("A", _vp), ("Bm", _vp), ("Cm", _vp), ("Dskip", _vp), ("delta_bias", _vp),
    ("z", _vp), ("z_stride_b", _i64), ("z_stride_d", _i64),
    ("y", _vp), ("y_stride_b", _i64), ("y_stride_d", _i64),
    ("stream", _vp),
]


class StepArgs(ctypes.Structure):                 # lrnnx_ss_step_args
    _fields_ = _STEP_FIELDS


class StepComplexArgs(ctypes.Structure):          # lrnnx_ss_step_complex_args
    _fields_ = _STEP_FIELDS


class LtiStepArgs(ctypes.Structure):
    _fields_ = [("struct_size", _sz), ("B", _i32), ("P", _i32), ("lambda_", _vp), ("x", _vp), ("v", _vp), ("stream", _vp)]


_lib = None


def lib():
    """The loaded C library.  Raises if it was not built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2602_08810_amd.build` "
                               "(the scan has no CPU or PyTorch fallback)")
        L = ctypes.CDLL(LIB_PATH)
        L.lrnnx_selective_scan_fwd.argtypes = [ctypes.POINTER(FwdArgs)]
        L.lrnnx_selective_scan_bwd.argtypes = [ctypes.POINTER(BwdArgs)]
        L.lrnnx_selective_scan_fwd_complex.argtypes = [ctypes.POINTER(FwdComplexArgs)]
        L.lrnnx_selective_scan_fwd_complex.restype = ctypes.c_int
        L.lrnnx_selective_scan_bwd_complex.argtypes = [ctypes.POINTER(BwdComplexArgs)]
        L.lrnnx_selective_scan_bwd_complex.restype = ctypes.c_int
        L.lrnnx_lti_diag_scan.argtypes = [ctypes.POINTER(LtiArgs)]
        L.lrnnx_lti_diag_scan_static.argtypes = [ctypes.POINTER(LtiArgs)]
        L.lrnnx_lti_diag_scan_static.restype = ctypes.c_int
        L.lrnnx_static_scratch_bytes.restype = _sz
        L.lrnnx_lti_diag_scan_bwd.argtypes = [ctypes.POINTER(LtiBwdArgs)]
        L.lrnnx_lti_diag_scan_bwd.restype = ctypes.c_int
        L.lrnnx_diag_scan.argtypes = [ctypes.POINTER(DiagScanArgs)]
        L.lrnnx_diag_scan.restype = ctypes.c_int
        L.lrnnx_diag_scan_bwd.argtypes = [ctypes.POINTER(DiagScanBwdArgs)]
        L.lrnnx_diag_scan_bwd.restype = ctypes.c_int
        L.lrnnx_selective_step.argtypes = [ctypes.POINTER(StepArgs)]
        L.lrnnx_selective_step_complex.argtypes = [ctypes.POINTER(StepComplexArgs)]
        L.lrnnx_selective_step_complex.restype = ctypes.c_int
        L.lrnnx_lti_step.argtypes = [ctypes.POINTER(LtiStepArgs)]
        L.lrnnx_selective_step.restype = ctypes.c_int
        L.lrnnx_lti_step.restype = ctypes.c_int
        for f in (L.lrnnx_selective_scan_fwd, L.lrnnx_selective_scan_bwd, L.lrnnx_lti_diag_scan, L.lrnnx_version):
            f.restype = ctypes.c_int
        L.lrnnx_workspace_bytes.argtypes = [ctypes.c_int, _i64, _i64, _i64, _i64, ctypes.c_int, ctypes.c_int, ctypes.c_int]
        L.lrnnx_workspace_bytes.restype = _sz
        L.lrnnx_selective_scan_bwd_chunks.argtypes = [_i64, _i64, _i64, _i64, ctypes.c_int, ctypes.c_int, ctypes.c_int]
        L.lrnnx_selective_scan_bwd_chunks.restype = ctypes.c_int
        L.lrnnx_selective_scan_fwd_complex_chunks.argtypes = [_i64, _i64, _i64, _i64, ctypes.c_int, ctypes.c_int]
        L.lrnnx_selective_scan_fwd_complex_chunks.restype = ctypes.c_int
        L.lrnnx_ckpt_interval.restype = _i64
        L.lrnnx_status_string.argtypes = [ctypes.c_int]
        L.lrnnx_status_string.restype = ctypes.c_char_p
        _lib = L
    return _lib


class LrnnxError(RuntimeError):
    def __init__(self, code):
        self.code = code
        super().__init__(f"lrnnx status {code}: {lib().lrnnx_status_string(code).decode()}")


def _check(code):
    if code != 0:
        raise LrnnxError(code)


def _ptr(t):
    return None if t is None else t.data_ptr()


def _io_dtype(t):
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"I/O dtype must be float32 or bfloat16, got {t.dtype}")


def _bdl(t, name, io=None, shape=None, out=False):
    """(ptr, stride_b, stride_d) of a [B,D,L] tensor whose last axis is contiguous.  `shape`: the (B, D, L) every
    per-channel tensor of the call must have (the kernels index all of them with the same b, d, l; only a stride of
    0 may broadcast an input).  `out`: an output, whose rows must not overlap."""
    if t is None:
        return None, 0, 0
    if t.dim() != 3 or (t.shape[2] > 1 and t.stride(2) != 1):
        raise ValueError(f"{name}: expected [B,D,L] with contiguous time axis")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: expected shape {tuple(shape)}, got {tuple(t.shape)}")
    if out:
        # rows (b, d) of L elements at b * stride_b + d * stride_d: the axis with the smaller stride must step over a
        # whole row, the other one over all rows of the first (either axis may be the inner one)
        axes = sorted((t.stride(i), t.shape[i]) for i in (0, 1) if t.shape[i] > 1)
        need = t.shape[2]
        for stride, count in axes:
            if stride < need:
                raise ValueError(f"{name}: output rows overlap")
            need = stride * count
    if io is not None and t.dtype != io:
        raise TypeError(f"{name}: dtype {t.dtype} differs from the I/O dtype {io}")
    return t.data_ptr(), t.stride(0), t.stride(1)


def _f32c(t, name, shape=None):
    if t is None:
        return None
    if t.dtype != torch.float32 or not t.is_contiguous():
        raise TypeError(f"{name}: expected a contiguous float32 tensor")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: expected shape {tuple(shape)}, got {tuple(t.shape)}")
    return t


def _status_word(t):
    """Device pointer of an optional int32 status word (a one-element tensor the caller has cleared)."""
    if t is None:
        return None
    if t.dtype != torch.int32 or t.numel() != 1 or not t.is_cuda:
        raise ValueError("chain_status: expected a one-element int32 device tensor")
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _device_checked(fn):
    """Every tensor argument of a compute entry point must live on ONE GPU: the library takes device pointers and
    has no CPU path, so a host tensor is refused here, before anything is launched.  (Kept cheap: the single-token
    step is called once per generated token.)"""
    name = fn.__name__
    Tensor = torch.Tensor

    def bad(v, dev):
        if not v.is_cuda:
            return TypeError(f"{name}: a tensor argument is on {v.device}; the scan library needs GPU tensors")
        return TypeError(f"{name}: tensors on different devices (cuda:{dev} and {v.device})")

    @functools.wraps(fn)
    def wrapper(*args, **kwargs):
        dev = -1
        for v in args + tuple(kwargs.values()):
            if isinstance(v, Tensor):
                d = v.get_device()                    # -1 for a host tensor
                if d < 0 or (dev >= 0 and d != dev):
                    raise bad(v, dev)
                dev = d
            elif isinstance(v, dict):
                for t in v.values():
                    if isinstance(t, Tensor):
                        d = t.get_device()
                        if d < 0 or (dev >= 0 and d != dev):
                            raise bad(t, dev)
                        dev = d
        return fn(*args, **kwargs)
    return wrapper


def lrnnx_ckpt_interval() -> int:
    return int(lib().lrnnx_ckpt_interval())


def lrnnx_workspace_bytes(which, B, D, N, L, io_dtype, bc_groups=1, packed=False) -> int:
    return int(lib().lrnnx_workspace_bytes(which, B, D, N, L, io_dtype, bc_groups, int(bool(packed))))


def _check_cu(cu):
    """Number of sequences of a packed batch; cu is int64 [S+1] on the device."""
    if cu.dtype != torch.int64 or cu.dim() != 1 or not cu.is_contiguous() or not cu.is_cuda or cu.numel() < 2:
        raise ValueError("cu_seqlens: expected a contiguous int64 device tensor [S+1]")
    return cu.numel() - 1


def _bc_groups(Bm, Cm, io, Bsz, D, L, N):
    """Number of groups of the maps: [B,L,N] -> 1, [B,G,L,N] -> G (channel d reads group d // (D/G))."""
    for name, t in (("Bm", Bm), ("Cm", Cm)):
        ok = t.dtype == io and t.is_contiguous() and t.shape == Bm.shape and (
            tuple(t.shape) == (Bsz, L, N) or (t.dim() == 4 and t.shape[0] == Bsz and tuple(t.shape[2:]) == (L, N)))
        if not ok:
            raise ValueError(f"{name}: expected contiguous [B,L,N] or [B,G,L,N] of dtype {io}")
    G = Bm.shape[1] if Bm.dim() == 4 else 1
    if D % G:
        raise ValueError("D must be a multiple of the number of Bm/Cm groups")
    return G


@_device_checked
def lrnnx_selective_scan_fwd(u, delta, A, Bm, Cm, Dskip=None, delta_bias=None, z=None, x0=None,
                             disc="zoh_s6", delta_softplus=True, path="auto",
                             return_last_state=False, return_ckpt=False, out=None, ckpt_out=None, workspace=None,
                             cu_seqlens=None):
    """y (and optionally x_last, ckpt) of the forward selective scan; see lrnnx_ss_fwd_args.

    `out`, `ckpt_out` and `workspace` may supply preallocated buffers (ckpt_out implies return_ckpt).
    With `cu_seqlens` (int64 [S+1] on the device) the call is in packed variable-length mode: u, delta, z, y are
    [D,L], Bm and Cm [L,N] or [G,L,N], x0 and x_last [S,D,N]."""
    io = u.dtype
    packed = cu_seqlens is not None
    if packed:
        Bsz = _check_cu(cu_seqlens)
        u, delta, z, out = (None if t is None else t.unsqueeze(0) for t in (u, delta, z, out))
        Bm, Cm = Bm.unsqueeze(0), Cm.unsqueeze(0)
    Bio = 1 if packed else u.shape[0]                   # leading dimension of the I/O tensors and of the maps
    if not packed:
        Bsz = Bio
    _, D, L = u.shape
    N = A.shape[1]
    a = FwdArgs()
    a.struct_size = ctypes.sizeof(FwdArgs)
    a.B, a.D, a.N, a.L = Bsz, D, N, L
    a.cu_seqlens = _ptr(cu_seqlens)
    a.io_dtype = _io_dtype(u)
    a.disc = DISC[disc] if isinstance(disc, str) else int(disc)
    a.delta_softplus = int(bool(delta_softplus))
    a.path = PATH[path] if isinstance(path, str) else int(path)
    bdl = (Bio, D, L)
    a.u, a.u_stride_b, a.u_stride_d = _bdl(u, "u", io, bdl)
    a.delta, a.delta_stride_b, a.delta_stride_d = _bdl(delta, "delta", io, bdl)
    a.z, a.z_stride_b, a.z_stride_d = _bdl(z, "z", io, bdl)
    a.A = _ptr(_f32c(A, "A", (D, N)))
    a.bc_groups = _bc_groups(Bm, Cm, io, Bio, D, L, N)
    a.Bm, a.Cm = Bm.data_ptr(), Cm.data_ptr()
    a.Dskip = _ptr(_f32c(Dskip, "Dskip", (D,)))
    a.delta_bias = _ptr(_f32c(delta_bias, "delta_bias", (D,)))
    a.x0 = _ptr(_f32c(x0, "x0", (Bsz, D, N)))
    y = out if out is not None else torch.empty((Bio, D, L), dtype=io, device=u.device)
    a.y, a.y_stride_b, a.y_stride_d = _bdl(y, "y", io, bdl, out=True)
    x_last = torch.empty((Bsz, D, N), dtype=torch.float32, device=u.device) if return_last_state else None
    a.x_last = _ptr(x_last)
    ckpt = ckpt_out
    return_ckpt = return_ckpt or ckpt_out is not None
    if return_ckpt:
        I = lrnnx_ckpt_interval()
        ck_shape = (D, L // I + Bsz, N) if packed else (Bsz, D, (L + I - 1) // I, N)
        if ckpt is None:
            ckpt = torch.empty(ck_shape, dtype=torch.float32, device=u.device)
        _f32c(ckpt, "ckpt_out", ck_shape)
    a.ckpt = _ptr(ckpt)
    if workspace is None:
        nbytes = lrnnx_workspace_bytes(WS_FWD, Bsz, D, N, L, a.io_dtype, a.bc_groups, packed)
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=u.device) if nbytes else None
    if workspace is not None:
        a.workspace, a.workspace_bytes = workspace.data_ptr(), workspace.numel()
    a.stream = _stream()
    _check(lib().lrnnx_selective_scan_fwd(ctypes.byref(a)))
    res = (y[0] if packed else y,)
    if return_last_state:
        res += (x_last,)
    if return_ckpt:
        res += (ckpt,)
    return res[0] if len(res) == 1 else res


@_device_checked
def lrnnx_selective_scan_fwd_complex(u, delta, A, Bm, Cm, Dskip=None, delta_bias=None, z=None, x0=None,
                                     disc="zoh_s6", delta_softplus=True, return_last_state=False, out=None,
                                     return_ckpt=False, ckpt_out=None, cu_seqlens=None, path="auto", workspace=None):
    """y (and optionally x_last, ckpt) of the forward selective scan with complex A, Bm, Cm; see
    lrnnx_ss_fwd_complex_args.  `ckpt_out`: a preallocated checkpoint array to fill (implies return_ckpt).

    A [D,N] complex64.  Bm, Cm [B,L,N]: complex64 for float32 I/O; for bfloat16 I/O a bfloat16 tensor [B,L,N,2]
    of (re, im) pairs.  x0, x_last [B,D,N] complex64; ckpt [B,D,ceil(L/interval),N] complex64.
    With `cu_seqlens` (int64 [S+1] on the device) the call is in packed variable-length mode: u, delta, z, y are
    [D,L], Bm and Cm [L,N] or [G,L,N] (plus the pair axis for bfloat16), x0 and x_last [S,D,N], ckpt
    [D, L // interval + S, N].  `path`: "auto", "single_pass" or "chunk_carry" (few rows, long sequences); `workspace`
    may supply the scratch buffer of the latter."""
    io = u.dtype
    packed = cu_seqlens is not None
    if packed:
        Bsz = _check_cu(cu_seqlens)
        u, delta, z, out = (None if t is None else t.unsqueeze(0) for t in (u, delta, z, out))
        Bm, Cm = Bm.unsqueeze(0), Cm.unsqueeze(0)
    Bio = 1 if packed else u.shape[0]                   # leading dimension of the I/O tensors and of the maps
    if not packed:
        Bsz = Bio
    _, D, L = u.shape
    N, G = _check_complex_maps(A, Bm, Cm, io, Bio, D, L)
    a = FwdComplexArgs()
    a.struct_size = ctypes.sizeof(FwdComplexArgs)
    a.B, a.D, a.N, a.L = Bsz, D, N, L
    a.bc_groups = G
    a.cu_seqlens = _ptr(cu_seqlens)
    a.io_dtype = _io_dtype(u)
    a.disc = DISC[disc] if isinstance(disc, str) else int(disc)
    a.delta_softplus = int(bool(delta_softplus))
    bdl = (Bio, D, L)
    a.u, a.u_stride_b, a.u_stride_d = _bdl(u, "u", io, bdl)
    a.delta, a.delta_stride_b, a.delta_stride_d = _bdl(delta, "delta", io, bdl)
    a.z, a.z_stride_b, a.z_stride_d = _bdl(z, "z", io, bdl)
    a.A, a.Bm, a.Cm = A.data_ptr(), Bm.data_ptr(), Cm.data_ptr()
    a.Dskip = _ptr(_f32c(Dskip, "Dskip", (D,)))
    a.delta_bias = _ptr(_f32c(delta_bias, "delta_bias", (D,)))
    if x0 is not None:
        if x0.dtype != torch.complex64 or not x0.is_contiguous() or tuple(x0.shape) != (Bsz, D, N):
            raise ValueError("x0: expected contiguous complex64 [B,D,N]")
        a.x0 = x0.data_ptr()
    y = out if out is not None else torch.empty((Bio, D, L), dtype=io, device=u.device)
    a.y, a.y_stride_b, a.y_stride_d = _bdl(y, "y", io, bdl, out=True)
    x_last = torch.empty((Bsz, D, N), dtype=torch.complex64, device=u.device) if return_last_state else None
    a.x_last = _ptr(x_last)
    ckpt = None
    if return_ckpt or ckpt_out is not None:
        I = lrnnx_ckpt_interval()
        shape = (D, L // I + Bsz, N) if packed else (Bsz, D, -(-L // I), N)
        ckpt = ckpt_out if ckpt_out is not None else torch.empty(shape, dtype=torch.complex64, device=u.device)
        if ckpt.dtype != torch.complex64 or not ckpt.is_contiguous() or tuple(ckpt.shape) != shape:
            raise ValueError(f"ckpt_out: expected contiguous complex64 {shape}")
        a.ckpt = ckpt.data_ptr()
        return_ckpt = True
    a.path = PATH[path] if isinstance(path, str) else int(path)
    if workspace is None:
        nbytes = lrnnx_workspace_bytes(WS_FWD_COMPLEX, Bsz, D, N, L, a.io_dtype, G, packed)
        if nbytes:
            workspace = torch.empty(nbytes, dtype=torch.uint8, device=u.device)
    if workspace is not None:
        a.workspace, a.workspace_bytes = workspace.data_ptr(), workspace.numel()
    a.stream = _stream()
    _check(lib().lrnnx_selective_scan_fwd_complex(ctypes.byref(a)))
    res = (y[0] if packed else y,) + ((x_last,) if return_last_state else ()) + ((ckpt,) if return_ckpt else ())
    return res if len(res) > 1 else y


def _check_complex_maps(A, Bm, Cm, io, Bsz, D, L):
    """Validate A [D,N] complex64 and the complex maps for this I/O type ([B,L,N], or [B,G,L,N] with G groups; the
    bfloat16 form has a trailing axis of (re, im) pairs); returns (N, G)."""
    if A.dtype != torch.complex64 or A.dim() != 2 or A.shape[0] != D or not A.is_contiguous():
        raise ValueError("A: expected contiguous complex64 [D,N]")
    N = A.shape[1]
    G = None
    for name, t in (("Bm", Bm), ("Cm", Cm)):
        shape = tuple(t.shape)
        if io == torch.bfloat16:
            ok = t.dtype == torch.bfloat16 and shape[-1:] == (2,)
            shape = shape[:-1]
        else:
            ok = io == torch.float32 and t.dtype == torch.complex64
        ok = ok and t.is_contiguous() and (shape == (Bsz, L, N) or (len(shape) == 4 and shape[0] == Bsz and shape[2:] == (L, N)))
        g = shape[1] if ok and len(shape) == 4 else 1
        if not ok or (G is not None and g != G):
            raise ValueError(f"{name}: expected contiguous complex64 [B,L,N] or [B,G,L,N] (float32 I/O), or bfloat16 "
                             "with a trailing (re, im) axis")
        G = g
    if D % G:
        raise ValueError("D must be a multiple of the number of Bm/Cm groups")
    return N, G


@_device_checked
def lrnnx_selective_scan_bwd_complex(u, delta, A, Bm, Cm, dy, Dskip=None, delta_bias=None, z=None, x0=None,
                                     ckpt=None, disc="zoh_s6", delta_softplus=True, want_dx0=False, outs=None,
                                     workspace=None, cu_seqlens=None, path="auto", max_seqlen=None):
    """Gradients of sum(dy*y) of the complex-A selective scan as a dict; see lrnnx_ss_bwd_complex_args.
    dA [D,N], dBm, dCm [B,L,N], dx0 [B,D,N] are complex64 (dLoss/dRe + i dLoss/dIm); du, ddelta, dz in the I/O
    type; dD, dbias float32.  `ckpt`: the checkpoints a forward call returned (else they are recomputed).
    `cu_seqlens`: packed variable-length mode as in the forward call (du, ddelta, dz are [D,L]; dBm, dCm [L,N] or
    [G,L,N]; dx0 [S,D,N]).  `path`: "auto", "single_pass" or "chunk_carry" as for the real scan.  `max_seqlen`: as
    for the real scan."""
    io = u.dtype
    packed = cu_seqlens is not None
    if packed:
        Bsz = _check_cu(cu_seqlens)
        u, delta, z, dy = (None if t is None else t.unsqueeze(0) for t in (u, delta, z, dy))
        Bm, Cm = Bm.unsqueeze(0), Cm.unsqueeze(0)
    Bio = 1 if packed else u.shape[0]
    if not packed:
        Bsz = Bio
    _, D, L = u.shape
    N, G = _check_complex_maps(A, Bm, Cm, io, Bio, D, L)
    dev = u.device
    outs = dict(outs or {})
    if packed:                                          # caller-supplied outputs are in the packed shapes
        outs = {k: (v.unsqueeze(0) if k in ("du", "ddelta", "dz", "dBm", "dCm") else v) for k, v in outs.items()}

    def new(name, shape, dtype):
        if name not in outs:
            outs[name] = torch.empty(shape, dtype=dtype, device=dev)
        t = outs[name]
        strided_ok = name in ("du", "ddelta", "dz")          # [B,D,L] outputs are passed with their strides
        if t.dtype != dtype or tuple(t.shape) != tuple(shape) or not (strided_ok or t.is_contiguous()):
            raise ValueError(f"{name}: expected {dtype} {tuple(shape)}" + ("" if strided_ok else ", contiguous"))
        return t

    a = BwdComplexArgs()
    a.struct_size = ctypes.sizeof(BwdComplexArgs)
    a.B, a.D, a.N, a.L = Bsz, D, N, L
    a.bc_groups = G
    a.cu_seqlens = _ptr(cu_seqlens)
    a.max_seqlen = 0 if max_seqlen is None else int(max_seqlen)
    a.path = PATH[path] if isinstance(path, str) else int(path)
    a.io_dtype = _io_dtype(u)
    a.disc = DISC[disc] if isinstance(disc, str) else int(disc)
    a.delta_softplus = int(bool(delta_softplus))
    bdl = (Bio, D, L)
    a.u, a.u_stride_b, a.u_stride_d = _bdl(u, "u", io, bdl)
    a.delta, a.delta_stride_b, a.delta_stride_d = _bdl(delta, "delta", io, bdl)
    a.z, a.z_stride_b, a.z_stride_d = _bdl(z, "z", io, bdl)
    a.dy, a.dy_stride_b, a.dy_stride_d = _bdl(dy, "dy", io, bdl)
    a.A, a.Bm, a.Cm = A.data_ptr(), Bm.data_ptr(), Cm.data_ptr()
    a.Dskip = _ptr(_f32c(Dskip, "Dskip", (D,)))
    a.delta_bias = _ptr(_f32c(delta_bias, "delta_bias", (D,)))
    I = lrnnx_ckpt_interval()
    ck_shape = (D, L // I + Bsz, N) if packed else (Bsz, D, -(-L // I), N)
    for name, t, shape in (("x0", x0, (Bsz, D, N)), ("ckpt", ckpt, ck_shape)):
        if t is not None:
            if t.dtype != torch.complex64 or not t.is_contiguous() or tuple(t.shape) != shape:
                raise ValueError(f"{name}: expected contiguous complex64 {shape}")
            setattr(a, name, t.data_ptr())
    a.du, a.du_stride_b, a.du_stride_d = _bdl(new("du", bdl, io), "du", io, bdl, out=True)
    a.ddelta, a.ddelta_stride_b, a.ddelta_stride_d = _bdl(new("ddelta", bdl, io), "ddelta", io, bdl, out=True)
    if z is not None:
        a.dz, a.dz_stride_b, a.dz_stride_d = _bdl(new("dz", bdl, io), "dz", io, bdl, out=True)
    c64 = torch.complex64
    a.dA = new("dA", (D, N), c64).data_ptr()
    map_shape = (Bio, L, N) if (Bm.dim() == 3 + (io == torch.bfloat16)) else (Bio, G, L, N)
    a.dBm = new("dBm", map_shape, c64).data_ptr()
    a.dCm = new("dCm", map_shape, c64).data_ptr()
    if Dskip is not None:
        a.dD = new("dD", (D,), torch.float32).data_ptr()
    if delta_bias is not None:
        a.dbias = new("dbias", (D,), torch.float32).data_ptr()
    if want_dx0:
        a.dx0 = new("dx0", (Bsz, D, N), c64).data_ptr()
    if workspace is None:
        # with the forward's checkpoints only the chunk aggregates (or the launch order of a packed batch) are needed
        nbytes = lrnnx_workspace_bytes(WS_BWD_COMPLEX, Bsz, D, N, L, a.io_dtype, G, packed)
        if ckpt is not None:
            nbytes -= (ckpt.numel() * 8 + 255) // 256 * 256
        if nbytes:
            workspace = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    if workspace is not None:
        a.workspace, a.workspace_bytes = workspace.data_ptr(), workspace.numel()
    a.stream = _stream()
    _check(lib().lrnnx_selective_scan_bwd_complex(ctypes.byref(a)))
    if packed:
        outs = {k: (v[0] if k in ("du", "ddelta", "dz", "dBm", "dCm") else v) for k, v in outs.items()}
    return outs


@_device_checked
def lrnnx_selective_scan_bwd(u, delta, A, Bm, Cm, dy, Dskip=None, delta_bias=None, z=None, x0=None,
                             ckpt=None, disc="zoh_s6", delta_softplus=True, want_dx0=False,
                             outs=None, workspace=None, cu_seqlens=None, path="auto", max_seqlen=None):
    """Gradients of sum(dy*y) as a dict; see lrnnx_ss_bwd_args.  `outs` may supply preallocated outputs.
    `cu_seqlens`: packed variable-length mode as in the forward call (du, ddelta, dz are [D,L]; dBm, dCm as Bm).
    `path`: "auto", "single_pass" or "chunk_carry" (time axis cut into chunks that run side by side).
    `max_seqlen`: packed mode, the longest sequence of the batch if the host knows it (a hint for the launch shape
    that keeps one long sequence from setting the time of the whole launch, and lets "auto" cut a few long sequences
    into chunks; the lengths themselves stay on the device)."""
    io = u.dtype
    packed = cu_seqlens is not None
    if packed:
        Bsz = _check_cu(cu_seqlens)
        u, delta, z, dy = (None if t is None else t.unsqueeze(0) for t in (u, delta, z, dy))
        Bm, Cm = Bm.unsqueeze(0), Cm.unsqueeze(0)
    Bio = 1 if packed else u.shape[0]
    if not packed:
        Bsz = Bio
    _, D, L = u.shape
    N = A.shape[1]
    dev = u.device
    outs = dict(outs or {})
    if packed:                                          # caller-supplied outputs are in the packed shapes
        outs = {k: (v.unsqueeze(0) if k in ("du", "ddelta", "dz", "dBm", "dCm") else v) for k, v in outs.items()}

    def new(name, shape, dtype):
        if name not in outs:
            outs[name] = torch.empty(shape, dtype=dtype, device=dev)
        t = outs[name]
        strided_ok = name in ("du", "ddelta", "dz")          # [B,D,L] outputs are passed with their strides
        if t.dtype != dtype or tuple(t.shape) != tuple(shape) or not (strided_ok or t.is_contiguous()):
            raise ValueError(f"{name}: expected {dtype} {tuple(shape)}" + ("" if strided_ok else ", contiguous"))
        return t

    a = BwdArgs()
    a.struct_size = ctypes.sizeof(BwdArgs)
    a.B, a.D, a.N, a.L = Bsz, D, N, L
    a.cu_seqlens = _ptr(cu_seqlens)
    a.max_seqlen = 0 if max_seqlen is None else int(max_seqlen)
    a.path = PATH[path] if isinstance(path, str) else int(path)
    a.io_dtype = _io_dtype(u)
    a.disc = DISC[disc] if isinstance(disc, str) else int(disc)
    a.delta_softplus = int(bool(delta_softplus))
    bdl = (Bio, D, L)
    a.u, a.u_stride_b, a.u_stride_d = _bdl(u, "u", io, bdl)
    a.delta, a.delta_stride_b, a.delta_stride_d = _bdl(delta, "delta", io, bdl)
    a.z, a.z_stride_b, a.z_stride_d = _bdl(z, "z", io, bdl)
    a.dy, a.dy_stride_b, a.dy_stride_d = _bdl(dy, "dy", io, bdl)
    a.A = _ptr(_f32c(A, "A", (D, N)))
    a.bc_groups = _bc_groups(Bm, Cm, io, Bio, D, L, N)
    a.Bm, a.Cm = Bm.data_ptr(), Cm.data_ptr()
    a.Dskip = _ptr(_f32c(Dskip, "Dskip", (D,)))
    a.delta_bias = _ptr(_f32c(delta_bias, "delta_bias", (D,)))
    a.x0 = _ptr(_f32c(x0, "x0", (Bsz, D, N)))
    I = lrnnx_ckpt_interval()
    a.ckpt = _ptr(_f32c(ckpt, "ckpt", (D, L // I + Bsz, N) if packed else (Bsz, D, -(-L // I), N)))
    a.du, a.du_stride_b, a.du_stride_d = _bdl(new("du", bdl, io), "du", io, bdl, out=True)
    a.ddelta, a.ddelta_stride_b, a.ddelta_stride_d = _bdl(new("ddelta", bdl, io), "ddelta", io, bdl, out=True)
    if z is not None:
        a.dz, a.dz_stride_b, a.dz_stride_d = _bdl(new("dz", bdl, io), "dz", io, bdl, out=True)
    a.dA = new("dA", (D, N), torch.float32).data_ptr()
    a.dBm = new("dBm", tuple(Bm.shape), torch.float32).data_ptr()
    a.dCm = new("dCm", tuple(Cm.shape), torch.float32).data_ptr()
    if Dskip is not None:
        a.dD = new("dD", (D,), torch.float32).data_ptr()
    if delta_bias is not None:
        a.dbias = new("dbias", (D,), torch.float32).data_ptr()
    if want_dx0:
        a.dx0 = new("dx0", (Bsz, D, N), torch.float32).data_ptr()
    if workspace is None:
        kind = WS_BWD if ckpt is None else WS_BWD_CARRY
        nbytes = lrnnx_workspace_bytes(kind, Bsz, D, N, L, a.io_dtype, a.bc_groups, packed)
        if nbytes:
            workspace = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    if workspace is not None:
        a.workspace, a.workspace_bytes = workspace.data_ptr(), workspace.numel()
    a.stream = _stream()
    _check(lib().lrnnx_selective_scan_bwd(ctypes.byref(a)))
    if packed:
        outs = {k: (v[0] if k in ("du", "ddelta", "dz", "dBm", "dCm") else v) for k, v in outs.items()}
    return outs


@_device_checked
def lrnnx_lti_diag_scan(lam, v, x0=None, return_last_state=False, out=None, workspace=None, path="auto",
                        chain_status=None):
    """x [B,L,P] complex64 of x_k = lam * x_{k-1} + v_k; see lrnnx_lti_args.  `chain_status`: an int32 device word the
    library sets to 1 should a bounded wait between workgroups ever run out (clear it first)."""
    if v.dtype != torch.complex64 or lam.dtype != torch.complex64:
        raise TypeError("lam and v must be complex64")
    if not v.is_contiguous() or not lam.is_contiguous():
        raise ValueError("lam and v must be contiguous")
    Bsz, L, P = v.shape
    if tuple(lam.shape) != (P,):
        raise ValueError(f"lam: expected shape ({P},), got {tuple(lam.shape)}")
    if out is not None and (out.dtype != torch.complex64 or not out.is_contiguous() or out.shape != v.shape):
        raise ValueError("out: expected a contiguous complex64 tensor of the shape of v")
    a = LtiArgs()
    a.struct_size = ctypes.sizeof(LtiArgs)
    a.B, a.P, a.L = Bsz, P, L
    a.path = PATH[path] if isinstance(path, str) else int(path)
    a.lambda_, a.v = lam.data_ptr(), v.data_ptr()
    if x0 is not None:
        if x0.dtype != torch.complex64 or not x0.is_contiguous() or tuple(x0.shape) != (Bsz, P):
            raise ValueError("x0: expected contiguous complex64 [B,P]")
        a.x0 = x0.data_ptr()
    x = out if out is not None else torch.empty_like(v)
    a.x = x.data_ptr()
    x_last = torch.empty((Bsz, P), dtype=torch.complex64, device=v.device) if return_last_state else None
    a.x_last = _ptr(x_last)
    a.chain_status = _status_word(chain_status)
    if workspace is None:
        nbytes = lrnnx_workspace_bytes(WS_LTI, Bsz, P, 0, L, 0)
        workspace = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=v.device)
    a.workspace, a.workspace_bytes = workspace.data_ptr(), workspace.numel()
    a.stream = _stream()
    _check(lib().lrnnx_lti_diag_scan(ctypes.byref(a)))
    return (x, x_last) if return_last_state else x


@_device_checked
def lrnnx_lti_diag_scan_static(lam, v, out, x0=None, x_last_out=None):
    """The LTI scan on the library's own static scratch array: no workspace is passed and the C call allocates
    nothing; see lrnnx_lti_diag_scan_static.  The caller supplies every buffer: `out` [B,L,P] complex64 (may be v
    itself) and optionally `x_last_out` [B,P].  Returns `out`."""
    for name, t in (("lam", lam), ("v", v), ("out", out)):
        if t.dtype != torch.complex64 or not t.is_contiguous():
            raise ValueError(f"{name}: expected contiguous complex64")
    Bsz, L, P = v.shape
    if tuple(out.shape) != (Bsz, L, P) or tuple(lam.shape) != (P,):
        raise ValueError("shape mismatch between lam [P], v and out [B,L,P]")
    a = LtiArgs()
    a.struct_size = ctypes.sizeof(LtiArgs)
    a.B, a.P, a.L = Bsz, P, L
    a.path = PATH["auto"]
    a.lambda_, a.v, a.x = lam.data_ptr(), v.data_ptr(), out.data_ptr()
    for name, t in (("x0", x0), ("x_last_out", x_last_out)):
        if t is not None and (t.dtype != torch.complex64 or not t.is_contiguous() or tuple(t.shape) != (Bsz, P)):
            raise ValueError(f"{name}: expected contiguous complex64 [B,P]")
    a.x0, a.x_last = _ptr(x0), _ptr(x_last_out)
    a.stream = _stream()
    _check(lib().lrnnx_lti_diag_scan_static(ctypes.byref(a)))
    return out


@_device_checked
def lrnnx_lti_diag_scan_bwd(lam, x, gx, x0=None, want_dx0=True, out=None, workspace=None, chain_status=None):
    """(dv [B,L,P], dlam [P], dx0 [B,P] or None) from the saved states x and the incoming gradient gx;
    see lrnnx_lti_bwd_args."""
    for t, name in ((lam, "lam"), (x, "x"), (gx, "gx")):
        if t.dtype != torch.complex64 or not t.is_contiguous():
            raise ValueError(f"{name}: expected contiguous complex64")
    Bsz, L, P = x.shape
    if tuple(gx.shape) != (Bsz, L, P) or tuple(lam.shape) != (P,):
        raise ValueError("shape mismatch between lam [P], x and gx [B,L,P]")
    a = LtiBwdArgs()
    a.struct_size = ctypes.sizeof(LtiBwdArgs)
    a.B, a.P, a.L = Bsz, P, L
    a.lambda_, a.x, a.gx = lam.data_ptr(), x.data_ptr(), gx.data_ptr()
    if x0 is not None:
        if x0.dtype != torch.complex64 or not x0.is_contiguous() or tuple(x0.shape) != (Bsz, P):
            raise ValueError("x0: expected contiguous complex64 [B,P]")
        a.x0 = x0.data_ptr()
    if out is not None and (out.dtype != torch.complex64 or not out.is_contiguous() or out.shape != gx.shape):
        raise ValueError("out: expected a contiguous complex64 tensor of the shape of gx")
    dv = out if out is not None else torch.empty_like(gx)
    dlam = torch.empty(P, dtype=torch.complex64, device=x.device)
    dx0 = torch.empty((Bsz, P), dtype=torch.complex64, device=x.device) if want_dx0 else None
    a.dv, a.dlambda, a.dx0 = dv.data_ptr(), dlam.data_ptr(), _ptr(dx0)
    a.chain_status = _status_word(chain_status)
    if workspace is None:
        nbytes = lrnnx_workspace_bytes(WS_LTI_BWD, Bsz, P, 0, L, 0)
        workspace = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=x.device)
    a.workspace, a.workspace_bytes = workspace.data_ptr(), workspace.numel()
    a.stream = _stream()
    _check(lib().lrnnx_lti_diag_scan_bwd(ctypes.byref(a)))
    return dv, dlam, dx0


@_device_checked
def lrnnx_diag_scan(a, b, x0=None, return_last_state=False, out=None, workspace=None, chain_status=None):
    """x [B,L,P] of x_k = a_k * x_{k-1} + b_k for float32 or complex64 a, b; see lrnnx_diag_scan_args."""
    if a.dtype not in (torch.float32, torch.complex64) or b.dtype != a.dtype:
        raise TypeError("a and b must both be float32 or both complex64")
    if not a.is_contiguous() or not b.is_contiguous() or a.shape != b.shape or b.dim() != 3:
        raise ValueError("a and b must be contiguous [B,L,P] tensors of one shape")
    Bsz, L, P = b.shape
    dt = C64 if a.dtype == torch.complex64 else F32
    g = DiagScanArgs()
    g.struct_size = ctypes.sizeof(DiagScanArgs)
    g.B, g.P, g.L, g.dtype = Bsz, P, L, dt
    g.a, g.b = a.data_ptr(), b.data_ptr()
    if x0 is not None:
        if x0.dtype != a.dtype or not x0.is_contiguous() or tuple(x0.shape) != (Bsz, P):
            raise ValueError("x0: expected a contiguous [B,P] tensor of the dtype of a")
        g.x0 = x0.data_ptr()
    if out is not None and (out.dtype != b.dtype or not out.is_contiguous() or out.shape != b.shape):
        raise ValueError("out: expected a contiguous tensor of the dtype and shape of b")
    x = out if out is not None else torch.empty_like(b)
    g.x = x.data_ptr()
    x_last = torch.empty((Bsz, P), dtype=a.dtype, device=b.device) if return_last_state else None
    g.x_last = _ptr(x_last)
    g.chain_status = _status_word(chain_status)
    if workspace is None:
        nbytes = lrnnx_workspace_bytes(WS_DIAG, Bsz, P, 0, L, dt)
        workspace = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=b.device)
    g.workspace, g.workspace_bytes = workspace.data_ptr(), workspace.numel()
    g.stream = _stream()
    _check(lib().lrnnx_diag_scan(ctypes.byref(g)))
    return (x, x_last) if return_last_state else x


@_device_checked
def lrnnx_diag_scan_bwd(a, x, gx, x0=None, want_dx0=True, workspace=None, chain_status=None):
    """(da, db [B,L,P], dx0 [B,P] or None) from the forward call's a, saved states x and the incoming gradient gx;
    see lrnnx_diag_scan_bwd_args."""
    for t, name in ((a, "a"), (x, "x"), (gx, "gx")):
        if t.dtype != a.dtype or not t.is_contiguous() or t.shape != a.shape:
            raise ValueError(f"{name}: expected a contiguous tensor of the dtype and shape of a")
    if a.dtype not in (torch.float32, torch.complex64) or a.dim() != 3:
        raise TypeError("a must be a float32 or complex64 [B,L,P] tensor")
    Bsz, L, P = a.shape
    dt = C64 if a.dtype == torch.complex64 else F32
    g = DiagScanBwdArgs()
    g.struct_size = ctypes.sizeof(DiagScanBwdArgs)
    g.B, g.P, g.L, g.dtype = Bsz, P, L, dt
    g.a, g.x, g.gx = a.data_ptr(), x.data_ptr(), gx.data_ptr()
    if x0 is not None:
        if x0.dtype != a.dtype or not x0.is_contiguous() or tuple(x0.shape) != (Bsz, P):
            raise ValueError("x0: expected a contiguous [B,P] tensor of the dtype of a")
        g.x0 = x0.data_ptr()
    da, db = torch.empty_like(a), torch.empty_like(a)
    dx0 = torch.empty((Bsz, P), dtype=a.dtype, device=a.device) if want_dx0 else None
    g.da, g.db, g.dx0 = da.data_ptr(), db.data_ptr(), _ptr(dx0)
    g.chain_status = _status_word(chain_status)
    if workspace is None:
        nbytes = lrnnx_workspace_bytes(WS_DIAG_BWD, Bsz, P, 0, L, dt)
        workspace = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=a.device)
    g.workspace, g.workspace_bytes = workspace.data_ptr(), workspace.numel()
    g.stream = _stream()
    _check(lib().lrnnx_diag_scan_bwd(ctypes.byref(g)))
    return da, db, dx0


def _bd(t, name, io):
    """(ptr, stride_b, stride_d) of a [B,D] tensor (any strides)."""
    if t is None:
        return None, 0, 0
    if t.dim() != 2 or t.dtype != io:
        raise ValueError(f"{name}: expected a [B,D] tensor of dtype {io}")
    return t.data_ptr(), t.stride(0), t.stride(1)


@_device_checked
def lrnnx_selective_step(x, u, delta, A, Bm, Cm, Dskip=None, delta_bias=None, z=None,
                         disc="zoh_s6", delta_softplus=True, out=None):
    """One token: updates the state x [B,D,N] in place and returns y [B,D]; see lrnnx_ss_step_args."""
    io = u.dtype
    Bsz, D, N = x.shape
    _f32c(x, "x", (Bsz, D, N))
    a = StepArgs()
    a.struct_size = ctypes.sizeof(StepArgs)
    a.B, a.D, a.N = Bsz, D, N
    a.io_dtype = _io_dtype(u)
    a.disc = DISC[disc] if isinstance(disc, str) else int(disc)
    a.delta_softplus = int(bool(delta_softplus))
    a.x = x.data_ptr()
    a.u, a.u_stride_b, a.u_stride_d = _bd(u, "u", io)
    a.delta, a.delta_stride_b, a.delta_stride_d = _bd(delta, "delta", io)
    a.z, a.z_stride_b, a.z_stride_d = _bd(z, "z", io)
    a.A = _ptr(_f32c(A, "A", (D, N)))
    for name, t in (("Bm", Bm), ("Cm", Cm)):
        ok = t.dtype == io and t.is_contiguous() and t.shape == Bm.shape and (
            tuple(t.shape) == (Bsz, N) or (t.dim() == 3 and t.shape[0] == Bsz and t.shape[2] == N))
        if not ok:
            raise ValueError(f"{name}: expected contiguous [B,N] or [B,G,N] of dtype {io}")
    a.bc_groups = Bm.shape[1] if Bm.dim() == 3 else 1
    if D % a.bc_groups:
        raise ValueError("D must be a multiple of the number of Bm/Cm groups")
    a.Bm, a.Cm = Bm.data_ptr(), Cm.data_ptr()
    a.Dskip = _ptr(_f32c(Dskip, "Dskip", (D,)))
    a.delta_bias = _ptr(_f32c(delta_bias, "delta_bias", (D,)))
    y = out if out is not None else torch.empty((Bsz, D), dtype=io, device=u.device)
    a.y, a.y_stride_b, a.y_stride_d = _bd(y, "y", io)
    a.stream = _stream()
    _check(lib().lrnnx_selective_step(ctypes.byref(a)))
    return y


@_device_checked
def lrnnx_selective_step_complex(x, u, delta, A, Bm, Cm, Dskip=None, delta_bias=None, z=None,
                                 disc="zoh_s6", delta_softplus=True, out=None):
    """One token of the complex-A scan: updates the state x [B,D,N] complex64 in place and returns y [B,D]; see
    lrnnx_ss_step_complex_args.  Bm, Cm [B,N]: complex64 (float32 I/O) or bfloat16 [B,N,2] (re, im) pairs."""
    io = u.dtype
    if x.dtype != torch.complex64 or x.dim() != 3 or not x.is_contiguous():
        raise ValueError("x: expected contiguous complex64 [B,D,N]")
    Bsz, D, N = x.shape
    if A.dtype != torch.complex64 or tuple(A.shape) != (D, N) or not A.is_contiguous():
        raise ValueError("A: expected contiguous complex64 [D,N]")
    G = None
    for name, t in (("Bm", Bm), ("Cm", Cm)):
        shape = tuple(t.shape)
        if io == torch.bfloat16:
            ok = t.dtype == torch.bfloat16 and shape[-1:] == (2,)
            shape = shape[:-1]
        else:
            ok = io == torch.float32 and t.dtype == torch.complex64
        ok = ok and t.is_contiguous() and (shape == (Bsz, N) or (len(shape) == 3 and shape[0] == Bsz and shape[2] == N))
        g = shape[1] if ok and len(shape) == 3 else 1
        if not ok or (G is not None and g != G):
            raise ValueError(f"{name}: expected contiguous complex64 [B,N] or [B,G,N] (float32 I/O), or bfloat16 with a "
                             "trailing (re, im) axis")
        G = g
    if D % G:
        raise ValueError("D must be a multiple of the number of Bm/Cm groups")
    a = StepComplexArgs()
    a.struct_size = ctypes.sizeof(StepComplexArgs)
    a.B, a.D, a.N = Bsz, D, N
    a.bc_groups = G
    a.io_dtype = _io_dtype(u)
    a.disc = DISC[disc] if isinstance(disc, str) else int(disc)
    a.delta_softplus = int(bool(delta_softplus))
    a.x = x.data_ptr()
    a.u, a.u_stride_b, a.u_stride_d = _bd(u, "u", io)
    a.delta, a.delta_stride_b, a.delta_stride_d = _bd(delta, "delta", io)
    a.z, a.z_stride_b, a.z_stride_d = _bd(z, "z", io)
    a.A, a.Bm, a.Cm = A.data_ptr(), Bm.data_ptr(), Cm.data_ptr()
    a.Dskip = _ptr(_f32c(Dskip, "Dskip", (D,)))
    a.delta_bias = _ptr(_f32c(delta_bias, "delta_bias", (D,)))
    y = out if out is not None else torch.empty((Bsz, D), dtype=io, device=u.device)
    a.y, a.y_stride_b, a.y_stride_d = _bd(y, "y", io)
    a.stream = _stream()
    _check(lib().lrnnx_selective_step_complex(ctypes.byref(a)))
    return y


@_device_checked
def lrnnx_lti_step(lam, x, v):
    """One token of the LTI recurrence: x [B,P] complex64 is updated in place and returned."""
    for name, t in (("lam", lam), ("x", x), ("v", v)):
        if t.dtype != torch.complex64 or not t.is_contiguous():
            raise TypeError(f"{name}: expected contiguous complex64")
    Bsz, P = x.shape
    a = LtiStepArgs()
    a.struct_size = ctypes.sizeof(LtiStepArgs)
    a.B, a.P = Bsz, P
    a.lambda_, a.x, a.v = lam.data_ptr(), x.data_ptr(), v.data_ptr()
    a.stream = _stream()
    _check(lib().lrnnx_lti_step(ctypes.byref(a)))
    return x
