"""fp64 CPU oracle for the diagonal linear-recurrence scan -- TEST INFRASTRUCTURE ONLY.

This package wraps ``lrnnx_oracle.c`` (plain sequential C, fp64) with ctypes and
numpy.  It states what the paper's Eq. 2 (Sec. 2.2) computes for a diagonal
state matrix under the discretisations named in Sec. 3; see the C file's header
for the formulas, the layouts and the list of pins.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import it.  It imports nothing from the HIP package and the
HIP package imports nothing from here.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lrnnx_oracle.c")
_LIB = os.path.join(_HERE, "liblrnnx_oracle.so")

DISC = {"zoh_s6": 0, "zoh": 1, "bilinear": 2, "dirac": 3}


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP, no fast-math). Returns the .so path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.lrnnx_oracle_softplus.restype = ctypes.c_double
        _lib.lrnnx_oracle_softplus.argtypes = [ctypes.c_double]
        _lib.lrnnx_oracle_disc.restype = None
        _lib.lrnnx_oracle_disc_complex.restype = None
        _lib.lrnnx_oracle_num_threads.restype = ctypes.c_int
    return _lib


def _p(a):
    """double* of a contiguous float64 array, or NULL."""
    if a is None:
        return ctypes.c_void_p(0)
    assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.c_void_p)


def _f64(a):
    return None if a is None else np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _c128(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.complex128))


def num_threads() -> int:
    return int(_load().lrnnx_oracle_num_threads())


def softplus(s: float) -> float:
    return float(_load().lrnnx_oracle_softplus(float(s)))


def disc_terms(disc, dt: float, A: float):
    """(a, g, da/ddt, da/dA, dg/ddt, dg/dA) of one discretisation at (dt, A)."""
    out = (ctypes.c_double * 6)()
    _load().lrnnx_oracle_disc(ctypes.c_int(_disc(disc)), ctypes.c_double(dt), ctypes.c_double(A), out)
    return tuple(out)


def _disc(disc) -> int:
    return DISC[disc] if isinstance(disc, str) else int(disc)


def _groups(Bm, Cm, Bsz, L, N):
    """Number of B/C groups: Bm, Cm are [B,L,N] (one group) or [B,G,L,N] (channel d reads group d // (D/G))."""
    assert Bm.shape == Cm.shape
    if Bm.ndim == 3:
        assert Bm.shape == (Bsz, L, N)
        return 1
    assert Bm.ndim == 4 and Bm.shape[0] == Bsz and Bm.shape[2:] == (L, N)
    return Bm.shape[1]


def selective_scan_fwd(u, delta, A, Bm, Cm, Dskip=None, delta_bias=None, z=None, x0=None,
                       disc="zoh_s6", delta_softplus=True, return_states=False):
    """y [B,D,L], x_last [B,D,N] (and every state [B,D,L,N] if asked) of Eq. 2 with diagonal A(k)."""
    u, delta, A, Bm, Cm = map(_f64, (u, delta, A, Bm, Cm))
    Dskip, delta_bias, z, x0 = map(_f64, (Dskip, delta_bias, z, x0))
    Bsz, D, L = u.shape
    N = A.shape[1]
    assert delta.shape == (Bsz, D, L) and A.shape == (D, N)
    G = _groups(Bm, Cm, Bsz, L, N)
    y = np.empty((Bsz, D, L))
    x_last = np.empty((Bsz, D, N))
    xs = np.empty((Bsz, D, L, N)) if return_states else None
    rc = _load().lrnnx_oracle_selective_scan_fwd(
        ctypes.c_int(Bsz), ctypes.c_int(D), ctypes.c_int(N), ctypes.c_int(G), ctypes.c_long(L),
        ctypes.c_int(_disc(disc)), ctypes.c_int(int(bool(delta_softplus))),
        _p(u), _p(delta), _p(A), _p(Bm), _p(Cm), _p(Dskip), _p(delta_bias), _p(z), _p(x0),
        _p(y), _p(x_last), _p(xs))
    if rc != 0:
        raise ValueError(f"oracle fwd: bad arguments (rc={rc})")
    return (y, x_last, xs) if return_states else (y, x_last)


def selective_scan_fwd_complex(u, delta, A, Bm, Cm, Dskip=None, delta_bias=None, z=None, x0=None,
                               disc="zoh_s6", delta_softplus=True):
    """y [B,D,L] (real) and x_last [B,D,N] (complex128) of Eq. 2 with a complex diagonal A [D,N] and complex
    maps Bm, Cm [B,L,N]: y = Re(sum_n Cm x) + Dskip u, then the optional gate."""
    u, delta = _f64(u), _f64(delta)
    A, Bm, Cm = _c128(A), _c128(Bm), _c128(Cm)
    Dskip, delta_bias, z = map(_f64, (Dskip, delta_bias, z))
    x0c = None if x0 is None else _c128(x0)
    Bsz, D, L = u.shape
    N = A.shape[1]
    assert A.shape == (D, N)
    G = _groups(Bm, Cm, Bsz, L, N)
    y = np.empty((Bsz, D, L))
    x_last = np.empty((Bsz, D, N), dtype=np.complex128)
    cp = lambda t: ctypes.c_void_p(0) if t is None else t.ctypes.data_as(ctypes.c_void_p)
    rc = _load().lrnnx_oracle_selective_scan_fwd_complex(
        ctypes.c_int(Bsz), ctypes.c_int(D), ctypes.c_int(N), ctypes.c_int(G), ctypes.c_long(L),
        ctypes.c_int(_disc(disc)), ctypes.c_int(int(bool(delta_softplus))),
        _p(u), _p(delta), cp(A), cp(Bm), cp(Cm), _p(Dskip), _p(delta_bias), _p(z), cp(x0c), _p(y), cp(x_last))
    if rc != 0:
        raise ValueError(f"oracle complex fwd: bad arguments (rc={rc})")
    return y, x_last


def disc_terms_complex(disc, dt: float, A: complex):
    """(a, g, da/ddt, da/dA, dg/ddt, dg/dA) of one discretisation at real dt and complex A, as complex numbers."""
    out = (ctypes.c_double * 12)()
    A = complex(A)
    _load().lrnnx_oracle_disc_complex(ctypes.c_int(_disc(disc)), ctypes.c_double(dt), ctypes.c_double(A.real),
                                      ctypes.c_double(A.imag), out)
    return tuple(complex(out[2 * i], out[2 * i + 1]) for i in range(6))


def selective_scan_bwd_complex(u, delta, A, Bm, Cm, dy, Dskip=None, delta_bias=None, z=None, x0=None,
                               disc="zoh_s6", delta_softplus=True):
    """Gradients of sum(dy * y) for selective_scan_fwd_complex.  The gradient of a complex input q is
    dLoss/dRe q + i dLoss/dIm q (complex128: dA, dBm, dCm, dx0); du, ddelta, dz, dD, dbias are real."""
    u, delta, dy = _f64(u), _f64(delta), _f64(dy)
    A, Bm, Cm = _c128(A), _c128(Bm), _c128(Cm)
    Dskip, delta_bias, z = map(_f64, (Dskip, delta_bias, z))
    x0c = None if x0 is None else _c128(x0)
    Bsz, D, L = u.shape
    N = A.shape[1]
    assert A.shape == (D, N) and dy.shape == (Bsz, D, L)
    G = _groups(Bm, Cm, Bsz, L, N)
    c128 = np.complex128
    out = {
        "du": np.empty((Bsz, D, L)), "ddelta": np.empty((Bsz, D, L)),
        "dA": np.empty((D, N), dtype=c128), "dBm": np.empty(Bm.shape, dtype=c128), "dCm": np.empty(Cm.shape, dtype=c128),
        "dD": np.empty(D) if Dskip is not None else None,
        "dbias": np.empty(D) if delta_bias is not None else None,
        "dz": np.empty((Bsz, D, L)) if z is not None else None,
        "dx0": np.empty((Bsz, D, N), dtype=c128),
    }
    cp = lambda t: ctypes.c_void_p(0) if t is None else t.ctypes.data_as(ctypes.c_void_p)
    rc = _load().lrnnx_oracle_selective_scan_bwd_complex(
        ctypes.c_int(Bsz), ctypes.c_int(D), ctypes.c_int(N), ctypes.c_int(G), ctypes.c_long(L),
        ctypes.c_int(_disc(disc)), ctypes.c_int(int(bool(delta_softplus))),
        _p(u), _p(delta), cp(A), cp(Bm), cp(Cm), _p(Dskip), _p(delta_bias), _p(z), cp(x0c), _p(dy),
        _p(out["du"]), _p(out["ddelta"]), cp(out["dA"]), cp(out["dBm"]), cp(out["dCm"]),
        _p(out["dD"]), _p(out["dbias"]), _p(out["dz"]), cp(out["dx0"]))
    if rc != 0:
        raise ValueError(f"oracle complex bwd: bad arguments (rc={rc})")
    return out


def selective_scan_bwd(u, delta, A, Bm, Cm, dy, Dskip=None, delta_bias=None, z=None, x0=None,
                       disc="zoh_s6", delta_softplus=True):
    """Gradients of sum(dy * y) w.r.t. every input, as a dict of float64 arrays."""
    u, delta, A, Bm, Cm, dy = map(_f64, (u, delta, A, Bm, Cm, dy))
    Dskip, delta_bias, z, x0 = map(_f64, (Dskip, delta_bias, z, x0))
    Bsz, D, L = u.shape
    N = A.shape[1]
    G = _groups(Bm, Cm, Bsz, L, N)
    out = {
        "du": np.empty((Bsz, D, L)), "ddelta": np.empty((Bsz, D, L)),
        "dA": np.empty((D, N)), "dBm": np.empty(Bm.shape), "dCm": np.empty(Cm.shape),
        "dD": np.empty(D) if Dskip is not None else None,
        "dbias": np.empty(D) if delta_bias is not None else None,
        "dz": np.empty((Bsz, D, L)) if z is not None else None,
        "dx0": np.empty((Bsz, D, N)),
    }
    rc = _load().lrnnx_oracle_selective_scan_bwd(
        ctypes.c_int(Bsz), ctypes.c_int(D), ctypes.c_int(N), ctypes.c_int(G), ctypes.c_long(L),
        ctypes.c_int(_disc(disc)), ctypes.c_int(int(bool(delta_softplus))),
        _p(u), _p(delta), _p(A), _p(Bm), _p(Cm), _p(Dskip), _p(delta_bias), _p(z), _p(x0), _p(dy),
        _p(out["du"]), _p(out["ddelta"]), _p(out["dA"]), _p(out["dBm"]), _p(out["dCm"]),
        _p(out["dD"]), _p(out["dbias"]), _p(out["dz"]), _p(out["dx0"]))
    if rc != 0:
        raise ValueError(f"oracle bwd: bad arguments (rc={rc})")
    return out


def lti_diag_scan(lam, v, x0=None):
    """x [B,L,P] complex128 of x_k = lam * x_{k-1} + v_k (S5/LRU recurrence, Sec. 2.2.1)."""
    lam, v = _c128(lam), _c128(v)
    Bsz, L, P = v.shape
    assert lam.shape == (P,)
    x0c = None if x0 is None else _c128(x0)
    x = np.empty((Bsz, L, P), dtype=np.complex128)
    rc = _load().lrnnx_oracle_lti_diag_scan(
        ctypes.c_int(Bsz), ctypes.c_long(L), ctypes.c_int(P),
        lam.ctypes.data_as(ctypes.c_void_p), v.ctypes.data_as(ctypes.c_void_p),
        ctypes.c_void_p(0) if x0c is None else x0c.ctypes.data_as(ctypes.c_void_p),
        x.ctypes.data_as(ctypes.c_void_p))
    if rc != 0:
        raise ValueError(f"oracle lti: bad arguments (rc={rc})")
    return x


def _packed_slices(cu, L):
    cu = [int(c) for c in np.asarray(cu).ravel()]
    assert len(cu) >= 2 and all(0 <= cu[i] <= cu[i + 1] <= L for i in range(len(cu) - 1))
    return [(cu[i], cu[i + 1]) for i in range(len(cu) - 1)]


def _maps4(M):
    """Packed maps [L,N] or [G,L,N] as [1,G,L,N]."""
    M = np.asarray(M, dtype=np.float64)
    return M[None, None] if M.ndim == 2 else M[None]


def selective_scan_fwd_packed(u, delta, A, Bm, Cm, cu_seqlens, Dskip=None, delta_bias=None, z=None, x0=None,
                              disc="zoh_s6", delta_softplus=True):
    """Packed variable-length batch: S independent sequences lie one after the other on one time axis; sequence s is
    steps cu[s] .. cu[s+1]-1 and starts from x0[s] (or 0).  u, delta, z: [D,L]; Bm, Cm: [L,N] or [G,L,N];
    x0: [S,D,N].  By definition the result is the plain scan of every sequence on its own slice.  Returns
    y [D,L] (zero outside every sequence) and x_last [S,D,N]."""
    u, delta = _f64(u), _f64(delta)
    D, L = u.shape
    Bm4, Cm4 = _maps4(Bm), _maps4(Cm)
    sl = _packed_slices(cu_seqlens, L)
    y = np.zeros((D, L))
    x_last = np.zeros((len(sl), D, np.asarray(A).shape[1]))
    for s, (o, e) in enumerate(sl):
        ys, xs = selective_scan_fwd(u[None, :, o:e], delta[None, :, o:e], A, Bm4[:, :, o:e], Cm4[:, :, o:e], Dskip=Dskip,
                                    delta_bias=delta_bias, z=None if z is None else np.asarray(z)[None, :, o:e],
                                    x0=None if x0 is None else np.asarray(x0)[s:s + 1], disc=disc,
                                    delta_softplus=delta_softplus)
        y[:, o:e], x_last[s] = ys[0], xs[0]
    return y, x_last


def selective_scan_bwd_packed(u, delta, A, Bm, Cm, dy, cu_seqlens, Dskip=None, delta_bias=None, z=None, x0=None,
                              disc="zoh_s6", delta_softplus=True):
    """Gradients of sum(dy * y) for the packed batch above: per-step gradients are those of each sequence on its
    slice, parameter gradients (dA, dD, dbias) add up over the sequences; dBm, dCm have the shape of Bm."""
    u, delta, dy = _f64(u), _f64(delta), _f64(dy)
    D, L = u.shape
    Bm4, Cm4 = _maps4(Bm), _maps4(Cm)
    sl = _packed_slices(cu_seqlens, L)
    N = np.asarray(A).shape[1]
    out = {"du": np.zeros((D, L)), "ddelta": np.zeros((D, L)), "dz": None if z is None else np.zeros((D, L)),
           "dA": np.zeros((D, N)), "dBm": np.zeros(Bm4.shape[1:]), "dCm": np.zeros(Cm4.shape[1:]),
           "dD": None if Dskip is None else np.zeros(D), "dbias": None if delta_bias is None else np.zeros(D),
           "dx0": np.zeros((len(sl), D, N))}
    for s, (o, e) in enumerate(sl):
        g = selective_scan_bwd(u[None, :, o:e], delta[None, :, o:e], A, Bm4[:, :, o:e], Cm4[:, :, o:e], dy[None, :, o:e],
                               Dskip=Dskip, delta_bias=delta_bias, z=None if z is None else np.asarray(z)[None, :, o:e],
                               x0=None if x0 is None else np.asarray(x0)[s:s + 1], disc=disc,
                               delta_softplus=delta_softplus)
        for k in ("du", "ddelta", "dz"):
            if out[k] is not None:
                out[k][:, o:e] = g[k][0]
        out["dBm"][:, o:e], out["dCm"][:, o:e] = g["dBm"][0], g["dCm"][0]
        for k in ("dA", "dD", "dbias"):
            if out[k] is not None:
                out[k] += g[k]
        out["dx0"][s] = g["dx0"][0]
    if np.asarray(Bm).ndim == 2:
        out["dBm"], out["dCm"] = out["dBm"][0], out["dCm"][0]
    return out


def _cmaps4(M):
    """Packed complex maps [L,N] or [G,L,N] as [1,G,L,N]."""
    M = _c128(M)
    return M[None, None] if M.ndim == 2 else M[None]


def selective_scan_fwd_complex_packed(u, delta, A, Bm, Cm, cu_seqlens, Dskip=None, delta_bias=None, z=None, x0=None,
                                      disc="zoh_s6", delta_softplus=True):
    """The packed variable-length batch of selective_scan_fwd_packed with a complex diagonal A: by definition the
    complex scan of every sequence on its own slice.  u, delta, z: [D,L]; Bm, Cm: complex [L,N] or [G,L,N];
    x0: complex [S,D,N].  Returns y [D,L] (zero outside every sequence) and x_last [S,D,N] complex128."""
    u, delta = _f64(u), _f64(delta)
    D, L = u.shape
    Bm4, Cm4 = _cmaps4(Bm), _cmaps4(Cm)
    sl = _packed_slices(cu_seqlens, L)
    y = np.zeros((D, L))
    x_last = np.zeros((len(sl), D, np.asarray(A).shape[1]), dtype=np.complex128)
    for s, (o, e) in enumerate(sl):
        ys, xs = selective_scan_fwd_complex(u[None, :, o:e], delta[None, :, o:e], A, Bm4[:, :, o:e], Cm4[:, :, o:e],
                                            Dskip=Dskip, delta_bias=delta_bias,
                                            z=None if z is None else np.asarray(z)[None, :, o:e],
                                            x0=None if x0 is None else np.asarray(x0)[s:s + 1], disc=disc,
                                            delta_softplus=delta_softplus)
        y[:, o:e], x_last[s] = ys[0], xs[0]
    return y, x_last


def selective_scan_bwd_complex_packed(u, delta, A, Bm, Cm, dy, cu_seqlens, Dskip=None, delta_bias=None, z=None,
                                      x0=None, disc="zoh_s6", delta_softplus=True):
    """Gradients of sum(dy * y) for the packed complex batch above: per-step gradients are those of each sequence on
    its slice, parameter gradients (dA, dD, dbias) add up over the sequences; dBm, dCm have the shape of Bm."""
    u, delta, dy = _f64(u), _f64(delta), _f64(dy)
    D, L = u.shape
    Bm4, Cm4 = _cmaps4(Bm), _cmaps4(Cm)
    sl = _packed_slices(cu_seqlens, L)
    N = np.asarray(A).shape[1]
    c128 = np.complex128
    out = {"du": np.zeros((D, L)), "ddelta": np.zeros((D, L)), "dz": None if z is None else np.zeros((D, L)),
           "dA": np.zeros((D, N), dtype=c128), "dBm": np.zeros(Bm4.shape[1:], dtype=c128),
           "dCm": np.zeros(Cm4.shape[1:], dtype=c128),
           "dD": None if Dskip is None else np.zeros(D), "dbias": None if delta_bias is None else np.zeros(D),
           "dx0": np.zeros((len(sl), D, N), dtype=c128)}
    for s, (o, e) in enumerate(sl):
        g = selective_scan_bwd_complex(u[None, :, o:e], delta[None, :, o:e], A, Bm4[:, :, o:e], Cm4[:, :, o:e],
                                       dy[None, :, o:e], Dskip=Dskip, delta_bias=delta_bias,
                                       z=None if z is None else np.asarray(z)[None, :, o:e],
                                       x0=None if x0 is None else np.asarray(x0)[s:s + 1], disc=disc,
                                       delta_softplus=delta_softplus)
        for k in ("du", "ddelta", "dz"):
            if out[k] is not None:
                out[k][:, o:e] = g[k][0]
        out["dBm"][:, o:e], out["dCm"][:, o:e] = g["dBm"][0], g["dCm"][0]
        for k in ("dA", "dD", "dbias"):
            if out[k] is not None:
                out[k] += g[k]
        out["dx0"][s] = g["dx0"][0]
    if np.asarray(Bm).ndim == 2:
        out["dBm"], out["dCm"] = out["dBm"][0], out["dCm"][0]
    return out


def diag_scan(a, b, x0=None):
    """x [B,L,P] of x_k = a_k * x_{k-1} + b_k for caller-supplied coefficients; real (float64) or complex (complex128)
    according to the dtype of the inputs."""
    cplx = np.iscomplexobj(a) or np.iscomplexobj(b) or (x0 is not None and np.iscomplexobj(x0))
    conv = _c128 if cplx else _f64
    a, b = conv(a), conv(b)
    Bsz, L, P = b.shape
    assert a.shape == b.shape
    x0c = None if x0 is None else conv(x0)
    x = np.empty((Bsz, L, P), dtype=np.complex128 if cplx else np.float64)
    cp = lambda t: ctypes.c_void_p(0) if t is None else t.ctypes.data_as(ctypes.c_void_p)
    rc = _load().lrnnx_oracle_diag_scan(ctypes.c_int(Bsz), ctypes.c_long(L), ctypes.c_int(P), ctypes.c_int(int(cplx)),
                                        cp(a), cp(b), cp(x0c), cp(x))
    if rc != 0:
        raise ValueError(f"oracle diag scan: bad arguments (rc={rc})")
    return x


def diag_scan_bwd(a, b, gx, x0=None):
    """Gradients (da, db [B,L,P], dx0 [B,P]) of a real loss through x_k = a_k x_{k-1} + b_k, gx being the gradient
    reaching the states; real or complex like diag_scan."""
    cplx = any(np.iscomplexobj(t) for t in (a, b, gx) if t is not None) or (x0 is not None and np.iscomplexobj(x0))
    conv = _c128 if cplx else _f64
    a, b, gx = conv(a), conv(b), conv(gx)
    Bsz, L, P = b.shape
    assert a.shape == b.shape == gx.shape
    x0c = None if x0 is None else conv(x0)
    dt = np.complex128 if cplx else np.float64
    da, db, dx0 = np.empty((Bsz, L, P), dtype=dt), np.empty((Bsz, L, P), dtype=dt), np.empty((Bsz, P), dtype=dt)
    cp = lambda t: ctypes.c_void_p(0) if t is None else t.ctypes.data_as(ctypes.c_void_p)
    rc = _load().lrnnx_oracle_diag_scan_bwd(ctypes.c_int(Bsz), ctypes.c_long(L), ctypes.c_int(P), ctypes.c_int(int(cplx)),
                                            cp(a), cp(b), cp(x0c), cp(gx), cp(da), cp(db), cp(dx0))
    if rc != 0:
        raise ValueError(f"oracle diag scan bwd: bad arguments (rc={rc})")
    return da, db, dx0


def lti_diag_scan_bwd(lam, v, gx, x0=None):
    """Gradients (dv [B,L,P], dlam [P], dx0 [B,P]) of a real loss with dLoss/dRe(x) + i dLoss/dIm(x) = gx."""
    lam, v, gx = _c128(lam), _c128(v), _c128(gx)
    Bsz, L, P = v.shape
    assert lam.shape == (P,) and gx.shape == v.shape
    x0c = None if x0 is None else _c128(x0)
    dv = np.empty((Bsz, L, P), dtype=np.complex128)
    dlam = np.empty(P, dtype=np.complex128)
    dx0 = np.empty((Bsz, P), dtype=np.complex128)
    cp = lambda a: ctypes.c_void_p(0) if a is None else a.ctypes.data_as(ctypes.c_void_p)
    rc = _load().lrnnx_oracle_lti_diag_scan_bwd(
        ctypes.c_int(Bsz), ctypes.c_long(L), ctypes.c_int(P), cp(lam), cp(v), cp(x0c), cp(gx), cp(dv), cp(dlam), cp(dx0))
    if rc != 0:
        raise ValueError(f"oracle lti bwd: bad arguments (rc={rc})")
    return dv, dlam, dx0


def selective_step(x, u, delta, A, Bm, Cm, Dskip=None, delta_bias=None, z=None, disc="zoh_s6", delta_softplus=True):
    """One token: returns (y [B,D], new state [B,D,N]); the input state is not modified."""
    x = np.array(_f64(x), copy=True)
    u, delta, A, Bm, Cm = map(_f64, (u, delta, A, Bm, Cm))
    Dskip, delta_bias, z = map(_f64, (Dskip, delta_bias, z))
    Bsz, D, N = x.shape
    assert u.shape == (Bsz, D) and delta.shape == (Bsz, D) and Bm.shape == Cm.shape
    assert Bm.shape == (Bsz, N) or (Bm.ndim == 3 and Bm.shape[0] == Bsz and Bm.shape[2] == N)
    G = 1 if Bm.ndim == 2 else Bm.shape[1]
    y = np.empty((Bsz, D))
    rc = _load().lrnnx_oracle_selective_step(
        ctypes.c_int(Bsz), ctypes.c_int(D), ctypes.c_int(N), ctypes.c_int(G), ctypes.c_int(_disc(disc)),
        ctypes.c_int(int(bool(delta_softplus))), _p(x), _p(u), _p(delta), _p(A), _p(Bm), _p(Cm),
        _p(Dskip), _p(delta_bias), _p(z), _p(y))
    if rc != 0:
        raise ValueError(f"oracle step: bad arguments (rc={rc})")
    return y, x


def selective_step_complex(x, u, delta, A, Bm, Cm, Dskip=None, delta_bias=None, z=None, disc="zoh_s6",
                           delta_softplus=True):
    """One token with a complex diagonal A: returns (y [B,D] real, new state [B,D,N] complex128); the input state is
    not modified.  Bm, Cm [B,N] complex."""
    x = np.array(_c128(x), copy=True)
    u, delta = _f64(u), _f64(delta)
    A, Bm, Cm = _c128(A), _c128(Bm), _c128(Cm)
    Dskip, delta_bias, z = map(_f64, (Dskip, delta_bias, z))
    Bsz, D, N = x.shape
    assert u.shape == (Bsz, D) and delta.shape == (Bsz, D) and A.shape == (D, N)
    assert Bm.shape == Cm.shape
    assert Bm.shape == (Bsz, N) or (Bm.ndim == 3 and Bm.shape[0] == Bsz and Bm.shape[2] == N)
    G = 1 if Bm.ndim == 2 else Bm.shape[1]
    y = np.empty((Bsz, D))
    cp = lambda t: t.ctypes.data_as(ctypes.c_void_p)
    rc = _load().lrnnx_oracle_selective_step_complex(
        ctypes.c_int(Bsz), ctypes.c_int(D), ctypes.c_int(N), ctypes.c_int(G), ctypes.c_int(_disc(disc)),
        ctypes.c_int(int(bool(delta_softplus))), cp(x), _p(u), _p(delta), cp(A), cp(Bm), cp(Cm),
        _p(Dskip), _p(delta_bias), _p(z), _p(y))
    if rc != 0:
        raise ValueError(f"oracle complex step: bad arguments (rc={rc})")
    return y, x


def lti_step(lam, x, v):
    """One token of x <- lam * x + v for complex [B,P] arrays; returns the new state."""
    lam, v = _c128(lam), _c128(v)
    x = np.array(_c128(x), copy=True)
    Bsz, P = x.shape
    rc = _load().lrnnx_oracle_lti_step(ctypes.c_int(Bsz), ctypes.c_int(P), lam.ctypes.data_as(ctypes.c_void_p),
                                       x.ctypes.data_as(ctypes.c_void_p), v.ctypes.data_as(ctypes.c_void_p))
    if rc != 0:
        raise ValueError(f"oracle lti step: bad arguments (rc={rc})")
    return x
