"""Seeded synthetic inputs for the five benchmark configurations.

This module holds no scan arithmetic: it only draws random tensors with the
shapes and distributions of the Mamba / LRU-shaped workloads (the paper
benchmarks on random tensors, Sec. 4.2) and rounds them once to the I/O dtype,
so that the CPU oracle and the HIP library consume identical bits.  It is the
only module both sides import.

All arrays are numpy.  Values of a bf16 configuration are returned as float32
arrays that are exactly representable in bf16 (round-to-nearest-even applied
here), so ``torch.from_numpy(a).to(torch.bfloat16)`` is lossless.
"""
from __future__ import annotations

import numpy as np

# name -> description of the benchmark configurations 0..4
CONFIGS = {
    "c0": dict(kind="selective", B=1, D=16, N=4, L=256, io="f32", gate=False,
               bias=("const", -2.0), seed=0),
    "c1": dict(kind="lti", B=4, P=256, L=4096, seed=1),
    "c2": dict(kind="selective", B=8, D=1536, N=16, L=2048, io="bf16", gate=True,
               bias=("uniform", -4.0, -2.0), seed=2),
    "c3": dict(kind="selective", B=1, D=2048, N=16, L=65536, io="bf16", gate=False,
               bias=("uniform", -4.0, -2.0), seed=3),
    "c4": dict(kind="selective", B=16, D=2560, N=16, L=4096, io="bf16", gate=True,
               bias=("uniform", -4.0, -2.0), seed=4),
}


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 -> nearest bf16 (ties to even), returned as float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    rounded = (bits + (((bits >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF))) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def _io_round(x: np.ndarray, io: str) -> np.ndarray:
    return round_to_bf16(x) if io == "bf16" else np.ascontiguousarray(x, dtype=np.float32)


def make_selective(B, D, N, L, io="f32", gate=False, bias=("const", -2.0), seed=0,
                   with_dy=True, with_x0=False, bc_groups=1, **_unused):
    """Inputs of the selective scan.

    A[d,n] = -exp(U(-1,1)); delta ~ N(0,1) (raw, pre-bias, pre-softplus);
    delta_bias constant or U(lo,hi) per channel; Bm, Cm ~ N(0,1) [B,L,N] shared
    by all channels ([B,G,L,N] with bc_groups = G > 1); u, Dskip, z, dy ~ N(0,1).
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    f32 = np.float32
    out = {}
    out["A"] = (-np.exp(rng.uniform(-1.0, 1.0, size=(D, N)))).astype(f32)
    out["Dskip"] = rng.standard_normal(D, dtype=f32)
    if bias is None:
        out["delta_bias"] = None
    elif bias[0] == "const":
        out["delta_bias"] = np.full(D, bias[1], dtype=f32)
    else:
        out["delta_bias"] = rng.uniform(bias[1], bias[2], size=D).astype(f32)
    bc_shape = (B, L, N) if bc_groups <= 1 else (B, bc_groups, L, N)
    out["Bm"] = _io_round(rng.standard_normal(bc_shape, dtype=f32), io)
    out["Cm"] = _io_round(rng.standard_normal(bc_shape, dtype=f32), io)
    out["u"] = _io_round(rng.standard_normal((B, D, L), dtype=f32), io)
    out["delta"] = _io_round(rng.standard_normal((B, D, L), dtype=f32), io)
    out["z"] = _io_round(rng.standard_normal((B, D, L), dtype=f32), io) if gate else None
    out["dy"] = _io_round(rng.standard_normal((B, D, L), dtype=f32), io) if with_dy else None
    out["x0"] = rng.standard_normal((B, D, N), dtype=f32) if with_x0 else None
    return out


def make_selective_complex(B, D, N, L, io="f32", gate=False, seed=0, with_x0=False, bc_groups=1):
    """Inputs of the selective scan with a complex diagonal A: as make_selective, with
    A[d,n] = -exp(U(-1,1)) + i U(-10,10) (complex64) and Bm, Cm = (N(0,1) + i N(0,1)) / sqrt(2), stored as
    float32 [B,L,N,2] (re, im) rounded to the I/O type ([B,G,L,N,2] with bc_groups = G > 1); delta_bias ~ U(-4,-2)
    per channel; x0 complex64."""
    rng = np.random.Generator(np.random.PCG64(seed))
    f32 = np.float32
    out = {}
    out["A"] = (-np.exp(rng.uniform(-1.0, 1.0, size=(D, N))) + 1j * rng.uniform(-10.0, 10.0, size=(D, N))).astype(np.complex64)
    out["Dskip"] = rng.standard_normal(D, dtype=f32)
    out["delta_bias"] = rng.uniform(-4.0, -2.0, size=D).astype(f32)
    s = f32(1.0 / np.sqrt(2.0))
    mshape = (B, L, N, 2) if bc_groups <= 1 else (B, bc_groups, L, N, 2)
    out["Bm"] = _io_round(rng.standard_normal(mshape, dtype=f32) * s, io)
    out["Cm"] = _io_round(rng.standard_normal(mshape, dtype=f32) * s, io)
    out["u"] = _io_round(rng.standard_normal((B, D, L), dtype=f32), io)
    out["delta"] = _io_round(rng.standard_normal((B, D, L), dtype=f32), io)
    out["z"] = _io_round(rng.standard_normal((B, D, L), dtype=f32), io) if gate else None
    out["x0"] = ((rng.standard_normal((B, D, N)) + 1j * rng.standard_normal((B, D, N))).astype(np.complex64)
                 if with_x0 else None)
    return out


def make_packed(D, N, lengths, io="f32", gate=True, seed=0, bc_groups=1, gap=0):
    """A packed variable-length batch: sequences of the given lengths one after the other on one time axis
    (`gap` unused steps before the first and after the last).  Same distributions as make_selective; returns the
    [D,L] / [L,N] (or [G,L,N]) arrays, x0 [S,D,N] and cu_seqlens (int64 [S+1])."""
    L = int(sum(lengths)) + 2 * gap
    p = make_selective(B=1, D=D, N=N, L=L, io=io, gate=gate, bias=("uniform", -4.0, -2.0), seed=seed,
                       bc_groups=bc_groups)
    out = {k: (None if v is None else v[0]) for k, v in p.items() if k in ("u", "delta", "z", "dy", "Bm", "Cm")}
    out.update(A=p["A"], Dskip=p["Dskip"], delta_bias=p["delta_bias"])
    rng = np.random.Generator(np.random.PCG64(seed + 1000))
    out["x0"] = rng.standard_normal((len(lengths), D, N), dtype=np.float32)
    out["cu_seqlens"] = (gap + np.concatenate([[0], np.cumsum(lengths)])).astype(np.int64)
    return out


def make_packed_complex(D, N, lengths, io="f32", gate=True, seed=0, bc_groups=1, gap=0):
    """make_packed for the complex-A scan: the arrays of make_selective_complex on one packed time axis ([D,L],
    maps [L,N,2] or [G,L,N,2]), x0 complex64 [S,D,N], dy [D,L] and cu_seqlens (int64 [S+1])."""
    L = int(sum(lengths)) + 2 * gap
    p = make_selective_complex(B=1, D=D, N=N, L=L, io=io, gate=gate, seed=seed, bc_groups=bc_groups)
    out = {k: (None if v is None else v[0]) for k, v in p.items() if k in ("u", "delta", "z", "Bm", "Cm")}
    out.update(A=p["A"], Dskip=p["Dskip"], delta_bias=p["delta_bias"])
    rng = np.random.Generator(np.random.PCG64(seed + 1000))
    S = len(lengths)
    out["x0"] = (rng.standard_normal((S, D, N)) + 1j * rng.standard_normal((S, D, N))).astype(np.complex64)
    out["dy"] = _io_round(rng.standard_normal((D, L), dtype=np.float32), io)
    out["cu_seqlens"] = (gap + np.concatenate([[0], np.cumsum(lengths)])).astype(np.int64)
    return out


def make_lti(B, P, L, seed=1, with_x0=False, with_gx=False, **_unused):
    """Inputs of the LTI complex-diagonal scan.

    lambda = r e^{i theta}, r ~ U(0.9, 0.999), theta ~ U(0, 2 pi);
    v = (N(0,1) + i N(0,1)) / sqrt(2), complex64 [B,L,P]; gx (the gradient reaching the states, for the
    backward pass) is drawn like v, after everything else.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    r = rng.uniform(0.9, 0.999, size=P)
    th = rng.uniform(0.0, 2.0 * np.pi, size=P)
    lam = (r * np.exp(1j * th)).astype(np.complex64)
    v = np.empty((B, L, P), dtype=np.complex64)
    s = np.float32(1.0 / np.sqrt(2.0))
    v.real = rng.standard_normal((B, L, P), dtype=np.float32) * s
    v.imag = rng.standard_normal((B, L, P), dtype=np.float32) * s
    x0 = None
    if with_x0:
        x0 = (rng.standard_normal((B, P)) + 1j * rng.standard_normal((B, P))).astype(np.complex64)
    gx = None
    if with_gx:
        gx = np.empty((B, L, P), dtype=np.complex64)
        gx.real = rng.standard_normal((B, L, P), dtype=np.float32) * s
        gx.imag = rng.standard_normal((B, L, P), dtype=np.float32) * s
    return {"lam": lam, "v": v, "x0": x0, "gx": gx}


def make_diag(B, P, L, cplx=False, seed=1, with_x0=False, with_gx=False, **_unused):
    """Inputs of the scan with caller-supplied coefficients (time-varying S5-style / gated recurrences).

    real: a ~ U(0.5, 1) (a forget gate), b ~ N(0,1), float32; complex: a = r e^{i theta} with r ~ U(0.9, 0.999),
    theta ~ U(0, 2 pi) drawn per element, b = (N(0,1) + i N(0,1)) / sqrt(2), complex64.  All [B,L,P].
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    if not cplx:
        a = rng.uniform(0.5, 1.0, size=(B, L, P)).astype(np.float32)
        b = rng.standard_normal((B, L, P), dtype=np.float32)
        x0 = rng.standard_normal((B, P), dtype=np.float32) if with_x0 else None
        gx = rng.standard_normal((B, L, P), dtype=np.float32) if with_gx else None      # drawn last
        return {"a": a, "b": b, "x0": x0, "gx": gx}
    r = rng.uniform(0.9, 0.999, size=(B, L, P))
    th = rng.uniform(0.0, 2.0 * np.pi, size=(B, L, P))
    a = (r * np.exp(1j * th)).astype(np.complex64)
    s = np.float32(1.0 / np.sqrt(2.0))
    b = np.empty((B, L, P), dtype=np.complex64)
    b.real = rng.standard_normal((B, L, P), dtype=np.float32) * s
    b.imag = rng.standard_normal((B, L, P), dtype=np.float32) * s
    x0 = (rng.standard_normal((B, P)) + 1j * rng.standard_normal((B, P))).astype(np.complex64) if with_x0 else None
    gx = None
    if with_gx:                                                                          # drawn last, like b
        gx = np.empty((B, L, P), dtype=np.complex64)
        gx.real = rng.standard_normal((B, L, P), dtype=np.float32) * s
        gx.imag = rng.standard_normal((B, L, P), dtype=np.float32) * s
    return {"a": a, "b": b, "x0": x0, "gx": gx}


def make(name: str, **overrides):
    """Inputs of benchmark configuration ``name`` ("c0".."c4"), optionally with fields overridden."""
    cfg = dict(CONFIGS[name])
    cfg.update(overrides)
    return (make_lti if cfg["kind"] == "lti" else make_selective)(**cfg), cfg
