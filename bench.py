#!/usr/bin/env python3
"""Benchmark of the MI355X diagonal linear-recurrence scan (one GPU).

A step is one forward + one backward selective scan on benchmark configuration 2 (Mamba-block
shape: B=8, D=1536, N=16, L=2048, bf16 I/O, fp32 state, SiLU gate), inputs resident in
HBM.  The metric is scan elements/s, elements = B*L*D*N per pass (2 passes per step).
The same run also times the other single-kernel workloads (config 1 LTI scan, config 3
long-sequence forward on both paths, config 4 backward) and reports them under
"other_configs"; they are not part of `value`.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline] [--quick] [--alu-probe]

Prints ONE JSON line.  `roofline` is for the dominant kernel of the step (the backward
kernel): algorithmic HBM bytes per launch / average launch time measured with HIP
events on the launch stream, against the 8 TB/s HBM peak.  `roofline_alu` prices the
same launch against the fp32 vector-ALU issue rate, which is the tighter bound for this
path (N exponentials per loaded element).  `cpu_baseline` is the fp64
oracle timed on the host cores on the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# 256 CUs x 4 SIMDs x 32 lanes per clock x 2.4 GHz = 78.6e12 plain fp32 lane-instructions/s: the published
# 157.3 TFLOP/s fp32 vector peak counts an FMA as two flops and needs no packed form.  Measured with the probe
# (`--alu-probe`, csrc/valu_probe.hip): a plain FMA/MUL/ADD issues every 2.6 nominal cycles per SIMD (60e12 lanes/s),
# an instruction with a DPP or scalar-register operand, a select, a conversion or a min/max every 4.4 (35e12), a
# transcendental every 8.4 (18e12); one wavefront alone issues at most every 5.5 cycles.
VALU_PEAK_TLANEOPS = 78.6
PROBE = os.path.join(ROOT, "paper_2602_08810_amd", "valu_probe")

# Measured HBM traffic of the backward kernel on config 2 comes from the counter summary under profiles/ (rocprofv3
# --pmc FETCH_SIZE / WRITE_SIZE, scaled by a copy kernel of known size).  The summary names the sources of the kernel
# it was taken on by a hash; if they have changed since, the figure is stale and `traffic` is null.
TRAFFIC_SUMMARY = os.path.join(ROOT, "profiles", "config2_fwd_bwd_hbm_traffic.md")
KERNEL_SOURCES = [os.path.join(ROOT, "paper_2602_08810_amd", "csrc", f)
                  for f in ("selective_bwd.hip", "scan_common.hpp", "kernels.hpp")]


def _alu_probe():
    """Runs the stand-alone probe (its own process: it shares nothing with the library) and returns
    {instruction: {"chains c, w waves/SIMD": cycles per instruction and SIMD at the nominal 2.4 GHz}}."""
    import re
    import subprocess
    if not os.path.exists(PROBE):
        raise SystemExit(f"bench.py: {PROBE} is not built (python -m paper_2602_08810_amd.build)")
    r = subprocess.run([PROBE], capture_output=True, text=True, timeout=120)
    if r.returncode != 0:
        raise SystemExit(f"bench.py: the ALU probe failed:\n{r.stderr}")
    out = {}
    for m in re.finditer(r"^(.*?)\s+chains (\d+)\s+waves/SIMD (\d+)\s+([0-9.]+) cycles", r.stdout, re.M):
        out.setdefault(m.group(1).strip(), {})[f"chains {m.group(2)}, {m.group(3)} waves/SIMD"] = float(m.group(4))
    return out


def kernel_source_hash():
    import hashlib
    h = hashlib.sha256()
    for f in KERNEL_SOURCES:
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def measured_traffic():
    """(bytes per launch or None, note) from the machine-readable line of the counter summary."""
    import re
    try:
        text = open(TRAFFIC_SUMMARY).read()
    except OSError:
        return None, "no counter summary"
    m = re.search(r"bwd_traffic_bytes_per_launch\s*=\s*(\d+)\s*;\s*kernel_source_hash\s*=\s*([0-9a-f]+)", text)
    if not m:
        return None, "counter summary has no traffic line"
    if m.group(2) != kernel_source_hash():
        return None, f"stale: counters were taken on kernel sources {m.group(2)}, this tree has {kernel_source_hash()}"
    return int(m.group(1)), "profiles/config2_fwd_bwd_hbm_traffic.md"


def _selective_bytes(B, D, N, L, es, gate, bwd):
    """Algorithmic HBM bytes: every I/O tensor once, Bm/Cm once, reduced grads once, no state traffic."""
    per = B * D * L * es
    bc = 2 * B * L * N * es
    if not bwd:
        return per * (3 + (1 if gate else 0)) + bc
    return per * (5 + (2 if gate else 0)) + bc + 2 * B * L * N * 4


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=90)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--repeats", type=int, default=5,
                    help="experiments of --steps steps each (the paper's protocol, Sec. 4.2: mean and std over the "
                         "experiments' means); the timed region is --repeats x --steps steps")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--quick", action="store_true", help="skip the other configs")
    ap.add_argument("--alu-probe", action="store_true",
                    help="also run the vector-ALU issue-rate probe (paper_2602_08810_amd/valu_probe) and report it")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain device copy of 256 MiB (reference for scaling rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(rows (b,d) are independent recurrences: a multi-GPU job would shard B or D and all-reduce the shared gradients)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2602_08810_amd import api, workloads
    api.lib()                                   # fail loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")

    # ------------------------------------------------------------------ headline workload: config 2, fwd + bwd
    p, cfg = workloads.make("c2")
    B, D, N, L = cfg["B"], cfg["D"], cfg["N"], cfg["L"]
    io = torch.bfloat16

    def up(a, dt=None):
        t = torch.from_numpy(a).to(dev)
        return t.to(dt) if dt is not None else t

    t = dict(u=up(p["u"], io), delta=up(p["delta"], io), A=up(p["A"]), Bm=up(p["Bm"], io), Cm=up(p["Cm"], io),
             Dskip=up(p["Dskip"]), delta_bias=up(p["delta_bias"]), z=up(p["z"], io))
    dy = up(p["dy"], io)
    I = api.lrnnx_ckpt_interval()
    y = torch.empty_like(t["u"])
    ckpt = torch.empty((B, D, (L + I - 1) // I, N), dtype=torch.float32, device=dev)
    outs = {k: torch.empty_like(t["u"]) for k in ("du", "ddelta", "dz")}
    outs.update(dA=torch.empty((D, N), device=dev), dBm=torch.empty((B, L, N), device=dev),
                dCm=torch.empty((B, L, N), device=dev), dD=torch.empty(D, device=dev), dbias=torch.empty(D, device=dev))
    ws = torch.empty(max(api.lrnnx_workspace_bytes(api.WS_FWD, B, D, N, L, api.BF16), 16), dtype=torch.uint8, device=dev)

    def fwd():
        api.lrnnx_selective_scan_fwd(**t, out=y, ckpt_out=ckpt, workspace=ws)

    def bwd():
        api.lrnnx_selective_scan_bwd(**t, dy=dy, ckpt=ckpt, outs=outs)

    def step():
        fwd()
        bwd()

    if args.copy_calibration:
        src = torch.zeros(64 * 1024 * 1024, dtype=torch.float32, device=dev)      # 256 MiB read + 256 MiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # what a plain device copy reaches on this machine (1 GiB read + 1 GiB written, far beyond the Infinity Cache): the
    # practical ceiling next to the 8 TB/s data-sheet peak
    src = torch.zeros(256 * 1024 * 1024, dtype=torch.float32, device=dev)
    dst = torch.empty_like(src)
    copy_t = _time(torch, lambda: dst.copy_(src), 10)
    copy_ceiling = 2 * src.numel() * 4 / copy_t / 1e9
    del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # timed region: exactly K steps; per-kernel HIP events (torch events on the current stream, which is the
    # stream handed to the library) bracket the forward and the backward launches inside it
    K = args.steps
    exp_means = []
    fwd_ms, bwd_ms = [], []
    for _rep in range(max(1, args.repeats)):
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(K)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(K):
            ev[k][0].record()
            fwd()
            ev[k][1].record()
            bwd()
            ev[k][2].record()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        exp_means.append((t1 - t0) * 1e3 / K)
        fwd_ms += [ev[k][0].elapsed_time(ev[k][1]) for k in range(K)]
        bwd_ms += [ev[k][1].elapsed_time(ev[k][2]) for k in range(K)]
    ms_per_step = float(np.mean(exp_means))
    elements = B * L * D * N
    value = 2 * elements / (ms_per_step * 1e-3)
    fwd_t, bwd_t = float(np.mean(fwd_ms)) * 1e-3, float(np.mean(bwd_ms)) * 1e-3

    fwd_bytes = _selective_bytes(B, D, N, L, 2, True, False) + ckpt.numel() * 4
    bwd_bytes = _selective_bytes(B, D, N, L, 2, True, True) + ckpt.numel() * 4
    traffic, traffic_note = measured_traffic()
    roofline = {"bound": "hbm", "kernel": "k_ss_bwd<bf16,N=16> (config 2 backward)",
                "achieved": bwd_bytes / bwd_t / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": bwd_bytes / bwd_t / 1e9 / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_note,
                "algorithmic_bytes": bwd_bytes, "avg_launch_us": bwd_t * 1e6,
                "copy_ceiling_GBs": copy_ceiling, "frac_of_copy_ceiling": bwd_bytes / bwd_t / 1e9 / copy_ceiling}
    # Algorithmic VALU work per element, in issue slots of a plain fp32 instruction (the exponential runs at a quarter
    # of that rate: 4 slots).  Backward: multiplier (1 + 4), state recompute (2), adjoint recurrence (2), gradient
    # terms (9) = 18 slots, 15 instructions, 24 flops (an FMA counts two).  Forward: multiplier (1 + 4), input term
    # (1), fold, state update and projection (3) = 9 slots, 6 instructions, 8 flops.  Scans, softplus and gate are not
    # counted.  Peak: 78.6e12 slots/s = the published 157.3 TFLOP/s at two flops per FMA.
    def alu(slots, instrs, flops, t_s, kernel):
        return {"bound": "alu", "kernel": kernel, "achieved": elements * slots / t_s / 1e12, "peak": VALU_PEAK_TLANEOPS,
                "unit": "T issue slots/s", "frac": elements * slots / t_s / 1e12 / VALU_PEAK_TLANEOPS,
                "slots_per_element": slots, "instructions_per_element": instrs,
                "achieved_TFLOPs": elements * flops / t_s / 1e12, "peak_TFLOPs_published": 157.3,
                "flops_per_element": flops}
    roofline_alu = alu(18.0, 15.0, 24.0, bwd_t, roofline["kernel"])
    roofline_alu_fwd = alu(9.0, 6.0, 8.0, fwd_t, "k_ss_fwd<bf16,N=16> (config 2 forward)")

    result = {
        "metric": "scan elements/s (B*L*D*N) fwd & bwd", "value": value, "unit": "elements/s",
        "n_gpus": 1, "steps": K, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "config 2: selective scan fwd+bwd, B=8 D=1536 N=16 L=2048, bf16 I/O, fp32 state, SiLU gate",
                   "io_dtype": "bf16", "disc": "zoh_s6", "elements_per_pass": elements},
        "ms_per_step_std": float(np.std(exp_means)), "experiments": len(exp_means),
        "fwd": {"us": fwd_t * 1e6, "elements_per_s": elements / fwd_t, "hbm_GBs": fwd_bytes / fwd_t / 1e9,
                "hbm_frac": fwd_bytes / fwd_t / 1e9 / HBM_PEAK_GBS},
        "bwd": {"us": bwd_t * 1e6, "elements_per_s": elements / bwd_t, "hbm_GBs": bwd_bytes / bwd_t / 1e9,
                "hbm_frac": bwd_bytes / bwd_t / 1e9 / HBM_PEAK_GBS},
        "roofline": roofline, "roofline_alu": roofline_alu, "roofline_alu_fwd": roofline_alu_fwd,
        "copy_ceiling_GBs": copy_ceiling,
    }
    for k in ("fwd", "bwd"):
        result[k]["frac_of_copy_ceiling"] = result[k]["hbm_GBs"] / copy_ceiling

    # ------------------------------------------------------------------ the other configs (context, not `value`)
    if not args.quick:
        result["other_configs"] = _other_configs(api, torch, dev)

    # ------------------------------------------------------------------ vector-ALU issue rates (on request)
    if args.alu_probe:
        result["alu_probe"] = _alu_probe()

    # ------------------------------------------------------------------ CPU baseline: the oracle as it stands
    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        t0 = time.perf_counter()
        oracle.selective_scan_fwd(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], Dskip=p["Dskip"],
                                  delta_bias=p["delta_bias"], z=p["z"])
        t1 = time.perf_counter()
        oracle.selective_scan_bwd(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], p["dy"], Dskip=p["Dskip"],
                                  delta_bias=p["delta_bias"], z=p["z"])
        t2 = time.perf_counter()
        result["cpu_baseline"] = {
            "value": 2 * elements / (t2 - t0), "unit": "elements/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "the whole config-2 workload, one fwd + one bwd pass of the fp64 C oracle (OpenMP over rows), "
                      "including its float64 input conversion",
            "fwd_s": t1 - t0, "bwd_s": t2 - t1}
    print(json.dumps(result))


def _time(torch, fn, reps, warm=3, warm_ms=25.0):
    """Average time of one call of fn over `reps` calls, after `warm` untimed calls and at least `warm_ms` of untimed
    work (a timing loop of a millisecond or two right after the host prepared inputs would otherwise be measured
    while the GPU's clocks are still coming up: 10 % slower on the shapes of this file)."""
    import time
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    while (time.perf_counter() - t0) * 1e3 < warm_ms:
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / reps


def _other_configs(api, torch, dev):
    """Configs 1, 3, 4 with seeded on-device random inputs of the stated distributions (timing only)."""
    out = {}
    g = torch.Generator(device=dev).manual_seed(1234)
    bf = torch.bfloat16

    def sel(B, D, N, L, gate):
        r = lambda *s: torch.randn(*s, device=dev, generator=g)
        return dict(u=r(B, D, L).to(bf), delta=r(B, D, L).to(bf),
                    A=-torch.exp(torch.rand(D, N, device=dev, generator=g) * 2 - 1),
                    Bm=r(B, L, N).to(bf), Cm=r(B, L, N).to(bf), Dskip=r(D),
                    delta_bias=torch.rand(D, device=dev, generator=g) * 2 - 4,
                    z=r(B, D, L).to(bf) if gate else None)

    # config 1: LTI complex-diagonal scan
    Bq, P, Lq = 4, 256, 4096
    lam = torch.polar(torch.rand(P, device=dev, generator=g) * 0.099 + 0.9,
                      torch.rand(P, device=dev, generator=g) * 6.2831853)
    v = torch.randn(Bq, Lq, P, dtype=torch.complex64, device=dev, generator=g) * 0.70710678
    x = torch.empty_like(v)
    ws = torch.empty(max(api.lrnnx_workspace_bytes(api.WS_LTI, Bq, P, 0, Lq, 0), 16), dtype=torch.uint8, device=dev)
    nb = 2 * Bq * Lq * P * 8
    for path in ("single_pass", "chunk_carry"):
        tt = _time(torch, lambda: api.lrnnx_lti_diag_scan(lam, v, out=x, workspace=ws, path=path), 50)
        out[f"c1_lti_{path}"] = {"us": tt * 1e6, "elements_per_s": Bq * Lq * P / tt, "hbm_GBs": nb / tt / 1e9,
                                 "hbm_frac": nb / tt / 1e9 / HBM_PEAK_GBS}

    # backward of the LTI scan at config 1's shape: reads gx and the saved states, writes dv
    gx = torch.randn(Bq, Lq, P, dtype=torch.complex64, device=dev, generator=g) * 0.70710678
    api.lrnnx_lti_diag_scan(lam, v, out=x, workspace=ws)
    dvq = torch.empty_like(v)
    wsb = torch.empty(max(api.lrnnx_workspace_bytes(api.WS_LTI_BWD, Bq, P, 0, Lq, 0), 16), dtype=torch.uint8, device=dev)
    tt = _time(torch, lambda: api.lrnnx_lti_diag_scan_bwd(lam, x, gx, out=dvq, workspace=wsb), 50)
    nb = 3 * Bq * Lq * P * 8
    out["c1_lti_bwd"] = {"us": tt * 1e6, "elements_per_s": Bq * Lq * P / tt, "hbm_GBs": nb / tt / 1e9,
                         "hbm_frac": nb / tt / 1e9 / HBM_PEAK_GBS}
    del gx, dvq, wsb

    # the same two calls on tensors well beyond the 256 MB Infinity Cache (B=8, P=1024, L=8192: 512 MiB each)
    Bl, Pl, Ll = 8, 1024, 8192
    laml = torch.polar(torch.rand(Pl, device=dev, generator=g) * 0.099 + 0.9,
                       torch.rand(Pl, device=dev, generator=g) * 6.2831853)
    vl = torch.randn(Bl, Ll, Pl, dtype=torch.complex64, device=dev, generator=g) * 0.70710678
    xl = torch.empty_like(vl)
    wsl = torch.empty(max(api.lrnnx_workspace_bytes(api.WS_LTI, Bl, Pl, 0, Ll, 0),
                          api.lrnnx_workspace_bytes(api.WS_LTI_BWD, Bl, Pl, 0, Ll, 0), 16), dtype=torch.uint8, device=dev)
    tt = _time(torch, lambda: api.lrnnx_lti_diag_scan(laml, vl, out=xl, workspace=wsl), 10)
    nb = 2 * Bl * Ll * Pl * 8
    out["lti_B8_P1024_L8192_fwd"] = {"us": tt * 1e6, "elements_per_s": Bl * Ll * Pl / tt, "hbm_GBs": nb / tt / 1e9,
                                     "hbm_frac": nb / tt / 1e9 / HBM_PEAK_GBS}
    gl = torch.randn(Bl, Ll, Pl, dtype=torch.complex64, device=dev, generator=g) * 0.70710678
    tt = _time(torch, lambda: api.lrnnx_lti_diag_scan_bwd(laml, xl, gl, out=gl, workspace=wsl), 10)
    nb = 3 * Bl * Ll * Pl * 8
    out["lti_B8_P1024_L8192_bwd"] = {"us": tt * 1e6, "elements_per_s": Bl * Ll * Pl / tt, "hbm_GBs": nb / tt / 1e9,
                                     "hbm_frac": nb / tt / 1e9 / HBM_PEAK_GBS}
    del vl, xl, gl, wsl

    # scan with caller-supplied (a_k, b_k): reads a and b, writes x
    for tag, dt, esz in (("real", torch.float32, 4), ("complex", torch.complex64, 8)):
        Bd, Pd, Ld = 8, 1024, 8192
        if dt == torch.float32:
            ad = torch.rand(Bd, Ld, Pd, device=dev, generator=g) * 0.5 + 0.5
            bd = torch.randn(Bd, Ld, Pd, device=dev, generator=g)
        else:
            ad = torch.polar(torch.rand(Bd, Ld, Pd, device=dev, generator=g) * 0.099 + 0.9,
                             torch.rand(Bd, Ld, Pd, device=dev, generator=g) * 6.2831853)
            bd = torch.randn(Bd, Ld, Pd, dtype=dt, device=dev, generator=g) * 0.70710678
        xd = torch.empty_like(bd)
        wsd = torch.empty(max(api.lrnnx_workspace_bytes(api.WS_DIAG, Bd, Pd, 0, Ld, api.C64 if esz == 8 else api.F32), 16),
                          dtype=torch.uint8, device=dev)
        tt = _time(torch, lambda: api.lrnnx_diag_scan(ad, bd, out=xd, workspace=wsd), 10)
        nb = 3 * Bd * Ld * Pd * esz
        out[f"diag_scan_{tag}_B8_P1024_L8192"] = {"us": tt * 1e6, "elements_per_s": Bd * Ld * Pd / tt,
                                                  "hbm_GBs": nb / tt / 1e9, "hbm_frac": nb / tt / 1e9 / HBM_PEAK_GBS}
        # its backward: reads a, x, gx, writes da, db
        wsb = torch.empty(max(api.lrnnx_workspace_bytes(api.WS_DIAG_BWD, Bd, Pd, 0, Ld, api.C64 if esz == 8 else api.F32), 16),
                          dtype=torch.uint8, device=dev)
        tt = _time(torch, lambda: api.lrnnx_diag_scan_bwd(ad, xd, bd, workspace=wsb), 10)   # bd stands in for gx
        nb = 5 * Bd * Ld * Pd * esz
        out[f"diag_scan_bwd_{tag}_B8_P1024_L8192"] = {"us": tt * 1e6, "elements_per_s": Bd * Ld * Pd / tt,
                                                      "hbm_GBs": nb / tt / 1e9, "hbm_frac": nb / tt / 1e9 / HBM_PEAK_GBS,
                                                      "note": "includes the allocation of da and db by the binding"}
        del ad, bd, xd, wsd, wsb

    # forward with a complex diagonal A and complex maps at config 2's shape (bf16 I/O)
    Bc, Dc, Nc, Lc = 8, 1536, 16, 2048
    tc = sel(Bc, Dc, Nc, Lc, True)
    Ac = torch.complex(tc["A"], torch.rand(Dc, Nc, device=dev, generator=g) * 20 - 10)
    Bmc = (torch.randn(Bc, Lc, Nc, 2, device=dev, generator=g) * 0.70710678).to(bf)
    Cmc = (torch.randn(Bc, Lc, Nc, 2, device=dev, generator=g) * 0.70710678).to(bf)
    yc = torch.empty_like(tc["u"])
    tt = _time(torch, lambda: api.lrnnx_selective_scan_fwd_complex(tc["u"], tc["delta"], Ac, Bmc, Cmc, Dskip=tc["Dskip"],
                                                                   delta_bias=tc["delta_bias"], z=tc["z"], out=yc), 10)
    nb = _selective_bytes(Bc, Dc, Nc, Lc, 2, True, False) + 2 * Bc * Lc * Nc * 2
    out["complex_fwd_B8_D1536_N16_L2048"] = {"us": tt * 1e6, "elements_per_s": Bc * Dc * Nc * Lc / tt,
                                             "hbm_GBs": nb / tt / 1e9, "hbm_frac": nb / tt / 1e9 / HBM_PEAK_GBS}
    # its backward with the forward's checkpoints: reads u, delta, z, dy, the maps and checkpoints; writes du, ddelta, dz
    # and the float32 complex dBm, dCm
    _, ckc = api.lrnnx_selective_scan_fwd_complex(tc["u"], tc["delta"], Ac, Bmc, Cmc, Dskip=tc["Dskip"],
                                                  delta_bias=tc["delta_bias"], z=tc["z"], out=yc, return_ckpt=True)
    dyc = torch.randn(Bc, Dc, Lc, device=dev, generator=g).to(bf)
    outs_c = {}
    tt = _time(torch, lambda: outs_c.update(api.lrnnx_selective_scan_bwd_complex(
        tc["u"], tc["delta"], Ac, Bmc, Cmc, dyc, Dskip=tc["Dskip"], delta_bias=tc["delta_bias"], z=tc["z"], ckpt=ckc,
        outs=outs_c)), 10)
    nb = 7 * Bc * Dc * Lc * 2 + 2 * Bc * Lc * Nc * 4 + 2 * Bc * Lc * Nc * 8 + Bc * Dc * (Lc // 256) * Nc * 8
    out["complex_bwd_B8_D1536_N16_L2048"] = {"us": tt * 1e6, "elements_per_s": Bc * Dc * Nc * Lc / tt,
                                             "hbm_GBs": nb / tt / 1e9, "hbm_frac": nb / tt / 1e9 / HBM_PEAK_GBS}
    del tc, Ac, Bmc, Cmc, yc, ckc, dyc, outs_c

    # single-token step (generation): state [B,D,N] read and written once per token
    Bs, Ds, Ns = 64, 1536, 16
    ts = sel(Bs, Ds, Ns, 1, True)
    xs = torch.randn(Bs, Ds, Ns, device=dev, generator=g)
    ys = torch.empty((Bs, Ds), dtype=bf, device=dev)
    us, ds_, zs = ts["u"][:, :, 0], ts["delta"][:, :, 0], ts["z"][:, :, 0]
    Bs1, Cs1 = ts["Bm"][:, 0].contiguous(), ts["Cm"][:, 0].contiguous()
    tt = _time(torch, lambda: api.lrnnx_selective_step(xs, us, ds_, ts["A"], Bs1, Cs1, Dskip=ts["Dskip"],
                                                       delta_bias=ts["delta_bias"], z=zs, out=ys), 200)
    nb = 2 * Bs * Ds * Ns * 4 + 4 * Bs * Ds * 2
    out["step_B64_D1536_N16"] = {"us": tt * 1e6, "elements_per_s": Bs * Ds * Ns / tt, "hbm_GBs": nb / tt / 1e9,
                                 "hbm_frac": nb / tt / 1e9 / HBM_PEAK_GBS,
                                 "note": "includes the Python call overhead of one launch per token"}

    # the same step as a generation loop of 64 tokens captured once in a HIP graph and replayed (Sec. 4.2 of the
    # paper measures generation this way): per-token time without the per-call host overhead
    Tg = 64
    tg = sel(Bs, Ds, Ns, Tg, True)
    ug, dg, zg = (tg[k].permute(2, 0, 1).contiguous() for k in ("u", "delta", "z"))         # [T,B,D]
    Bg, Cg = tg["Bm"].permute(1, 0, 2).contiguous(), tg["Cm"].permute(1, 0, 2).contiguous()  # [T,B,N]
    yg = torch.empty((Tg, Bs, Ds), dtype=bf, device=dev)

    def gen_loop():
        for t in range(Tg):
            api.lrnnx_selective_step(xs, ug[t], dg[t], ts["A"], Bg[t], Cg[t], Dskip=ts["Dskip"],
                                     delta_bias=ts["delta_bias"], z=zg[t], out=yg[t])
    gen_loop()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        gen_loop()
    tt = _time(torch, graph.replay, 20) / Tg
    out["step_B64_D1536_N16_graph"] = {"us": tt * 1e6, "elements_per_s": Bs * Ds * Ns / tt, "hbm_GBs": nb / tt / 1e9,
                                       "hbm_frac": nb / tt / 1e9 / HBM_PEAK_GBS,
                                       "note": "per token, 64 step calls replayed from one HIP graph"}
    del graph

    # packed variable-length batch of config 2's total size: 8 * 2048 steps as 24 sequences of mixed lengths
    lens = [3000, 1500, 1000, 2048, 512, 512, 700, 324, 100, 100, 60, 40, 2200, 1800, 32, 8, 448, 900, 300, 300, 200, 100,
            100, 100]
    assert sum(lens) == 16384
    Dp, Np, Lp = 1536, 16, 16384
    tp = sel(1, Dp, Np, Lp, True)
    cu = torch.tensor([0] + list(__import__("itertools").accumulate(lens)), dtype=torch.int64, device=dev)
    pk = {k: (v[0] if k in ("u", "delta", "z", "Bm", "Cm") else v) for k, v in tp.items()}
    dyp = torch.randn(Dp, Lp, device=dev, generator=g).to(bf)
    yp = torch.empty_like(pk["u"])
    ckp = torch.empty((Dp, Lp // api.lrnnx_ckpt_interval() + len(lens), Np), device=dev)
    outs_p = {k: torch.empty_like(pk["u"]) for k in ("du", "ddelta", "dz")}
    outs_p.update(dA=torch.empty((Dp, Np), device=dev), dBm=torch.empty((Lp, Np), device=dev),
                  dCm=torch.empty((Lp, Np), device=dev), dD=torch.empty(Dp, device=dev), dbias=torch.empty(Dp, device=dev))
    tf = _time(torch, lambda: api.lrnnx_selective_scan_fwd(**pk, cu_seqlens=cu, out=yp, ckpt_out=ckp), 10)
    tb = _time(torch, lambda: api.lrnnx_selective_scan_bwd(**pk, dy=dyp, cu_seqlens=cu, ckpt=ckp, outs=outs_p,
                                                           max_seqlen=max(lens)), 10)
    out["packed_24seq_D1536_L16384"] = {"fwd_us": tf * 1e6, "bwd_us": tb * 1e6,
                                        "elements_per_s": 2 * Dp * Np * Lp / (tf + tb),
                                        "note": "same total size as config 2; the backward call is given max_seqlen"}
    # the same steps as 8 sequences of 2048 (config 2 itself, packed): what the packed mode costs on equal lengths
    cu8 = torch.arange(0, Lp + 1, 2048, dtype=torch.int64, device=dev)
    ckp8 = torch.empty((Dp, Lp // api.lrnnx_ckpt_interval() + 8, Np), device=dev)
    tf = _time(torch, lambda: api.lrnnx_selective_scan_fwd(**pk, cu_seqlens=cu8, out=yp, ckpt_out=ckp8), 10)
    tb = _time(torch, lambda: api.lrnnx_selective_scan_bwd(**pk, dy=dyp, cu_seqlens=cu8, ckpt=ckp8, outs=outs_p,
                                                           max_seqlen=2048), 10)
    out["packed_8x2048_D1536"] = {"fwd_us": tf * 1e6, "bwd_us": tb * 1e6,
                                  "elements_per_s": 2 * Dp * Np * Lp / (tf + tb),
                                  "note": "config 2 as a packed batch; the backward call is given max_seqlen"}
    del tp, pk, dyp, yp, ckp, ckp8, outs_p

    # config 3: long-sequence forward, both paths
    B3, D3, N3, L3 = 1, 2048, 16, 65536
    t3 = sel(B3, D3, N3, L3, False)
    y3 = torch.empty_like(t3["u"])
    ws3 = torch.empty(max(api.lrnnx_workspace_bytes(api.WS_FWD, B3, D3, N3, L3, api.BF16), 16), dtype=torch.uint8, device=dev)
    nb = _selective_bytes(B3, D3, N3, L3, 2, False, False)
    for path in ("single_pass", "chunk_carry"):
        tt = _time(torch, lambda: api.lrnnx_selective_scan_fwd(**t3, path=path, out=y3, workspace=ws3), 5)
        out[f"c3_fwd_{path}"] = {"us": tt * 1e6, "elements_per_s": B3 * D3 * N3 * L3 / tt, "hbm_GBs": nb / tt / 1e9,
                                 "hbm_frac": nb / tt / 1e9 / HBM_PEAK_GBS}
    # the backward pass at config 3's shape (one batch entry: few rows, long sequence), single pass and chunked
    dy3 = torch.randn(B3, D3, L3, device=dev, generator=g).to(bf)
    _, ck3 = api.lrnnx_selective_scan_fwd(**t3, out=y3, workspace=ws3, return_ckpt=True)
    outs3 = {}
    nb = _selective_bytes(B3, D3, N3, L3, 2, False, True) + ck3.numel() * 4
    for path in ("single_pass", "chunk_carry"):
        tt = _time(torch, lambda: outs3.update(api.lrnnx_selective_scan_bwd(**t3, dy=dy3, ckpt=ck3, outs=outs3, path=path)), 3,
                   warm=2)
        out[f"c3_shape_bwd_{path}"] = {"us": tt * 1e6, "elements_per_s": B3 * D3 * N3 * L3 / tt, "hbm_GBs": nb / tt / 1e9,
                                       "hbm_frac": nb / tt / 1e9 / HBM_PEAK_GBS,
                                       "chunks": int(api.lib().lrnnx_selective_scan_bwd_chunks(B3, D3, N3, L3, 1, api.PATH[path], 0))}
    del t3, y3, ws3, dy3, ck3, outs3

    # config 2's shape with float32 I/O (the float32 kernels differ: no Bm/Cm row prefetch in the forward pass)
    Bf, Df, Nf, Lf = 8, 1536, 16, 2048
    tf32 = {k: (v.float() if (v is not None and v.dtype == bf) else v) for k, v in sel(Bf, Df, Nf, Lf, True).items()}
    dyf = torch.randn(Bf, Df, Lf, device=dev, generator=g)
    yf = torch.empty_like(tf32["u"])
    _, ckf = api.lrnnx_selective_scan_fwd(**tf32, out=yf, return_ckpt=True)
    outs_f = {}
    tt = _time(torch, lambda: api.lrnnx_selective_scan_fwd(**tf32, out=yf, ckpt_out=ckf), 10)
    nb = _selective_bytes(Bf, Df, Nf, Lf, 4, True, False) + ckf.numel() * 4
    out["c2_shape_f32io_fwd"] = {"us": tt * 1e6, "elements_per_s": Bf * Df * Nf * Lf / tt, "hbm_GBs": nb / tt / 1e9,
                                 "hbm_frac": nb / tt / 1e9 / HBM_PEAK_GBS}
    tt = _time(torch, lambda: outs_f.update(api.lrnnx_selective_scan_bwd(**tf32, dy=dyf, ckpt=ckf, outs=outs_f)), 10)
    nb = _selective_bytes(Bf, Df, Nf, Lf, 4, True, True) + ckf.numel() * 4
    out["c2_shape_f32io_bwd"] = {"us": tt * 1e6, "elements_per_s": Bf * Df * Nf * Lf / tt, "hbm_GBs": nb / tt / 1e9,
                                 "hbm_frac": nb / tt / 1e9 / HBM_PEAK_GBS}
    del tf32, dyf, yf, ckf, outs_f

    # config 2's shape under the other discretisation schemes (Sec. 3): exact zero-order hold, bilinear, dirac
    td = sel(Bf, Df, Nf, Lf, True)
    dyd = torch.randn(Bf, Df, Lf, device=dev, generator=g).to(bf)
    yd = torch.empty_like(td["u"])
    for disc in ("zoh", "bilinear", "dirac"):
        _, ckd = api.lrnnx_selective_scan_fwd(**td, out=yd, return_ckpt=True, disc=disc)
        outs_d = {}
        tf_ = _time(torch, lambda: api.lrnnx_selective_scan_fwd(**td, out=yd, ckpt_out=ckd, disc=disc), 10)
        tb_ = _time(torch, lambda: outs_d.update(api.lrnnx_selective_scan_bwd(**td, dy=dyd, ckpt=ckd, outs=outs_d, disc=disc)), 10)
        out[f"c2_shape_{disc}"] = {"fwd_us": tf_ * 1e6, "bwd_us": tb_ * 1e6,
                                   "elements_per_s": 2 * Bf * Df * Nf * Lf / (tf_ + tb_)}
        del ckd, outs_d
    del td, dyd, yd

    # config 4: backward only (checkpoints from one untimed forward)
    B4, D4, N4, L4 = 16, 2560, 16, 4096
    t4 = sel(B4, D4, N4, L4, True)
    dy4 = torch.randn(B4, D4, L4, device=dev, generator=g).to(bf)
    _, ck4 = api.lrnnx_selective_scan_fwd(**t4, return_ckpt=True)
    outs = {k: torch.empty_like(t4["u"]) for k in ("du", "ddelta", "dz")}
    outs.update(dA=torch.empty((D4, N4), device=dev), dBm=torch.empty((B4, L4, N4), device=dev),
                dCm=torch.empty((B4, L4, N4), device=dev), dD=torch.empty(D4, device=dev),
                dbias=torch.empty(D4, device=dev))
    tt = _time(torch, lambda: api.lrnnx_selective_scan_bwd(**t4, dy=dy4, ckpt=ck4, outs=outs), 5)
    nb = _selective_bytes(B4, D4, N4, L4, 2, True, True) + ck4.numel() * 4
    out["c4_bwd"] = {"us": tt * 1e6, "elements_per_s": B4 * D4 * N4 * L4 / tt, "hbm_GBs": nb / tt / 1e9,
                     "hbm_frac": nb / tt / 1e9 / HBM_PEAK_GBS}
    y4 = torch.empty_like(t4["u"])
    tt = _time(torch, lambda: api.lrnnx_selective_scan_fwd(**t4, out=y4), 5)
    nb = _selective_bytes(B4, D4, N4, L4, 2, True, False)
    out["c4_fwd"] = {"us": tt * 1e6, "elements_per_s": B4 * D4 * N4 * L4 / tt, "hbm_GBs": nb / tt / 1e9,
                     "hbm_frac": nb / tt / 1e9 / HBM_PEAK_GBS}
    return out


if __name__ == "__main__":
    main()
