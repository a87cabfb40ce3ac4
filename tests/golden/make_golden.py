"""Writes the stored expected values under tests/golden/ by calling only oracle/.

The paper prints no numeric worked example (all its results are figures), so
these files are regression anchors for the oracle, not values from the paper:
config-0 shaped selective scan (Eq. 2, Sec. 2.2; S6 row of Table 1) and a small
LTI complex-diagonal scan (Sec. 2.2.1).  Run:  python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle  # noqa: E402
from paper_2602_08810_amd import workloads  # noqa: E402


def main():
    p, cfg = workloads.make("c0")
    y, x_last = oracle.selective_scan_fwd(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], Dskip=p["Dskip"],
                                          delta_bias=p["delta_bias"], disc="zoh_s6", delta_softplus=True)
    g = oracle.selective_scan_bwd(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], p["dy"], Dskip=p["Dskip"],
                                  delta_bias=p["delta_bias"], disc="zoh_s6", delta_softplus=True)
    with open(os.path.join(HERE, "c0_selective_fp64.txt"), "w") as f:
        f.write("# config c0 (B=1,D=16,N=4,L=256, seed 0), oracle fp64; written by make_golden.py\n")
        f.write("# y[0,d,255] for d=0..15\n" + " ".join(f"{v:.17e}" for v in y[0, :, 255]) + "\n")
        f.write("# x_last[0,0,:]\n" + " ".join(f"{v:.17e}" for v in x_last[0, 0]) + "\n")
        f.write("# dA[0,:]\n" + " ".join(f"{v:.17e}" for v in g["dA"][0]) + "\n")
        f.write("# sum(du), sum(ddelta), sum(dBm), sum(dCm)\n" +
                " ".join(f"{float(np.sum(g[k])):.17e}" for k in ("du", "ddelta", "dBm", "dCm")) + "\n")
    q, _ = workloads.make("c1", B=1, P=4, L=64)
    x = oracle.lti_diag_scan(q["lam"], q["v"])
    with open(os.path.join(HERE, "c1_small_lti_fp64.txt"), "w") as f:
        f.write("# config c1 shrunk to B=1,P=4,L=64 (seed 1), oracle complex128; written by make_golden.py\n")
        f.write("# re,im of x[0,63,p] for p=0..3\n" +
                " ".join(f"{v.real:.17e} {v.imag:.17e}" for v in x[0, 63]) + "\n")


if __name__ == "__main__":
    main()
