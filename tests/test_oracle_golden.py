"""The oracle reproduces its stored anchors (tests/golden/, written by make_golden.py from oracle/ alone)."""
import os

import numpy as np

from paper_2602_08810_amd import workloads

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _rows(name):
    with open(os.path.join(GOLD, name)) as f:
        return [np.array([float(t) for t in ln.split()]) for ln in f if not ln.startswith("#")]


def test_c0_selective_anchor(oracle):
    p, _ = workloads.make("c0")
    y, x_last = oracle.selective_scan_fwd(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], Dskip=p["Dskip"],
                                          delta_bias=p["delta_bias"])
    g = oracle.selective_scan_bwd(p["u"], p["delta"], p["A"], p["Bm"], p["Cm"], p["dy"], Dskip=p["Dskip"],
                                  delta_bias=p["delta_bias"])
    rows = _rows("c0_selective_fp64.txt")
    np.testing.assert_allclose(y[0, :, 255], rows[0], rtol=1e-13)
    np.testing.assert_allclose(x_last[0, 0], rows[1], rtol=1e-13)
    np.testing.assert_allclose(g["dA"][0], rows[2], rtol=1e-12)
    np.testing.assert_allclose([np.sum(g[k]) for k in ("du", "ddelta", "dBm", "dCm")], rows[3], rtol=1e-10)


def test_c1_small_lti_anchor(oracle):
    q, _ = workloads.make("c1", B=1, P=4, L=64)
    x = oracle.lti_diag_scan(q["lam"], q["v"])
    flat = np.stack([x[0, 63].real, x[0, 63].imag], axis=1).ravel()
    np.testing.assert_allclose(flat, _rows("c1_small_lti_fp64.txt")[0], rtol=1e-13)


def test_workloads_are_seeded_and_bf16_exact():
    a, _ = workloads.make("c2", B=1, D=4, L=32)
    b, _ = workloads.make("c2", B=1, D=4, L=32)
    for k in a:
        if a[k] is not None:
            np.testing.assert_array_equal(a[k], b[k])
    for k in ("u", "delta", "z", "dy", "Bm", "Cm"):
        assert np.all((a[k].view(np.uint32) & 0xFFFF) == 0)          # representable in bf16
    assert np.all(a["A"] < 0) and np.all(a["delta_bias"] <= -2) and np.all(a["delta_bias"] >= -4)
    r = workloads.round_to_bf16(np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.00390625], dtype=np.float32))
    np.testing.assert_array_equal(r, np.array([1.0, 1.015625, 1.0], dtype=np.float32))  # ties to even
