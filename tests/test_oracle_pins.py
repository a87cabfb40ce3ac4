"""Pins for the fp64 CPU oracle: it is checked against things other than itself.

The paper prints no worked numeric example (its results are figures), so the
oracle is pinned to what the mathematics of Eq. 2 (Sec. 2.2) and of the
discretisations named in Sec. 3 fixes: brute-force unrolled sums, the LTI
convolution closed form, impulse responses, SciPy's lfilter and cont2discrete,
the textbook exactness of zero-order hold on a step input, central finite
differences, the adjoint dot test, and structural invariants.
"""
import numpy as np
import pytest
import scipy.signal

DISCS = ["zoh_s6", "zoh", "bilinear", "dirac"]


def _rand_problem(rng, B=2, D=3, N=4, L=9, gate=True, bias=True, x0=True, skip=True):
    p = dict(
        u=rng.standard_normal((B, D, L)),
        delta=rng.standard_normal((B, D, L)),
        A=-np.exp(rng.uniform(-1, 1, (D, N))),
        Bm=rng.standard_normal((B, L, N)),
        Cm=rng.standard_normal((B, L, N)),
        Dskip=rng.standard_normal(D) if skip else None,
        delta_bias=rng.uniform(-2, 0, D) if bias else None,
        z=rng.standard_normal((B, D, L)) if gate else None,
        x0=rng.standard_normal((B, D, N)) if x0 else None,
    )
    return p


def _disc_py(disc, dt, A):
    """Independent restatement of the four schemes with numpy scalars (pinned itself by cont2discrete below)."""
    if disc == "bilinear":
        return (1 + dt * A / 2) / (1 - dt * A / 2), dt / (1 - dt * A / 2)
    a = np.exp(dt * A)
    return a, {"zoh_s6": dt, "zoh": (a - 1) / A, "dirac": 1.0}[disc]


# ----------------------------------------------------------------------------- scalar pieces

@pytest.mark.parametrize("s", [-40.0, -6.0, -1.0, 0.0, 0.3, 5.0, 30.0, 800.0])
def test_softplus_matches_logaddexp(oracle, s):
    assert oracle.softplus(s) == pytest.approx(np.logaddexp(0.0, s), rel=1e-14, abs=1e-300)


@pytest.mark.parametrize("dt,A", [(0.05, -1.3), (0.7, -0.4), (1e-3, -2.5)])
def test_zoh_and_bilinear_match_scipy_cont2discrete(oracle, dt, A):
    """Ad, Bd of the scalar system x' = A x + 1*u from SciPy equal (a, g) of the oracle (Sec. 3 schemes)."""
    sys_c = (np.array([[A]]), np.array([[1.0]]), np.array([[1.0]]), np.array([[0.0]]))
    Ad, Bd, *_ = scipy.signal.cont2discrete(sys_c, dt, method="zoh")
    a, g, *_ = oracle.disc_terms("zoh", dt, A)
    assert a == pytest.approx(Ad[0, 0], rel=1e-13) and g == pytest.approx(Bd[0, 0], rel=1e-12)
    Ad, Bd, *_ = scipy.signal.cont2discrete(sys_c, dt, method="bilinear")
    a, g, *_ = oracle.disc_terms("bilinear", dt, A)
    assert a == pytest.approx(Ad[0, 0], rel=1e-13) and g == pytest.approx(Bd[0, 0], rel=1e-12)


def test_zoh_identity_and_other_input_gains(oracle):
    """Abar = exp(dt A) for the three exponential schemes; S6 gain is dt, dirac gain is 1."""
    for dt, A in [(0.2, -0.9), (1.1, -2.0)]:
        for disc in ["zoh_s6", "zoh", "dirac"]:
            assert oracle.disc_terms(disc, dt, A)[0] == pytest.approx(np.exp(dt * A), rel=1e-15)
        assert oracle.disc_terms("zoh_s6", dt, A)[1] == dt
        assert oracle.disc_terms("dirac", dt, A)[1] == 1.0


def test_bilinear_stability_and_order(oracle):
    """|a| < 1 iff A < 0, and a = exp(dt A) + O(dt^3)."""
    for A in [-3.0, -0.1]:
        for dt in [0.01, 1.0, 50.0]:
            assert abs(oracle.disc_terms("bilinear", dt, A)[0]) < 1
    assert abs(oracle.disc_terms("bilinear", 0.5, 0.7)[0]) > 1
    e1 = abs(oracle.disc_terms("bilinear", 1e-2, -1.0)[0] - np.exp(-1e-2))
    e2 = abs(oracle.disc_terms("bilinear", 5e-3, -1.0)[0] - np.exp(-5e-3))
    assert e1 / e2 == pytest.approx(8.0, rel=0.05)


@pytest.mark.parametrize("disc", DISCS)
def test_disc_partials_by_finite_differences(oracle, disc):
    dt, A, h = 0.37, -1.2, 1e-6
    a, g, a_t, a_A, g_t, g_A = oracle.disc_terms(disc, dt, A)
    ap, gp, *_ = oracle.disc_terms(disc, dt + h, A)
    am, gm, *_ = oracle.disc_terms(disc, dt - h, A)
    assert a_t == pytest.approx((ap - am) / (2 * h), rel=1e-7, abs=1e-9)
    assert g_t == pytest.approx((gp - gm) / (2 * h), rel=1e-7, abs=1e-9)
    ap, gp, *_ = oracle.disc_terms(disc, dt, A + h)
    am, gm, *_ = oracle.disc_terms(disc, dt, A - h)
    assert a_A == pytest.approx((ap - am) / (2 * h), rel=1e-7, abs=1e-9)
    assert g_A == pytest.approx((gp - gm) / (2 * h), rel=1e-7, abs=1e-9)


# ----------------------------------------------------------------------------- forward recurrence

@pytest.mark.parametrize("disc", DISCS)
@pytest.mark.parametrize("softplus", [True, False])
def test_fwd_matches_bruteforce_unrolled_sum(oracle, disc, softplus):
    """x_k = sum_{j<=k} (prod_{i=j+1..k} a_i) b_j + (prod_{i<=k} a_i) x0, written as an O(L^2) double sum."""
    rng = np.random.default_rng(11)
    p = _rand_problem(rng, B=2, D=2, N=3, L=7)
    if not softplus:
        p["delta"] = np.abs(p["delta"]) + 0.1
        p["delta_bias"] = None
    y, x_last, xs = oracle.selective_scan_fwd(**p, disc=disc, delta_softplus=softplus, return_states=True)
    B, D, L = p["u"].shape
    N = p["A"].shape[1]
    for b in range(B):
        for d in range(D):
            s = p["delta"][b, d] + (p["delta_bias"][d] if p["delta_bias"] is not None else 0.0)
            dt = np.logaddexp(0, s) if softplus else s
            for n in range(N):
                a = np.empty(L); bb = np.empty(L)
                for l in range(L):
                    a[l], g = _disc_py(disc, dt[l], p["A"][d, n])
                    bb[l] = g * p["Bm"][b, l, n] * p["u"][b, d, l]
                for k in range(L):
                    tot = np.prod(a[: k + 1]) * p["x0"][b, d, n]
                    for j in range(k + 1):
                        tot += np.prod(a[j + 1: k + 1]) * bb[j]
                    assert xs[b, d, k, n] == pytest.approx(tot, rel=1e-11, abs=1e-12)
            for k in range(L):
                ypre = np.dot(p["Cm"][b, k], xs[b, d, k]) + p["Dskip"][d] * p["u"][b, d, k]
                zz = p["z"][b, d, k]
                assert y[b, d, k] == pytest.approx(ypre * zz / (1 + np.exp(-zz)), rel=1e-11, abs=1e-12)
            np.testing.assert_allclose(x_last[b, d], xs[b, d, L - 1], rtol=0, atol=0)


@pytest.mark.parametrize("disc", DISCS)
def test_lti_special_case_is_a_convolution(oracle, disc):
    """Constant delta, B, C  =>  y = K * u with K_k = C Abar^k Bbar (+ D at k = 0)."""
    rng = np.random.default_rng(5)
    Bsz, D, N, L = 1, 2, 3, 24
    A = -np.exp(rng.uniform(-1, 1, (D, N)))
    dt = np.array([0.3, 0.8])
    Bv, Cv = rng.standard_normal(N), rng.standard_normal(N)
    Dskip = rng.standard_normal(D)
    u = rng.standard_normal((Bsz, D, L))
    delta = np.broadcast_to(dt[None, :, None], (Bsz, D, L)).copy()
    Bm = np.broadcast_to(Bv, (Bsz, L, N)).copy()
    Cm = np.broadcast_to(Cv, (Bsz, L, N)).copy()
    y, _ = oracle.selective_scan_fwd(u, delta, A, Bm, Cm, Dskip=Dskip, disc=disc, delta_softplus=False)
    for d in range(D):
        K = np.zeros(L)
        for n in range(N):
            a, g = _disc_py(disc, dt[d], A[d, n])
            K += Cv[n] * a ** np.arange(L) * g * Bv[n]
        K[0] += Dskip[d]
        np.testing.assert_allclose(y[0, d], np.convolve(u[0, d], K)[:L], rtol=1e-11, atol=1e-12)
    # impulse input => y_k = K_k
    u_imp = np.zeros((Bsz, D, L)); u_imp[:, :, 0] = 1.0
    y_imp, _ = oracle.selective_scan_fwd(u_imp, delta, A, Bm, Cm, Dskip=Dskip, disc=disc, delta_softplus=False)
    for d in range(D):
        K = sum(Cv[n] * _disc_py(disc, dt[d], A[d, n])[0] ** np.arange(L) * _disc_py(disc, dt[d], A[d, n])[1] * Bv[n]
                for n in range(N))
        K[0] += Dskip[d]
        np.testing.assert_allclose(y_imp[0, d], K, rtol=1e-11, atol=1e-13)


def test_exact_zoh_step_response_is_the_continuous_solution(oracle):
    """u = 1 held constant: exact ZOH reproduces x(t) = (e^{tA} - 1)/A * B at t = k*dt; the S6 form is off by dt*A/(e^{dt A}-1)."""
    A, dt, L, Bc = -0.7, 0.25, 40, 1.3
    u = np.ones((1, 1, L)); delta = np.full((1, 1, L), dt)
    Bm = np.full((1, L, 1), Bc); Cm = np.ones((1, L, 1))
    y, _ = oracle.selective_scan_fwd(u, delta, np.array([[A]]), Bm, Cm, disc="zoh", delta_softplus=False)
    t = dt * np.arange(1, L + 1)
    np.testing.assert_allclose(y[0, 0], np.expm1(t * A) / A * Bc, rtol=1e-12)
    y6, _ = oracle.selective_scan_fwd(u, delta, np.array([[A]]), Bm, Cm, disc="zoh_s6", delta_softplus=False)
    np.testing.assert_allclose(y6[0, 0] / y[0, 0], dt * A / np.expm1(dt * A), rtol=1e-12)


def test_linearity_causality_gate_and_chaining(oracle):
    rng = np.random.default_rng(3)
    p = _rand_problem(rng, B=2, D=3, N=4, L=20, gate=False, x0=False)
    y1, _ = oracle.selective_scan_fwd(**p)
    u2 = rng.standard_normal(p["u"].shape)
    y2, _ = oracle.selective_scan_fwd(**{**p, "u": u2})
    y12, _ = oracle.selective_scan_fwd(**{**p, "u": 2.0 * p["u"] - 3.0 * u2})
    np.testing.assert_allclose(y12, 2.0 * y1 - 3.0 * y2, rtol=1e-11, atol=1e-12)       # superposition in u
    pc = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in p.items()}
    pc["u"][:, :, 12:] += 5.0; pc["delta"][:, :, 12:] -= 1.0; pc["Bm"][:, 12:] *= 2; pc["Cm"][:, 12:] *= -1
    yc, _ = oracle.selective_scan_fwd(**pc)
    np.testing.assert_array_equal(yc[:, :, :12], y1[:, :, :12])                          # causality
    z = rng.standard_normal(p["u"].shape)
    yg, _ = oracle.selective_scan_fwd(**{**p, "z": z})
    np.testing.assert_allclose(yg, y1 * z / (1 + np.exp(-z)), rtol=1e-13)                # gate identity
    # scan(L1+L2) == scan(L1) then scan(L2, x0 = x_last)
    L1 = 7
    ya, xa = oracle.selective_scan_fwd(p["u"][:, :, :L1], p["delta"][:, :, :L1], p["A"], p["Bm"][:, :L1],
                                       p["Cm"][:, :L1], Dskip=p["Dskip"], delta_bias=p["delta_bias"])
    yb, xb = oracle.selective_scan_fwd(p["u"][:, :, L1:], p["delta"][:, :, L1:], p["A"], p["Bm"][:, L1:],
                                       p["Cm"][:, L1:], Dskip=p["Dskip"], delta_bias=p["delta_bias"], x0=xa)
    yfull, xfull = oracle.selective_scan_fwd(**p)
    np.testing.assert_allclose(np.concatenate([ya, yb], axis=2), yfull, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(xb, xfull, rtol=1e-12, atol=1e-13)


# ----------------------------------------------------------------------------- backward

def _loss(oracle, p, dy, disc, softplus):
    y, _ = oracle.selective_scan_fwd(**p, disc=disc, delta_softplus=softplus)
    return float(np.sum(dy * y))


@pytest.mark.parametrize("disc", DISCS)
@pytest.mark.parametrize("softplus,gate", [(True, True), (False, False)])
def test_bwd_matches_central_finite_differences(oracle, disc, softplus, gate):
    rng = np.random.default_rng(7)
    p = _rand_problem(rng, B=2, D=2, N=3, L=6, gate=gate)
    if not softplus:                      # caller-supplied positive step sizes; bias still added
        p["delta"] = np.abs(p["delta"]) + 2.2
    dy = rng.standard_normal(p["u"].shape)
    g = oracle.selective_scan_bwd(**p, dy=dy, disc=disc, delta_softplus=softplus)
    names = {"u": "du", "delta": "ddelta", "A": "dA", "Bm": "dBm", "Cm": "dCm", "Dskip": "dD",
             "delta_bias": "dbias", "z": "dz", "x0": "dx0"}
    h = 1e-6
    for key, gname in names.items():
        if p[key] is None:
            continue
        base = p[key]
        num = np.zeros_like(base)
        it = np.nditer(base, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            pp = dict(p); arr = base.copy(); arr[idx] += h; pp[key] = arr
            pm = dict(p); arr2 = base.copy(); arr2[idx] -= h; pm[key] = arr2
            num[idx] = (_loss(oracle, pp, dy, disc, softplus) - _loss(oracle, pm, dy, disc, softplus)) / (2 * h)
        scale = max(1.0, np.abs(num).max())
        np.testing.assert_allclose(g[gname], num, rtol=0, atol=2e-7 * scale, err_msg=f"{gname} ({disc})")


def test_bwd_adjoint_dot_test(oracle):
    """y is linear in u for fixed delta, B, C, z:  <dy, J du> == <J^T dy, du>."""
    rng = np.random.default_rng(9)
    p = _rand_problem(rng, B=2, D=3, N=4, L=33, x0=False)
    dy = rng.standard_normal(p["u"].shape)
    v = rng.standard_normal(p["u"].shape)
    Jv, _ = oracle.selective_scan_fwd(**{**p, "u": v})
    g = oracle.selective_scan_bwd(**p, dy=dy)
    assert np.sum(dy * Jv) == pytest.approx(np.sum(g["du"] * v), rel=1e-11)


def test_bwd_optional_outputs_absent(oracle):
    rng = np.random.default_rng(2)
    p = _rand_problem(rng, gate=False, bias=False, x0=False, skip=False)
    g = oracle.selective_scan_bwd(**p, dy=rng.standard_normal(p["u"].shape))
    assert g["dz"] is None and g["dD"] is None and g["dbias"] is None
    assert np.all(np.isfinite(g["du"])) and np.all(np.isfinite(g["dBm"]))


# ----------------------------------------------------------------------------- LTI complex-diagonal scan

def test_lti_scan_matches_scipy_lfilter_and_powers(oracle):
    rng = np.random.default_rng(4)
    Bsz, L, P = 2, 50, 5
    lam = rng.uniform(0.9, 0.999, P) * np.exp(1j * rng.uniform(0, 2 * np.pi, P))
    v = (rng.standard_normal((Bsz, L, P)) + 1j * rng.standard_normal((Bsz, L, P))) / np.sqrt(2)
    x = oracle.lti_diag_scan(lam, v)
    for b in range(Bsz):
        for p_ in range(P):
            ref = scipy.signal.lfilter([1.0], [1.0, -lam[p_]], v[b, :, p_])
            np.testing.assert_allclose(x[b, :, p_], ref, rtol=1e-12, atol=1e-13)
    imp = np.zeros((1, L, P), dtype=complex); imp[0, 0] = 1.0
    xi = oracle.lti_diag_scan(lam, imp)
    np.testing.assert_allclose(xi[0], lam[None, :] ** np.arange(L)[:, None], rtol=1e-12)   # impulse => lambda^k
    x0 = rng.standard_normal((Bsz, P)) + 1j * rng.standard_normal((Bsz, P))
    xz = oracle.lti_diag_scan(lam, np.zeros_like(v), x0=x0)
    np.testing.assert_allclose(xz, x0[:, None, :] * lam[None, None, :] ** np.arange(1, L + 1)[None, :, None], rtol=1e-12)


def test_lti_scan_agrees_with_selective_scan_on_a_real_pole(oracle):
    """A real lambda with dirac input map is the same recurrence through both oracle entry points."""
    rng = np.random.default_rng(8)
    L = 30
    A, dt = -0.5, 0.3
    lam = np.array([np.exp(A * dt) + 0j])
    vv = rng.standard_normal(L)
    x = oracle.lti_diag_scan(lam, vv[None, :, None] + 0j)
    y, _ = oracle.selective_scan_fwd(vv[None, None, :], np.full((1, 1, L), dt), np.array([[A]]),
                                     np.ones((1, L, 1)), np.ones((1, L, 1)), disc="dirac", delta_softplus=False)
    np.testing.assert_allclose(x[0, :, 0].real, y[0, 0], rtol=1e-13)
    assert np.all(x.imag == 0)


# ----------------------------------------------------------------------------- single-token step

@pytest.mark.parametrize("disc", DISCS)
def test_step_by_step_equals_the_scan(oracle, disc):
    """Mode equivalence (Sec. 3): L calls of the step update reproduce the scan, state and output, and a single
    step matches Eq. 2 written out by hand."""
    rng = np.random.default_rng(12)
    p = _rand_problem(rng, B=2, D=3, N=4, L=11)
    y_scan, x_last = oracle.selective_scan_fwd(**p, disc=disc)
    x = p["x0"].copy()
    for l in range(11):
        y, x = oracle.selective_step(x, p["u"][:, :, l], p["delta"][:, :, l], p["A"], p["Bm"][:, l], p["Cm"][:, l],
                                     Dskip=p["Dskip"], delta_bias=p["delta_bias"], z=p["z"][:, :, l], disc=disc)
        np.testing.assert_allclose(y, y_scan[:, :, l], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(x, x_last, rtol=1e-12, atol=1e-13)
    # one step by hand for (b, d, n) = (1, 2, 3)
    b, d, n = 1, 2, 3
    dt = np.logaddexp(0, p["delta"][b, d, 0] + p["delta_bias"][d])
    a, g = _disc_py(disc, dt, p["A"][d, n])
    _, x1 = oracle.selective_step(p["x0"], p["u"][:, :, 0], p["delta"][:, :, 0], p["A"], p["Bm"][:, 0], p["Cm"][:, 0],
                                  delta_bias=p["delta_bias"], disc=disc)
    assert x1[b, d, n] == pytest.approx(a * p["x0"][b, d, n] + g * p["Bm"][b, 0, n] * p["u"][b, d, 0], rel=1e-13)


def test_grouped_step_by_step_equals_the_grouped_scan(oracle):
    """With grouped maps [B,G,N] per token the step update reproduces the grouped scan (itself pinned above), and one
    state entry matches Eq. 2 written by hand with the group lookup."""
    p, _ = _grouped_problem(44, B=2, D=6, N=3, L=7, G=3)
    y_scan, x_last = oracle.selective_scan_fwd(**p)
    x = p["x0"].copy()
    for l in range(7):
        y, x = oracle.selective_step(x, p["u"][:, :, l], p["delta"][:, :, l], p["A"], p["Bm"][:, :, l], p["Cm"][:, :, l],
                                     Dskip=p["Dskip"], delta_bias=p["delta_bias"], z=p["z"][:, :, l])
        np.testing.assert_allclose(y, y_scan[:, :, l], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(x, x_last, rtol=1e-12, atol=1e-13)
    b, d, n = 1, 5, 2                                    # channel 5 of 6 in 3 groups -> group 2
    dt = np.logaddexp(0, p["delta"][b, d, 0] + p["delta_bias"][d])
    _, x1 = oracle.selective_step(p["x0"], p["u"][:, :, 0], p["delta"][:, :, 0], p["A"], p["Bm"][:, :, 0],
                                  p["Cm"][:, :, 0], delta_bias=p["delta_bias"])
    assert x1[b, d, n] == pytest.approx(np.exp(dt * p["A"][d, n]) * p["x0"][b, d, n]
                                        + dt * p["Bm"][b, 2, 0, n] * p["u"][b, d, 0], rel=1e-13)


def test_lti_step_equals_the_scan(oracle):
    rng = np.random.default_rng(13)
    Bsz, L, P = 2, 9, 5
    lam = rng.uniform(0.9, 0.999, P) * np.exp(1j * rng.uniform(0, 2 * np.pi, P))
    v = rng.standard_normal((Bsz, L, P)) + 1j * rng.standard_normal((Bsz, L, P))
    x0 = rng.standard_normal((Bsz, P)) + 1j * rng.standard_normal((Bsz, P))
    xs = oracle.lti_diag_scan(lam, v, x0=x0)
    x = x0
    for k in range(L):
        x = oracle.lti_step(lam, x, v[:, k])
        np.testing.assert_allclose(x, xs[:, k], rtol=1e-13)
    np.testing.assert_allclose(oracle.lti_step(lam, x0, v[:, 0]), lam[None, :] * x0 + v[:, 0], rtol=1e-15)


# ---------------------------------------------------------------------------------------------------------------
# LTI backward (adjoint of x_k = lam x_{k-1} + v_k, Sec. 2.2.1).  Convention: grad_z = dLoss/dRe z + i dLoss/dIm z.
# ---------------------------------------------------------------------------------------------------------------
def _lti_case(seed, B=2, L=9, P=3):
    rng = np.random.default_rng(seed)
    lam = (0.6 + 0.35 * rng.random(P)) * np.exp(1j * rng.uniform(-1.0, 1.0, P))
    c = lambda *s: rng.standard_normal(s) + 1j * rng.standard_normal(s)
    return lam, c(B, L, P), c(B, P), c(B, L, P)


def test_lti_bwd_finite_differences_real_and_imaginary(oracle):
    """Loss = sum Re(conj(w) x) has gx = w; every real and imaginary part of v, lam, x0 is perturbed."""
    lam, v, x0, w = _lti_case(21)
    dv, dlam, dx0 = oracle.lti_diag_scan_bwd(lam, v, w, x0=x0)
    loss = lambda lam_, v_, x0_: float(np.sum((np.conj(w) * oracle.lti_diag_scan(lam_, v_, x0=x0_)).real))
    h = 1e-6

    def fd(which, idx, unit):
        args = [lam.copy(), v.copy(), x0.copy()]
        args[which][idx] += h * unit
        up = loss(*args)
        args[which][idx] -= 2 * h * unit
        return (up - loss(*args)) / (2 * h)

    for which, grad in ((0, dlam), (1, dv), (2, dx0)):
        for idx in np.ndindex(grad.shape):
            num = fd(which, idx, 1.0) + 1j * fd(which, idx, 1j)
            assert abs(num - grad[idx]) <= 1e-7 * (1 + abs(grad[idx])), (which, idx, num, grad[idx])


def test_lti_bwd_single_step_closed_form(oracle):
    lam, v, x0, w = _lti_case(22, B=3, L=1, P=4)
    dv, dlam, dx0 = oracle.lti_diag_scan_bwd(lam, v, w, x0=x0)
    np.testing.assert_allclose(dv, w, rtol=1e-15)
    np.testing.assert_allclose(dx0, np.conj(lam)[None, :] * w[:, 0], rtol=1e-14)
    np.testing.assert_allclose(dlam, (np.conj(x0) * w[:, 0]).sum(0), rtol=1e-13)


def test_lti_bwd_dv_is_the_time_reversed_scan_with_conjugate_pole(oracle):
    """dv reversed in time obeys the forward recurrence with conj(lam) driven by the reversed gx; and with x0 = 0,
    a one-step sequence dlam vanishes (x_0 = 0 is the only state multiplied by lam)."""
    lam, v, x0, w = _lti_case(23, B=2, L=40, P=5)
    dv, dlam, dx0 = oracle.lti_diag_scan_bwd(lam, v, w, x0=x0)
    rev = oracle.lti_diag_scan(np.conj(lam), w[:, ::-1])[:, ::-1]
    np.testing.assert_allclose(dv, rev, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(dx0, np.conj(lam)[None, :] * dv[:, 0], rtol=1e-13)
    # dlam by the explicit double sum over pairs (j < k): x_{k-1} = lam^{k-1} x0 + sum_{j<k} lam^{k-1-j} v_j
    B, L, P = v.shape
    ref = np.zeros(P, dtype=complex)
    for b in range(B):
        for k in range(1, L + 1):                  # 1-based step k, state x_{k-1}
            xprev = lam ** (k - 1) * x0[b] + sum(lam ** (k - 1 - j) * v[b, j - 1] for j in range(1, k))
            ref += np.conj(xprev) * dv[b, k - 1]
    np.testing.assert_allclose(dlam, ref, rtol=1e-11)
    _, dl1, _ = oracle.lti_diag_scan_bwd(lam, v[:, :1], w[:, :1])
    assert np.all(dl1 == 0)


def test_lti_bwd_matches_library_autograd(oracle):
    """torch's complex autograd on a plain Python loop of the recurrence (its grad convention is the same)."""
    import torch
    lam, v, x0, w = _lti_case(24, B=2, L=12, P=3)
    tl, tv, tx0 = (torch.tensor(a, dtype=torch.complex128, requires_grad=True) for a in (lam, v, x0))
    x, xs = tx0, []
    for k in range(v.shape[1]):
        x = tl * x + tv[:, k]
        xs.append(x)
    loss = (torch.conj(torch.tensor(w)) * torch.stack(xs, 1)).real.sum()
    loss.backward()
    dv, dlam, dx0 = oracle.lti_diag_scan_bwd(lam, v, w, x0=x0)
    np.testing.assert_allclose(dv, tv.grad.numpy(), rtol=1e-12)
    np.testing.assert_allclose(dlam, tl.grad.numpy(), rtol=1e-12)
    np.testing.assert_allclose(dx0, tx0.grad.numpy(), rtol=1e-12)


# ---------------------------------------------------------------------------------------------------------------
# Caller-supplied (a_k, b_k) diagonal scan (the time-varying layers of Sec. 2.2.2 without their gating networks).
# ---------------------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("cplx", [False, True])
def test_diag_scan_product_sum_closed_form(oracle, cplx):
    """x_k = (prod_{i<=k} a_i) x0 + sum_j (prod_{j<i<=k} a_i) b_j, written with explicit products."""
    rng = np.random.default_rng(31)
    B, L, P = 2, 11, 3
    draw = (lambda *s: rng.uniform(0.5, 1.1, s) * np.exp(1j * rng.uniform(-1, 1, s))) if cplx else \
           (lambda *s: rng.uniform(-1.1, 1.1, s))
    a, b, x0 = draw(B, L, P), draw(B, L, P), draw(B, P)
    x = oracle.diag_scan(a, b, x0=x0)
    for k in range(L):
        ref = np.prod(a[:, :k + 1], axis=1) * x0
        for j in range(k + 1):
            ref = ref + np.prod(a[:, j + 1:k + 1], axis=1) * b[:, j]
        np.testing.assert_allclose(x[:, k], ref, rtol=1e-12, atol=1e-13)
    assert x.dtype == (np.complex128 if cplx else np.float64)


def test_diag_scan_reduces_to_the_lti_scan_and_to_the_selective_scan(oracle):
    rng = np.random.default_rng(32)
    B, L, P = 2, 50, 4
    lam = 0.9 * np.exp(1j * rng.uniform(0, 6.28, P))
    v = rng.standard_normal((B, L, P)) + 1j * rng.standard_normal((B, L, P))
    x0 = rng.standard_normal((B, P)) + 0j
    np.testing.assert_allclose(oracle.diag_scan(np.broadcast_to(lam, v.shape), v, x0=x0),
                               oracle.lti_diag_scan(lam, v, x0=x0), rtol=1e-13)
    # selective scan states: a = exp(dt A), b = dt B u per (d, n), with P = D * N
    D, N = 3, 2
    u, dl = rng.standard_normal((B, D, L)), rng.uniform(0.01, 0.2, (B, D, L))
    A, Bm, Cm = -rng.uniform(0.5, 2, (D, N)), rng.standard_normal((B, L, N)), rng.standard_normal((B, L, N))
    _, _, xs = oracle.selective_scan_fwd(u, dl, A, Bm, Cm, delta_softplus=False, return_states=True)
    a = np.exp(dl.transpose(0, 2, 1)[..., None] * A[None, None])                 # [B,L,D,N]
    b = (dl * u).transpose(0, 2, 1)[..., None] * Bm[:, :, None, :]
    got = oracle.diag_scan(a.reshape(B, L, D * N), b.reshape(B, L, D * N)).reshape(B, L, D, N)
    np.testing.assert_allclose(got, xs.transpose(0, 2, 1, 3), rtol=1e-12, atol=1e-14)


def test_diag_scan_chaining_and_gates(oracle):
    """Splitting the sequence and carrying the last state reproduces the one-shot scan; a_k = 0 resets the state and
    a_k = 1, b_k = 0 holds it (the two extremes of a gate)."""
    rng = np.random.default_rng(33)
    B, L, P = 1, 30, 2
    a, b = rng.uniform(0.2, 1.0, (B, L, P)), rng.standard_normal((B, L, P))
    x = oracle.diag_scan(a, b)
    x2 = oracle.diag_scan(a[:, 13:], b[:, 13:], x0=x[:, 12])
    np.testing.assert_allclose(x2, x[:, 13:], rtol=1e-14)
    a[:, 7], a[:, 20], b[:, 20] = 0.0, 1.0, 0.0
    x = oracle.diag_scan(a, b)
    np.testing.assert_array_equal(x[:, 7], b[:, 7])
    np.testing.assert_array_equal(x[:, 20], x[:, 19])


# ---------------------------------------------------------------------------------------------------------------
# Grouped input/output maps: Bm, Cm [B,G,L,N], channel d reads group d // (D/G)  (a workload variant of Eq. 2's
# B(k), C(k): several heads, each with its own input-dependent maps).
# ---------------------------------------------------------------------------------------------------------------
def _grouped_problem(seed, B=2, D=6, N=3, L=8, G=3):
    rng = np.random.default_rng(seed)
    p = _rand_problem(rng, B=B, D=D, N=N, L=L)
    p["Bm"], p["Cm"] = rng.standard_normal((B, G, L, N)), rng.standard_normal((B, G, L, N))
    return p, rng.standard_normal((B, D, L))


def test_grouped_forward_is_the_unrolled_sum_with_the_group_lookup(oracle):
    p, _ = _grouped_problem(41)
    B, D, L = p["u"].shape
    G, N = p["Bm"].shape[1], p["A"].shape[1]
    q = dict(p, z=None, x0=None)
    y, _ = oracle.selective_scan_fwd(**q)
    for b in range(B):
        for d in range(D):
            grp = d // (D // G)
            dt = np.logaddexp(0.0, p["delta"][b, d] + p["delta_bias"][d])
            for l in range(L):
                acc = p["Dskip"][d] * p["u"][b, d, l]
                for n in range(N):
                    for j in range(l + 1):
                        acc += p["Cm"][b, grp, l, n] * np.exp(p["A"][d, n] * dt[j + 1:l + 1].sum()) * dt[j] \
                               * p["Bm"][b, grp, j, n] * p["u"][b, d, j]
                assert y[b, d, l] == pytest.approx(acc, rel=1e-11, abs=1e-12)


def test_grouped_equals_one_ungrouped_problem_per_group(oracle):
    """Each group is an independent ungrouped problem over its own channels; its dBm, dCm sum over those channels only."""
    p, dy = _grouped_problem(42)
    D, G = p["u"].shape[1], p["Bm"].shape[1]
    y, xl = oracle.selective_scan_fwd(**p)
    g = oracle.selective_scan_bwd(dy=dy, **p)
    for grp in range(G):
        ds = slice(grp * (D // G), (grp + 1) * (D // G))
        q = dict(u=p["u"][:, ds], delta=p["delta"][:, ds], A=p["A"][ds], Bm=p["Bm"][:, grp], Cm=p["Cm"][:, grp],
                 Dskip=p["Dskip"][ds], delta_bias=p["delta_bias"][ds], z=p["z"][:, ds], x0=p["x0"][:, ds])
        yq, xq = oracle.selective_scan_fwd(**q)
        gq = oracle.selective_scan_bwd(dy=dy[:, ds], **q)
        np.testing.assert_allclose(y[:, ds], yq, rtol=1e-14)
        np.testing.assert_allclose(xl[:, ds], xq, rtol=1e-14)
        for k in ("du", "ddelta", "dz", "dx0"):
            np.testing.assert_allclose(g[k][:, ds], gq[k], rtol=1e-13, atol=1e-15)
        for k in ("dA", "dD", "dbias"):
            np.testing.assert_allclose(g[k][ds], gq[k], rtol=1e-13, atol=1e-15)
        for k in ("dBm", "dCm"):
            np.testing.assert_allclose(g[k][:, grp], gq[k], rtol=1e-13, atol=1e-15)


def test_grouped_gradients_of_the_maps_by_finite_differences(oracle):
    p, dy = _grouped_problem(43, B=1, D=4, N=2, L=5, G=2)
    g = oracle.selective_scan_bwd(dy=dy, **p)
    loss = lambda q: float((oracle.selective_scan_fwd(**q)[0] * dy).sum())
    h = 1e-6
    for k, gk in (("Bm", "dBm"), ("Cm", "dCm")):
        for idx in np.ndindex(p[k].shape):
            q = {n: (v.copy() if isinstance(v, np.ndarray) else v) for n, v in p.items()}
            q[k][idx] += h
            up = loss(q)
            q[k][idx] -= 2 * h
            num = (up - loss(q)) / (2 * h)
            assert num == pytest.approx(g[gk][idx], rel=1e-6, abs=1e-8), (k, idx)


# ---------------------------------------------------------------------------------------------------------------
# Packed variable-length batches (independent sequences one after the other on one time axis).
# ---------------------------------------------------------------------------------------------------------------
def _packed_problem(seed, D=3, N=2, L=23, cu=(0, 5, 6, 14, 23), G=None):
    rng = np.random.default_rng(seed)
    S = len(cu) - 1
    bc = (L, N) if G is None else (G, L, N)
    p = dict(u=rng.standard_normal((D, L)), delta=rng.standard_normal((D, L)), A=-np.exp(rng.uniform(-1, 1, (D, N))),
             Bm=rng.standard_normal(bc), Cm=rng.standard_normal(bc), Dskip=rng.standard_normal(D),
             delta_bias=rng.uniform(-2, 0, D), z=rng.standard_normal((D, L)), x0=rng.standard_normal((S, D, N)))
    return p, np.array(cu), rng.standard_normal((D, L))


def test_packed_states_equal_one_long_scan_whose_multiplier_is_zeroed_at_every_boundary(oracle):
    """An independent route to the same numbers: ONE recurrence over the whole packed axis in which the first step of
    every sequence forgets the past (a = 0) and takes that sequence's x0 through b."""
    p, cu, _ = _packed_problem(51)
    D, L = p["u"].shape
    N = p["A"].shape[1]
    dt = np.logaddexp(0.0, p["delta"] + p["delta_bias"][:, None])                       # [D,L]
    a = np.exp(dt.T[:, :, None] * p["A"][None])                                         # [L,D,N]
    b = (dt * p["u"]).T[:, :, None] * p["Bm"][:, None, :]
    for s, o in enumerate(cu[:-1]):
        if o < L:
            b[o] += a[o] * p["x0"][s]
            a[o] = 0.0
    x = oracle.diag_scan(a.reshape(1, L, D * N), b.reshape(1, L, D * N)).reshape(L, D, N)
    ypre = np.einsum("ln,ldn->dl", p["Cm"], x) + p["Dskip"][:, None] * p["u"]
    yref = ypre * p["z"] / (1 + np.exp(-p["z"]))
    y, x_last = oracle.selective_scan_fwd_packed(cu_seqlens=cu, **p)
    np.testing.assert_allclose(y, yref, rtol=1e-12, atol=1e-13)
    for s in range(len(cu) - 1):
        np.testing.assert_allclose(x_last[s], x[cu[s + 1] - 1], rtol=1e-12)


def test_packed_sequences_do_not_see_each_other(oracle):
    p, cu, dy = _packed_problem(52)
    y, xl = oracle.selective_scan_fwd_packed(cu_seqlens=cu, **p)
    g = oracle.selective_scan_bwd_packed(dy=dy, cu_seqlens=cu, **p)
    q = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in p.items()}
    o, e = cu[2], cu[3]                                    # disturb sequence 2 only
    q["u"][:, o:e] += 1.0
    q["Bm"][o:e] *= 2.0
    q["x0"][2] -= 3.0
    y2, xl2 = oracle.selective_scan_fwd_packed(cu_seqlens=cu, **q)
    g2 = oracle.selective_scan_bwd_packed(dy=dy, cu_seqlens=cu, **q)
    keep = np.ones(p["u"].shape[1], bool)
    keep[o:e] = False
    assert np.array_equal(y[:, keep], y2[:, keep]) and not np.allclose(y[:, o:e], y2[:, o:e])
    assert np.array_equal(np.delete(xl, 2, 0), np.delete(xl2, 2, 0))
    for k in ("du", "ddelta", "dz"):
        assert np.array_equal(g[k][:, keep], g2[k][:, keep]), k
    assert np.array_equal(g["dBm"][keep], g2["dBm"][keep]) and np.array_equal(g["dCm"][keep], g2["dCm"][keep])


def test_packed_with_one_sequence_is_the_plain_call_and_gaps_stay_zero(oracle):
    p, _, dy = _packed_problem(53, cu=(0, 23))
    y, xl = oracle.selective_scan_fwd_packed(cu_seqlens=np.array([0, 23]), **p)
    q = dict(u=p["u"][None], delta=p["delta"][None], A=p["A"], Bm=p["Bm"][None], Cm=p["Cm"][None], Dskip=p["Dskip"],
             delta_bias=p["delta_bias"], z=p["z"][None], x0=p["x0"])
    yr, xr = oracle.selective_scan_fwd(**q)
    np.testing.assert_array_equal(y, yr[0])
    np.testing.assert_array_equal(xl, xr)
    # a batch that leaves steps 0..2 and 20..22 outside every sequence, with an empty sequence in the middle
    cu = np.array([3, 9, 9, 20])
    p3, _, _ = _packed_problem(54, cu=(3, 9, 9, 20))
    y3, xl3 = oracle.selective_scan_fwd_packed(cu_seqlens=cu, **p3)
    assert np.all(y3[:, :3] == 0) and np.all(y3[:, 20:] == 0)
    np.testing.assert_array_equal(xl3[1], p3["x0"][1])     # an empty sequence hands its x0 through


def test_packed_backward_by_finite_differences_with_grouped_maps(oracle):
    p, cu, dy = _packed_problem(55, D=4, N=2, L=11, cu=(0, 4, 11), G=2)
    g = oracle.selective_scan_bwd_packed(dy=dy, cu_seqlens=cu, **p)
    loss = lambda q: float((oracle.selective_scan_fwd_packed(cu_seqlens=cu, **q)[0] * dy).sum())
    h = 1e-6
    names = {"u": "du", "delta": "ddelta", "A": "dA", "Bm": "dBm", "Cm": "dCm", "Dskip": "dD", "delta_bias": "dbias",
             "z": "dz", "x0": "dx0"}
    for k, gk in names.items():
        for idx in np.ndindex(p[k].shape):
            q = {n: (v.copy() if isinstance(v, np.ndarray) else v) for n, v in p.items()}
            q[k][idx] += h
            up = loss(q)
            q[k][idx] -= 2 * h
            num = (up - loss(q)) / (2 * h)
            assert num == pytest.approx(g[gk][idx], rel=2e-6, abs=1e-7), (k, idx)


# ---------------------------------------------------------------------------------------------------------------
# Selective scan with a complex diagonal A and complex maps: y = Re(sum_n C x) + D u  (Sec. 2.2.1 layers made
# input-dependent; the "Re" of the recurrence as the paper's complex-diagonal layers use it).
# ---------------------------------------------------------------------------------------------------------------
def _disc_py_c(disc, dt, A):
    """Independent restatement of the four schemes for complex A with numpy complex scalars."""
    if disc == "bilinear":
        return (1 + dt * A / 2) / (1 - dt * A / 2), dt / (1 - dt * A / 2)
    a = np.exp(dt * A)
    return a, {"zoh_s6": dt, "zoh": (a - 1) / A, "dirac": 1.0}[disc]


def _complex_problem(seed, B=2, D=3, N=4, L=9):
    rng = np.random.default_rng(seed)
    c = lambda *s: rng.standard_normal(s) + 1j * rng.standard_normal(s)
    return dict(u=rng.standard_normal((B, D, L)), delta=rng.standard_normal((B, D, L)),
                A=-np.exp(rng.uniform(-1, 1, (D, N))) + 1j * rng.uniform(-3, 3, (D, N)),
                Bm=c(B, L, N), Cm=c(B, L, N), Dskip=rng.standard_normal(D), delta_bias=rng.uniform(-2, 0, D),
                z=rng.standard_normal((B, D, L)), x0=c(B, D, N))


@pytest.mark.parametrize("disc", DISCS)
def test_complex_forward_is_the_unrolled_sum(oracle, disc):
    p = _complex_problem(61)
    B, D, L = p["u"].shape
    N = p["A"].shape[1]
    y, x_last = oracle.selective_scan_fwd_complex(**p, disc=disc)
    dt = np.logaddexp(0.0, p["delta"] + p["delta_bias"][None, :, None])
    for b in range(B):
        for d in range(D):
            a, g = _disc_py_c(disc, dt[b, d][:, None], p["A"][d][None, :])           # [L,N]
            g = np.broadcast_to(g, a.shape)
            bvec = g * p["Bm"][b] * p["u"][b, d][:, None]
            for l in range(L):
                x = np.prod(a[:l + 1], axis=0) * p["x0"][b, d]
                for j in range(l + 1):
                    x = x + np.prod(a[j + 1:l + 1], axis=0) * bvec[j]
                ypre = (p["Cm"][b, l] * x).sum().real + p["Dskip"][d] * p["u"][b, d, l]
                zz = p["z"][b, d, l]
                assert y[b, d, l] == pytest.approx(ypre * zz / (1 + np.exp(-zz)), rel=1e-10, abs=1e-11)
            np.testing.assert_allclose(x_last[b, d], x, rtol=1e-10)


@pytest.mark.parametrize("disc", DISCS)
def test_complex_forward_with_real_data_is_the_real_scan(oracle, disc):
    rng = np.random.default_rng(62)
    p = _rand_problem(rng, B=2, D=3, N=4, L=12)
    y, xl = oracle.selective_scan_fwd(**p, disc=disc)
    q = dict(p, A=p["A"] + 0j, Bm=p["Bm"] + 0j, Cm=p["Cm"] + 0j, x0=p["x0"] + 0j)
    yc, xlc = oracle.selective_scan_fwd_complex(**q, disc=disc)
    np.testing.assert_allclose(yc, y, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(xlc.real, xl, rtol=1e-12, atol=1e-13)
    assert np.all(xlc.imag == 0)


@pytest.mark.parametrize("dt,A", [(0.05, -1.3 + 2.0j), (0.7, -0.4 - 5.0j), (1e-4, -2.5 + 0.3j)])
def test_complex_zoh_and_bilinear_match_scipy_cont2discrete(oracle, dt, A):
    """One complex state driven by u = 1 from rest for one step: x_1 = g, and from x0 = 1 with u = 0: x_1 = a."""
    sys_c = (np.array([[A]]), np.array([[1.0 + 0j]]), np.array([[1.0 + 0j]]), np.array([[0.0 + 0j]]))
    one = np.ones((1, 1, 1))
    for disc in ("zoh", "bilinear"):
        Ad, Bd, *_ = scipy.signal.cont2discrete(sys_c, dt, method=disc)
        kw = dict(A=np.array([[A]]), Bm=one + 0j, Cm=one + 0j, disc=disc, delta_softplus=False)
        _, g = oracle.selective_scan_fwd_complex(one, dt * one, **kw)
        _, a = oracle.selective_scan_fwd_complex(0 * one, dt * one, x0=one + 0j, **kw)
        assert g[0, 0, 0] == pytest.approx(Bd[0, 0], rel=1e-11)
        assert a[0, 0, 0] == pytest.approx(Ad[0, 0], rel=1e-12)


def test_complex_forward_with_constant_step_is_the_lti_scan(oracle):
    """Constant Delta and time-invariant maps: the states are those of the LTI complex-diagonal scan with
    lambda = exp(Delta A) and v = Delta B u, and y = Re(sum C x)."""
    rng = np.random.default_rng(63)
    L, N = 40, 5
    A = -rng.uniform(0.1, 1, N) + 1j * rng.uniform(-3, 3, N)
    Bv, Cv = rng.standard_normal(N) + 1j * rng.standard_normal(N), rng.standard_normal(N) + 1j * rng.standard_normal(N)
    u = rng.standard_normal(L)
    dt = 0.3
    x = oracle.lti_diag_scan(np.exp(dt * A), (dt * Bv[None, :] * u[:, None])[None])            # [1,L,N]
    y, xl = oracle.selective_scan_fwd_complex(u[None, None], np.full((1, 1, L), dt), A[None], np.tile(Bv, (1, L, 1)),
                                              np.tile(Cv, (1, L, 1)), delta_softplus=False)
    np.testing.assert_allclose(y[0, 0], (x[0] * Cv[None, :]).sum(-1).real, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(xl[0, 0], x[0, -1], rtol=1e-12)


# ---------------------------------------------------------------------------------------------------------------
# Backward of the caller-supplied (a_k, b_k) scan.
# ---------------------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("cplx", [False, True])
def test_diag_scan_bwd_finite_differences(oracle, cplx):
    rng = np.random.default_rng(71)
    B, L, P = 2, 7, 3
    draw = (lambda *s: rng.standard_normal(s) + 1j * rng.standard_normal(s)) if cplx else (lambda *s: rng.standard_normal(s))
    a, b, x0, w = draw(B, L, P) * 0.7, draw(B, L, P), draw(B, P), draw(B, L, P)
    da, db, dx0 = oracle.diag_scan_bwd(a, b, w, x0=x0)
    loss = lambda a_, b_, x0_: float(np.sum((np.conj(w) * oracle.diag_scan(a_, b_, x0=x0_)).real))
    h = 1e-6
    for which, grad in ((0, da), (1, db), (2, dx0)):
        for idx in np.ndindex(grad.shape):
            num = 0.0
            for unit in ((1.0, 1j) if cplx else (1.0,)):
                args = [a.copy(), b.copy(), x0.copy()]
                args[which][idx] += h * unit
                up = loss(*args)
                args[which][idx] -= 2 * h * unit
                num = num + unit * (up - loss(*args)) / (2 * h)
            assert abs(num - grad[idx]) <= 1e-7 * (1 + abs(grad[idx])), (which, idx, num, grad[idx])


def test_diag_scan_bwd_one_step_and_constant_coefficient_cases(oracle):
    rng = np.random.default_rng(72)
    c = lambda *s: rng.standard_normal(s) + 1j * rng.standard_normal(s)
    a, b, x0, w = c(2, 1, 3), c(2, 1, 3), c(2, 3), c(2, 1, 3)
    da, db, dx0 = oracle.diag_scan_bwd(a, b, w, x0=x0)
    np.testing.assert_allclose(db, w, rtol=1e-15)
    np.testing.assert_allclose(da[:, 0], np.conj(x0) * w[:, 0], rtol=1e-14)
    np.testing.assert_allclose(dx0, np.conj(a[:, 0]) * w[:, 0], rtol=1e-14)
    # a_k = lambda for every k: db is the LTI backward's dv, dx0 agrees, and dlambda is the sum of da over b and k
    lam, v, x0l, wl = _lti_case(73, B=2, L=30, P=4)
    dv, dlam, dx0l = oracle.lti_diag_scan_bwd(lam, v, wl, x0=x0l)
    da, db, dx0 = oracle.diag_scan_bwd(np.broadcast_to(lam, v.shape), v, wl, x0=x0l)
    np.testing.assert_allclose(db, dv, rtol=1e-13)
    np.testing.assert_allclose(dx0, dx0l, rtol=1e-13)
    np.testing.assert_allclose(da.sum(axis=(0, 1)), dlam, rtol=1e-12)


def test_diag_scan_bwd_matches_library_autograd_on_real_gates(oracle):
    import torch
    rng = np.random.default_rng(74)
    a, b, x0, w = rng.uniform(0.2, 1.0, (2, 9, 3)), rng.standard_normal((2, 9, 3)), rng.standard_normal((2, 3)), rng.standard_normal((2, 9, 3))
    ta, tb, tx0 = (torch.tensor(t, requires_grad=True) for t in (a, b, x0))
    x, xs = tx0, []
    for k in range(9):
        x = ta[:, k] * x + tb[:, k]
        xs.append(x)
    (torch.tensor(w) * torch.stack(xs, 1)).sum().backward()
    da, db, dx0 = oracle.diag_scan_bwd(a, b, w, x0=x0)
    np.testing.assert_allclose(da, ta.grad.numpy(), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(db, tb.grad.numpy(), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(dx0, tx0.grad.numpy(), rtol=1e-12, atol=1e-14)
    assert da.dtype == np.float64


# ---------------------------------------------------------------------------------------------------------------
# Backward of the selective scan with a complex diagonal A (gradient of a complex q = dLoss/dRe q + i dLoss/dIm q).
# ---------------------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("disc", DISCS)
@pytest.mark.parametrize("dt,A", [(0.3, -0.8 + 2.5j), (1e-5, -1.5 - 0.7j), (2.0, -0.05 + 9.0j)])
def test_complex_disc_partials_by_finite_differences(oracle, disc, dt, A):
    """a and g restated with numpy complex scalars; their partials by central differences along dt and, a and g
    being holomorphic in A, along the real axis of A (the step along the imaginary axis must give the same)."""
    a, g, a_t, a_A, g_t, g_A = oracle.disc_terms_complex(disc, dt, A)
    ra, rg = _disc_py_c(disc, dt, A)
    assert a == pytest.approx(ra, rel=1e-12)
    assert g == pytest.approx(rg, rel=1e-9 if dt < 1e-3 else 1e-12)
    h = 1e-6 * max(dt, 1e-3)
    f = lambda t, z: np.array([complex(v) for v in _disc_py_c(disc, t, z)])
    num_t = (f(dt + h, A) - f(dt - h, A)) / (2 * h)
    hA = 1e-6
    num_A = (f(dt, A + hA) - f(dt, A - hA)) / (2 * hA)
    num_Ai = (f(dt, A + 1j * hA) - f(dt, A - 1j * hA)) / (2j * hA)
    tol = dict(rel=2e-5, abs=1e-9) if dt < 1e-3 else dict(rel=1e-7, abs=1e-10)
    assert a_t == pytest.approx(num_t[0], **tol) and g_t == pytest.approx(num_t[1], **tol)
    assert a_A == pytest.approx(num_A[0], **tol) and a_A == pytest.approx(num_Ai[0], **tol)
    if dt >= 1e-3:      # (e^z - 1)/A loses digits in the restated form for tiny z; the series is pinned below
        assert g_A == pytest.approx(num_A[1], **tol) and g_A == pytest.approx(num_Ai[1], **tol)


def test_complex_zoh_gain_series_meets_the_closed_form(oracle):
    """The exact-ZOH gain and its A-derivative switch to a power series for |dt A| < 1e-3: both branches agree at
    the switch, and for tiny z they tend to dt and dt^2/2."""
    A = -0.6 + 0.8j                                    # |A| = 1
    lo, hi = oracle.disc_terms_complex("zoh", 0.999e-3, A), oracle.disc_terms_complex("zoh", 1.001e-3, A)
    for i in (1, 5):
        scale = (1.001 / 0.999) ** (1 if i == 1 else 2)
        assert hi[i] == pytest.approx(lo[i] * scale, rel=1e-5)
        assert hi[i] == pytest.approx(lo[i] * scale * (1 + (0.002e-3 * A) * (0.5 if i == 1 else 2 / 3)), rel=1e-9)
    tiny = oracle.disc_terms_complex("zoh", 1e-9, A)
    assert tiny[1] == pytest.approx(1e-9, rel=1e-8) and tiny[5] == pytest.approx(0.5e-18, rel=1e-8)


@pytest.mark.parametrize("disc", DISCS)
@pytest.mark.parametrize("softplus", [True, False])
def test_complex_backward_finite_differences(oracle, disc, softplus):
    """Central differences of sum(dy * y) over every real input and over the real and imaginary parts of every
    complex input, against the forward oracle."""
    p = _complex_problem(81, B=2, D=2, N=3, L=6)
    if not softplus:
        p["delta"] = np.abs(p["delta"]) * 0.3 + 0.05
        p["delta_bias"] = np.abs(p["delta_bias"]) * 0.1
    rng = np.random.default_rng(82)
    dy = rng.standard_normal(p["u"].shape)
    kw = dict(disc=disc, delta_softplus=softplus)
    g = oracle.selective_scan_bwd_complex(**p, dy=dy, **kw)
    loss = lambda q: float(np.sum(dy * oracle.selective_scan_fwd_complex(**q, **kw)[0]))
    names = {"u": "du", "delta": "ddelta", "A": "dA", "Bm": "dBm", "Cm": "dCm", "Dskip": "dD", "delta_bias": "dbias",
             "z": "dz", "x0": "dx0"}
    h = 1e-6
    for k, gk in names.items():
        flat_idx = rng.choice(p[k].size, size=min(p[k].size, 6), replace=False)
        for fi in flat_idx:
            idx = np.unravel_index(fi, p[k].shape)
            parts = (1.0, 1j) if np.iscomplexobj(p[k]) else (1.0,)
            num = 0.0
            for part in parts:
                q = {n: (v.copy() if isinstance(v, np.ndarray) else v) for n, v in p.items()}
                q[k][idx] += h * part
                up = loss(q)
                q[k][idx] -= 2 * h * part
                num = num + part * (up - loss(q)) / (2 * h)
            assert num == pytest.approx(g[gk][idx], rel=2e-6, abs=2e-7), (k, idx)


@pytest.mark.parametrize("disc", DISCS)
def test_complex_backward_matches_library_autograd(oracle, disc):
    """torch's complex autograd (same gradient convention) on a plain Python loop of the recurrence."""
    import torch
    p = _complex_problem(83, B=2, D=2, N=3, L=7)
    dy = np.random.default_rng(84).standard_normal(p["u"].shape)
    t = {k: torch.tensor(v, dtype=torch.complex128 if np.iscomplexobj(v) else torch.float64, requires_grad=True)
         for k, v in p.items()}
    dt = torch.nn.functional.softplus(t["delta"] + t["delta_bias"][None, :, None])          # [B,D,L]
    x, ys = t["x0"], []
    for l in range(p["u"].shape[2]):
        zA = dt[:, :, l, None] * t["A"][None]                                                # [B,D,N]
        if disc == "bilinear":
            a, gain = (1 + zA / 2) / (1 - zA / 2), dt[:, :, l, None] / (1 - zA / 2)
        else:
            a = torch.exp(zA)
            gain = {"zoh_s6": dt[:, :, l, None] + 0j, "zoh": (a - 1) / t["A"][None], "dirac": torch.ones_like(a)}[disc]
        x = a * x + gain * t["Bm"][:, None, l, :] * t["u"][:, :, l, None]
        ypre = (t["Cm"][:, None, l, :] * x).sum(-1).real + t["Dskip"][None] * t["u"][:, :, l]
        ys.append(ypre * t["z"][:, :, l] * torch.sigmoid(t["z"][:, :, l]))
    (torch.stack(ys, -1) * torch.tensor(dy)).sum().backward()
    g = oracle.selective_scan_bwd_complex(**p, dy=dy, disc=disc)
    for k, gk in {"u": "du", "delta": "ddelta", "A": "dA", "Bm": "dBm", "Cm": "dCm", "Dskip": "dD",
                  "delta_bias": "dbias", "z": "dz", "x0": "dx0"}.items():
        np.testing.assert_allclose(g[gk], t[k].grad.numpy(), rtol=1e-10, atol=1e-12, err_msg=k)


@pytest.mark.parametrize("disc", DISCS)
def test_complex_backward_with_real_data_is_the_real_backward(oracle, disc):
    """Zero imaginary parts everywhere: the real parts of the gradients are those of the real scan's backward."""
    rng = np.random.default_rng(85)
    p = _rand_problem(rng, B=2, D=3, N=4, L=10)
    dy = rng.standard_normal(p["u"].shape)
    g = oracle.selective_scan_bwd(**p, dy=dy, disc=disc)
    q = dict(p, A=p["A"] + 0j, Bm=p["Bm"] + 0j, Cm=p["Cm"] + 0j, x0=p["x0"] + 0j)
    gc = oracle.selective_scan_bwd_complex(**q, dy=dy, disc=disc)
    for k in g:
        np.testing.assert_allclose(np.real(gc[k]), g[k], rtol=1e-11, atol=1e-13, err_msg=k)


def test_complex_backward_adjoint_dot_test(oracle):
    """y is linear in (u, Dskip-free) for fixed step sizes and maps, and real-linear in x0: for any direction
    (du, dx0), <dy, J (du, dx0)> must equal <J^T dy, (du, dx0)> with the real inner product Re(conj(a) b)."""
    p = _complex_problem(91, B=2, D=3, N=4, L=11)
    p["Dskip"] = None
    rng = np.random.default_rng(92)
    dy = rng.standard_normal(p["u"].shape)
    du = rng.standard_normal(p["u"].shape)
    dx0 = rng.standard_normal(p["x0"].shape) + 1j * rng.standard_normal(p["x0"].shape)
    for disc in DISCS:
        g = oracle.selective_scan_bwd_complex(**p, dy=dy, disc=disc)
        # without the gate y is linear in (u, x0): J applied to a direction is the forward pass of that direction
        q = dict(p, z=None)
        gq = oracle.selective_scan_bwd_complex(**q, dy=dy, disc=disc)
        Jd, _ = oracle.selective_scan_fwd_complex(**dict(q, u=du, x0=dx0), disc=disc)
        lhs = float(np.sum(dy * Jd))
        rhs = float(np.sum(gq["du"] * du) + np.sum((np.conj(gq["dx0"]) * dx0).real))
        assert lhs == pytest.approx(rhs, rel=1e-11)
        # with the gate: dz and the gated du follow from the ungated ones
        zz = p["z"]
        sg = 1 / (1 + np.exp(-zz))
        gz = oracle.selective_scan_bwd_complex(**q, dy=dy * zz * sg, disc=disc)
        np.testing.assert_allclose(g["du"], gz["du"], rtol=1e-11, atol=1e-13)
        ypre, _ = oracle.selective_scan_fwd_complex(**q, disc=disc)
        np.testing.assert_allclose(g["dz"], dy * ypre * sg * (1 + zz * (1 - sg)), rtol=1e-11, atol=1e-13)


def test_complex_forward_chains_through_x0_and_x_last(oracle):
    """Two calls on the halves of a sequence, the second starting from the first one's x_last, equal one call; the
    backward pass chains the other way through dx0 (the gradient of a loss on both halves w.r.t. the first half's
    inputs needs the second half's dx0 as the gradient reaching x_last)."""
    p = _complex_problem(93, B=2, D=2, N=3, L=14)
    cut = 6
    y, xl = oracle.selective_scan_fwd_complex(**p, disc="zoh")
    first = {k: (v[:, :, :cut] if k in ("u", "delta", "z") else v[:, :cut] if k in ("Bm", "Cm") else v) for k, v in p.items()}
    second = {k: (v[:, :, cut:] if k in ("u", "delta", "z") else v[:, cut:] if k in ("Bm", "Cm") else v) for k, v in p.items()}
    y1, xl1 = oracle.selective_scan_fwd_complex(**first, disc="zoh")
    y2, xl2 = oracle.selective_scan_fwd_complex(**dict(second, x0=xl1), disc="zoh")
    np.testing.assert_allclose(np.concatenate([y1, y2], axis=2), y, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(xl2, xl, rtol=1e-12)
    dy = np.random.default_rng(94).standard_normal(y.shape)
    g = oracle.selective_scan_bwd_complex(**p, dy=dy, disc="zoh")
    g2 = oracle.selective_scan_bwd_complex(**dict(second, x0=xl1), dy=dy[:, :, cut:], disc="zoh")
    np.testing.assert_allclose(g2["du"], g["du"][:, :, cut:], rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(g2["dCm"], g["dCm"][:, cut:], rtol=1e-11, atol=1e-13)
    # the first half sees the second half only through x_last: its gradient there is the second half's dx0.  With
    # y = Re(C x) the state enters linearly, so the contribution can be checked on dx0 of the whole sequence:
    # dx0(whole) = dx0(first half alone) + (prod of the first half's multipliers)^H dx0(second half)
    g1 = oracle.selective_scan_bwd_complex(**first, dy=dy[:, :, :cut], disc="zoh")
    dt = np.logaddexp(0.0, p["delta"] + p["delta_bias"][None, :, None])[:, :, :cut]          # [B,D,cut]
    prod_a = np.exp(dt.sum(-1)[..., None] * p["A"][None])                                      # [B,D,N]
    np.testing.assert_allclose(g["dx0"], g1["dx0"] + np.conj(prod_a) * g2["dx0"], rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("disc", DISCS)
def test_complex_step_by_step_equals_the_complex_scan(oracle, disc):
    """Mode equivalence (Sec. 3) for the complex-A scan: L step calls reproduce the scan, and one step matches the
    recurrence written out with numpy complex scalars; with zero imaginary parts it is the real step."""
    p = _complex_problem(95, B=2, D=3, N=4, L=9)
    y_scan, x_last = oracle.selective_scan_fwd_complex(**p, disc=disc)
    x = p["x0"].copy()
    for l in range(9):
        y, x = oracle.selective_step_complex(x, p["u"][:, :, l], p["delta"][:, :, l], p["A"], p["Bm"][:, l], p["Cm"][:, l],
                                             Dskip=p["Dskip"], delta_bias=p["delta_bias"], z=p["z"][:, :, l], disc=disc)
        np.testing.assert_allclose(y, y_scan[:, :, l], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(x, x_last, rtol=1e-12, atol=1e-13)
    b, d, n = 1, 2, 3
    dt = np.logaddexp(0, p["delta"][b, d, 0] + p["delta_bias"][d])
    a, g = _disc_py_c(disc, dt, p["A"][d, n])
    y1, x1 = oracle.selective_step_complex(p["x0"], p["u"][:, :, 0], p["delta"][:, :, 0], p["A"], p["Bm"][:, 0],
                                           p["Cm"][:, 0], delta_bias=p["delta_bias"], disc=disc)
    assert x1[b, d, n] == pytest.approx(a * p["x0"][b, d, n] + g * p["Bm"][b, 0, n] * p["u"][b, d, 0], rel=1e-12)
    assert y1[b, d] == pytest.approx((p["Cm"][b, 0] * x1[b, d]).sum().real, rel=1e-12)
    rng = np.random.default_rng(96)
    q = _rand_problem(rng, B=2, D=3, N=4, L=1)
    yr, xr = oracle.selective_step(q["x0"], q["u"][:, :, 0], q["delta"][:, :, 0], q["A"], q["Bm"][:, 0], q["Cm"][:, 0],
                                   Dskip=q["Dskip"], delta_bias=q["delta_bias"], z=q["z"][:, :, 0], disc=disc)
    yc, xc = oracle.selective_step_complex(q["x0"] + 0j, q["u"][:, :, 0], q["delta"][:, :, 0], q["A"] + 0j,
                                           q["Bm"][:, 0] + 0j, q["Cm"][:, 0] + 0j, Dskip=q["Dskip"],
                                           delta_bias=q["delta_bias"], z=q["z"][:, :, 0], disc=disc)
    np.testing.assert_allclose(yc, yr, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(xc.real, xr, rtol=1e-12, atol=1e-13)


def test_complex_grouped_equals_one_ungrouped_problem_per_group(oracle):
    """Grouped maps for the complex-A scan: each group is an independent ungrouped problem over its own channels
    (forward, backward and single-token step); the ungrouped functions are pinned above."""
    B, D, N, L, G = 2, 6, 3, 8, 3
    p = _complex_problem(97, B=B, D=D, N=N, L=L)
    rng = np.random.default_rng(98)
    c = lambda *s: rng.standard_normal(s) + 1j * rng.standard_normal(s)
    p["Bm"], p["Cm"] = c(B, G, L, N), c(B, G, L, N)
    dy = rng.standard_normal((B, D, L))
    y, xl = oracle.selective_scan_fwd_complex(**p, disc="zoh")
    g = oracle.selective_scan_bwd_complex(dy=dy, **p, disc="zoh")
    ys, xs = oracle.selective_step_complex(p["x0"], p["u"][:, :, 0], p["delta"][:, :, 0], p["A"], p["Bm"][:, :, 0],
                                           p["Cm"][:, :, 0], Dskip=p["Dskip"], delta_bias=p["delta_bias"],
                                           z=p["z"][:, :, 0], disc="zoh")
    np.testing.assert_allclose(ys, y[:, :, 0], rtol=1e-12, atol=1e-13)       # the step is the scan's first token
    for grp in range(G):
        ds = slice(grp * (D // G), (grp + 1) * (D // G))
        q = dict(u=p["u"][:, ds], delta=p["delta"][:, ds], A=p["A"][ds], Bm=p["Bm"][:, grp], Cm=p["Cm"][:, grp],
                 Dskip=p["Dskip"][ds], delta_bias=p["delta_bias"][ds], z=p["z"][:, ds], x0=p["x0"][:, ds])
        yq, xq = oracle.selective_scan_fwd_complex(**q, disc="zoh")
        gq = oracle.selective_scan_bwd_complex(dy=dy[:, ds], **q, disc="zoh")
        np.testing.assert_allclose(y[:, ds], yq, rtol=1e-14)
        np.testing.assert_allclose(xl[:, ds], xq, rtol=1e-14)
        for k in ("du", "ddelta", "dz", "dx0"):
            np.testing.assert_allclose(g[k][:, ds], gq[k], rtol=1e-13, atol=1e-15)
        for k in ("dA", "dD", "dbias"):
            np.testing.assert_allclose(g[k][ds], gq[k], rtol=1e-13, atol=1e-15)
        for k in ("dBm", "dCm"):
            np.testing.assert_allclose(g[k][:, grp], gq[k], rtol=1e-13, atol=1e-15)


# ---------------------------------------------------------------------------------------------------------------
# Packed variable-length batches of the complex-A scan.
# ---------------------------------------------------------------------------------------------------------------
def _packed_complex_problem(seed, D=3, N=2, L=23, cu=(0, 5, 6, 14, 23), G=None):
    rng = np.random.default_rng(seed)
    c = lambda *s: rng.standard_normal(s) + 1j * rng.standard_normal(s)
    S = len(cu) - 1
    bc = (L, N) if G is None else (G, L, N)
    p = dict(u=rng.standard_normal((D, L)), delta=rng.standard_normal((D, L)),
             A=-np.exp(rng.uniform(-1, 1, (D, N))) + 1j * rng.uniform(-3, 3, (D, N)),
             Bm=c(*bc), Cm=c(*bc), Dskip=rng.standard_normal(D), delta_bias=rng.uniform(-2, 0, D),
             z=rng.standard_normal((D, L)), x0=c(S, D, N))
    return p, np.array(cu), rng.standard_normal((D, L))


@pytest.mark.parametrize("disc", DISCS)
def test_packed_complex_states_equal_one_long_scan_zeroed_at_every_boundary(oracle, disc):
    """An independent route: ONE complex recurrence over the whole packed axis (the caller-coefficient scan) whose
    multiplier is zeroed at the first step of every sequence, that sequence's x0 entering through b."""
    p, cu, _ = _packed_complex_problem(151)
    D, L = p["u"].shape
    N = p["A"].shape[1]
    dt = np.logaddexp(0.0, p["delta"] + p["delta_bias"][:, None])                       # [D,L]
    a, g = _disc_py_c(disc, dt.T[:, :, None], p["A"][None])                             # [L,D,N]
    a = np.array(np.broadcast_to(a, (L, D, N)))
    b = np.broadcast_to(g, (L, D, N)) * p["u"].T[:, :, None] * p["Bm"][:, None, :]
    for s, o in enumerate(cu[:-1]):
        if o < L and cu[s + 1] > o:
            b[o] += a[o] * p["x0"][s]
            a[o] = 0.0
    x = oracle.diag_scan(a.reshape(1, L, D * N), b.reshape(1, L, D * N)).reshape(L, D, N)
    ypre = np.einsum("ln,ldn->dl", p["Cm"], x).real + p["Dskip"][:, None] * p["u"]
    yref = ypre * p["z"] / (1 + np.exp(-p["z"]))
    y, x_last = oracle.selective_scan_fwd_complex_packed(cu_seqlens=cu, **p, disc=disc)
    np.testing.assert_allclose(y, yref, rtol=1e-11, atol=1e-12)
    for s in range(len(cu) - 1):
        np.testing.assert_allclose(x_last[s], x[cu[s + 1] - 1], rtol=1e-11)


def test_packed_complex_gaps_empty_sequences_and_isolation(oracle):
    cu = np.array([3, 9, 9, 20])
    p, _, dy = _packed_complex_problem(152, cu=(3, 9, 9, 20))
    y, xl = oracle.selective_scan_fwd_complex_packed(cu_seqlens=cu, **p)
    g = oracle.selective_scan_bwd_complex_packed(dy=dy, cu_seqlens=cu, **p)
    assert np.all(y[:, :3] == 0) and np.all(y[:, 20:] == 0)
    np.testing.assert_array_equal(xl[1], p["x0"][1])       # an empty sequence hands its x0 through
    assert np.all(g["dx0"][1] == 0) and np.all(g["dBm"][:3] == 0) and np.all(g["du"][:, 20:] == 0)
    q = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in p.items()}
    q["u"][:, 9:20] += 1.0                                 # disturb the last sequence only
    q["x0"][2] *= 2.0
    y2, xl2 = oracle.selective_scan_fwd_complex_packed(cu_seqlens=cu, **q)
    g2 = oracle.selective_scan_bwd_complex_packed(dy=dy, cu_seqlens=cu, **q)
    assert np.array_equal(y[:, :9], y2[:, :9]) and not np.allclose(y[:, 9:20], y2[:, 9:20])
    assert np.array_equal(xl[:2], xl2[:2])
    for k in ("du", "ddelta", "dz"):
        assert np.array_equal(g[k][:, :9], g2[k][:, :9]), k
    assert np.array_equal(g["dBm"][:9], g2["dBm"][:9]) and np.array_equal(g["dCm"][:9], g2["dCm"][:9])


def test_packed_complex_backward_by_finite_differences_with_grouped_maps(oracle):
    p, cu, dy = _packed_complex_problem(153, D=4, N=2, L=9, cu=(0, 4, 9), G=2)
    g = oracle.selective_scan_bwd_complex_packed(dy=dy, cu_seqlens=cu, **p, disc="zoh")
    loss = lambda q: float((oracle.selective_scan_fwd_complex_packed(cu_seqlens=cu, **q, disc="zoh")[0] * dy).sum())
    h = 1e-6
    names = {"u": "du", "delta": "ddelta", "A": "dA", "Bm": "dBm", "Cm": "dCm", "Dskip": "dD", "delta_bias": "dbias",
             "z": "dz", "x0": "dx0"}
    for k, gk in names.items():
        for idx in np.ndindex(p[k].shape):
            parts = (1.0, 1j) if np.iscomplexobj(p[k]) else (1.0,)
            num = 0.0
            for part in parts:
                q = {n: (v.copy() if isinstance(v, np.ndarray) else v) for n, v in p.items()}
                q[k][idx] += h * part
                up = loss(q)
                q[k][idx] -= 2 * h * part
                num = num + part * (up - loss(q)) / (2 * h)      # dLoss/dRe + i dLoss/dIm
            assert abs(num - g[gk][idx]) <= 2e-6 * abs(g[gk][idx]) + 2e-7, (k, idx)
