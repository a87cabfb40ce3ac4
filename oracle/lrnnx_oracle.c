/*
 * lrnnx_oracle.c -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * Plain sequential fp64 CPU statement of the diagonal linear recurrence of the
 * lrnnx paper (Sec. 2.2 "Linear RNNs", Eq. 2):
 *
 *     x_k = A(k) x_{k-1} + B(k) u_k
 *     y_k = C(k) x_k     + D(k) u_k
 *
 * specialised to a diagonal A(k), as used by the time-varying S6 layer and the
 * time-invariant complex-diagonal S5/LRU layers the paper lists (Sec. 2.2.1,
 * 2.2.2, Table 1).  The paper names the discretisation schemes (Sec. 3:
 * "ZOH, bilinear, dirac") without printing their formulas; the standard
 * diagonal forms are written out in disc_eval() below.
 *
 * Only tests/, __graft_entry__.smoke() and the cpu_baseline leg of bench.py
 * may use this file.  It shares no code with the HIP library and is never on
 * the product path.  Rows (b,d) are independent recurrences, so the outer row
 * loop carries an OpenMP pragma; nothing else is blocked, fused or reordered.
 *
 * Parity pins (tests/test_oracle_pins.py): brute-force unrolled sum, LTI
 * convolution closed form, impulse response, scipy.signal.lfilter and
 * cont2discrete, exact-ZOH step response, central finite differences, adjoint
 * dot test, linearity / causality / chaining invariants; for the LTI backward: finite differences of a real
 * loss over real and imaginary parts, the L = 1 closed form, the reversed-forward-scan identity; for the
 * caller-supplied (a_k, b_k) scan: the product/sum closed form, reduction to the LTI and the selective scans.
 * Complex-A selective scan: the unrolled complex sum, reduction to the real scan and to the LTI scan, cont2discrete
 * with a complex pole; its backward: finite differences over real and imaginary parts, a library's complex
 * automatic differentiation of the plain loop, reduction to the real backward, the partials of the complex
 * discretisations one by one.
 * Parity unpinned: which of the two "ZOH" input maps (disc 0 or 1) the
 * paper's own "zoh" string selects; the paper's asynchronous scheme is read
 * as "the caller supplies Delta per step" (delta_softplus = 0).
 *
 * Layouts (all contiguous, all double):
 *   u, delta, z, y, dy, du, ddelta, dz : [B, D, L]
 *   A, dA                               : [D, N]
 *   Bm, Cm, dBm, dCm                    : [B, G, L, N] (shared by the D/G consecutive channels of a group;
 *                                          G = 1: by all channels)
 *   Dskip, delta_bias, dD, dbias        : [D]
 *   x0, x_last, dx0                     : [B, D, N]
 *   xs (optional dump of every state)   : [B, D, L, N]
 *   LTI: lambda [P], v, x [B, L, P], x0 [B, P] -- complex, (re, im) pairs
 */
#include <complex.h>
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { DISC_ZOH_S6 = 0, DISC_ZOH = 1, DISC_BILINEAR = 2, DISC_DIRAC = 3 };

/* Discretisation of the scalar continuous system x' = A x + B u with step dt
 * (Sec. 3 names the schemes).  Returns the state multiplier a and the input
 * gain g (so that Bbar = g * B), and their partial derivatives.
 *   ZOH_S6   : a = exp(dt A), g = dt            (S6 simplification of ZOH)
 *   ZOH      : a = exp(dt A), g = (a - 1) / A   (exact zero-order hold)
 *   BILINEAR : a = (1 + dt A/2)/(1 - dt A/2), g = dt/(1 - dt A/2)
 *   DIRAC    : a = exp(dt A), g = 1             (impulse input, B unchanged)
 */
static void disc_eval(int disc, double dt, double A, double *a, double *g,
                      double *da_ddt, double *da_dA, double *dg_ddt, double *dg_dA)
{
    double aa, gg, a_t, a_A, g_t, g_A;
    if (disc == DISC_BILINEAR) {
        double q = 1.0 / (1.0 - 0.5 * dt * A);
        aa = (1.0 + 0.5 * dt * A) * q;
        gg = dt * q;
        a_t = A * q * q;
        a_A = dt * q * q;
        g_t = q * q;
        g_A = 0.5 * dt * dt * q * q;
    } else {
        aa = exp(dt * A);
        a_t = A * aa;
        a_A = dt * aa;
        if (disc == DISC_ZOH_S6) {
            gg = dt; g_t = 1.0; g_A = 0.0;
        } else if (disc == DISC_ZOH) {
            double em1 = expm1(dt * A);
            if (A == 0.0) { gg = dt; g_t = 1.0; g_A = 0.5 * dt * dt; }
            else {
                gg = em1 / A;
                g_t = aa;
                g_A = (dt * A * aa - em1) / (A * A);
            }
        } else { /* DISC_DIRAC */
            gg = 1.0; g_t = 0.0; g_A = 0.0;
        }
    }
    *a = aa; *g = gg;
    if (da_ddt) { *da_ddt = a_t; *da_dA = a_A; *dg_ddt = g_t; *dg_dA = g_A; }
}

/* softplus(s) = log(1 + e^s), written so that neither branch overflows. */
static double softplus(double s) { return fmax(s, 0.0) + log1p(exp(-fabs(s))); }
static double sigmoid(double s)  { return s >= 0 ? 1.0 / (1.0 + exp(-s)) : exp(s) / (1.0 + exp(s)); }

int lrnnx_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Expose the scalar pieces so the tests can pin them one by one. */
void lrnnx_oracle_disc(int disc, double dt, double A, double *out6)
{
    disc_eval(disc, dt, A, &out6[0], &out6[1], &out6[2], &out6[3], &out6[4], &out6[5]);
}
double lrnnx_oracle_softplus(double s) { return softplus(s); }

/* Forward selective scan (Eq. 2 with diagonal, input-dependent A(k), B(k), C(k)).
 * Optional pointers may be NULL: Dskip, delta_bias, z, x0, x_last, xs.        */
int lrnnx_oracle_selective_scan_fwd(
    int B, int D, int N, int G, long L, int disc, int delta_softplus,
    const double *u, const double *delta, const double *A,
    const double *Bm, const double *Cm, const double *Dskip,
    const double *delta_bias, const double *z, const double *x0,
    double *y, double *x_last, double *xs)
{
    if (B < 0 || D < 0 || N < 1 || L < 0 || disc < 0 || disc > 3 || G < 1 || D % G) return 1;
    long rows = (long)B * D;
#pragma omp parallel for schedule(static)
    for (long row = 0; row < rows; ++row) {
        int b = (int)(row / D), d = (int)(row % D);
        long bg = (long)b * G + d / (D / G);          /* row of Bm, Cm this channel reads: its batch entry and group */
        double *x = (double *)malloc(sizeof(double) * N);
        for (int n = 0; n < N; ++n) x[n] = x0 ? x0[row * N + n] : 0.0;
        for (long l = 0; l < L; ++l) {
            double s = delta[row * L + l] + (delta_bias ? delta_bias[d] : 0.0);
            double dt = delta_softplus ? softplus(s) : s;
            double uu = u[row * L + l];
            double acc = 0.0;
            for (int n = 0; n < N; ++n) {
                double a, g;
                disc_eval(disc, dt, A[(long)d * N + n], &a, &g, 0, 0, 0, 0);
                x[n] = a * x[n] + g * Bm[(bg * L + l) * N + n] * uu;   /* Eq. 2, line 1 */
                acc += Cm[(bg * L + l) * N + n] * x[n];                /* Eq. 2, line 2 */
                if (xs) xs[(row * L + l) * N + n] = x[n];
            }
            double ypre = acc + (Dskip ? Dskip[d] * uu : 0.0);
            if (z) { double zz = z[row * L + l]; ypre *= zz * sigmoid(zz); }
            y[row * L + l] = ypre;
        }
        if (x_last) for (int n = 0; n < N; ++n) x_last[row * N + n] = x[n];
        free(x);
    }
    return 0;
}

/* Complex discretisation of x' = A x + B u for complex A (same four schemes as disc_eval, complex arithmetic).
 * a = (ar, ai) is the state multiplier, g = (gr, gi) the input gain (Bbar = g * B).                        */
static void disc_eval_c(int disc, double dt, double Ar, double Ai, double *ar, double *ai, double *gr, double *gi)
{
    if (disc == DISC_BILINEAR) {
        /* a = (1 + dt A/2) / (1 - dt A/2), g = dt / (1 - dt A/2) */
        double wr = 1.0 - 0.5 * dt * Ar, wi = -0.5 * dt * Ai;
        double nr = 1.0 + 0.5 * dt * Ar, ni = 0.5 * dt * Ai;
        double den = wr * wr + wi * wi;
        *ar = (nr * wr + ni * wi) / den;
        *ai = (ni * wr - nr * wi) / den;
        *gr = dt * wr / den;
        *gi = -dt * wi / den;
        return;
    }
    double e = exp(dt * Ar);
    *ar = e * cos(dt * Ai);
    *ai = e * sin(dt * Ai);
    if (disc == DISC_ZOH_S6) { *gr = dt; *gi = 0.0; }
    else if (disc == DISC_DIRAC) { *gr = 1.0; *gi = 0.0; }
    else {                                   /* exact ZOH: g = (a - 1) / A */
        if (Ar == 0.0 && Ai == 0.0) { *gr = dt; *gi = 0.0; return; }
        /* a - 1 without cancellation: exp(z) - 1 = expm1(zr) cos(zi) + (cos(zi) - 1) + i e^{zr} sin(zi),
         * and cos(zi) - 1 = -2 sin^2(zi/2) */
        double zr = dt * Ar, zi = dt * Ai, sh = sin(0.5 * zi);
        double mr = expm1(zr) * cos(zi) - 2.0 * sh * sh, mi = e * sin(zi);
        double den = Ar * Ar + Ai * Ai;
        *gr = (mr * Ar + mi * Ai) / den;
        *gi = (mi * Ar - mr * Ai) / den;
    }
}

/* Forward selective scan with a complex diagonal state matrix (the recurrence of Eq. 2 for the complex-diagonal
 * layers of Sec. 2.2.1 when their step size or maps depend on the input):
 *     x_{l,n} = a(Delta_l, A[d,n]) x_{l-1,n} + g(Delta_l, A[d,n]) Bm[b,l,n] u[b,d,l]      (complex)
 *     y[b,d,l] = Re( sum_n Cm[b,l,n] x_{l,n} ) + Dskip[d] u[b,d,l],   then the optional gate.
 * A [D,N], Bm, Cm [B,G,L,N] (channel d reads group d / (D/G); G = 1: [B,L,N]), x0, x_last [B,D,N] are complex
 * ((re, im) pairs of doubles); u, delta, z, y, Dskip, delta_bias real.  Optional (NULL allowed): Dskip, delta_bias, z, x0, x_last.                                 */
int lrnnx_oracle_selective_scan_fwd_complex(
    int B, int D, int N, int G, long L, int disc, int delta_softplus,
    const double *u, const double *delta, const double *A,
    const double *Bm, const double *Cm, const double *Dskip,
    const double *delta_bias, const double *z, const double *x0,
    double *y, double *x_last)
{
    if (B < 0 || D < 0 || N < 1 || L < 0 || disc < 0 || disc > 3 || G < 1 || D % G) return 1;
    long rows = (long)B * D;
#pragma omp parallel for schedule(static)
    for (long row = 0; row < rows; ++row) {
        int b = (int)(row / D), d = (int)(row % D);
        long bg = (long)b * G + d / (D / G);          /* row of Bm, Cm this channel reads: its batch entry and group */
        double *x = (double *)malloc(sizeof(double) * 2 * N);
        for (int n = 0; n < 2 * N; ++n) x[n] = x0 ? x0[row * 2 * N + n] : 0.0;
        for (long l = 0; l < L; ++l) {
            double s = delta[row * L + l] + (delta_bias ? delta_bias[d] : 0.0);
            double dt = delta_softplus ? softplus(s) : s;
            double uu = u[row * L + l];
            double acc = 0.0;
            for (int n = 0; n < N; ++n) {
                double ar, ai, gr, gi;
                disc_eval_c(disc, dt, A[2 * ((long)d * N + n)], A[2 * ((long)d * N + n) + 1], &ar, &ai, &gr, &gi);
                long bc = 2 * ((bg * L + l) * N + n);
                double br = (gr * Bm[bc] - gi * Bm[bc + 1]) * uu, bi = (gr * Bm[bc + 1] + gi * Bm[bc]) * uu;
                double xr = ar * x[2 * n] - ai * x[2 * n + 1] + br;
                double xi = ar * x[2 * n + 1] + ai * x[2 * n] + bi;
                x[2 * n] = xr; x[2 * n + 1] = xi;
                acc += Cm[bc] * xr - Cm[bc + 1] * xi;                       /* Re(C x) */
            }
            double ypre = acc + (Dskip ? Dskip[d] * uu : 0.0);
            if (z) { double zz = z[row * L + l]; ypre *= zz * sigmoid(zz); }
            y[row * L + l] = ypre;
        }
        if (x_last) for (int n = 0; n < 2 * N; ++n) x_last[row * 2 * N + n] = x[n];
        free(x);
    }
    return 0;
}

/* Reverse-mode derivative of the forward above for a given upstream dy.
 * Every state of a row is kept (L*N doubles) -- the oracle stores what the
 * GPU path recomputes.  Outputs dA, dD, dbias, dBm, dCm are overwritten.
 * Optional (may be NULL): Dskip, delta_bias, z, x0, dD, dbias, dz, dx0.       */
int lrnnx_oracle_selective_scan_bwd(
    int B, int D, int N, int G, long L, int disc, int delta_softplus,
    const double *u, const double *delta, const double *A,
    const double *Bm, const double *Cm, const double *Dskip,
    const double *delta_bias, const double *z, const double *x0,
    const double *dy,
    double *du, double *ddelta, double *dA, double *dBm, double *dCm,
    double *dD, double *dbias, double *dz, double *dx0)
{
    if (B < 0 || D < 0 || N < 1 || L < 0 || disc < 0 || disc > 3 || G < 1 || D % G) return 1;
    long nBC = (long)B * G * L * N;
    memset(dA, 0, sizeof(double) * (size_t)D * N);
    memset(dBm, 0, sizeof(double) * (size_t)nBC);
    memset(dCm, 0, sizeof(double) * (size_t)nBC);
    if (dD) memset(dD, 0, sizeof(double) * (size_t)D);
    if (dbias) memset(dbias, 0, sizeof(double) * (size_t)D);

    int nthreads = lrnnx_oracle_num_threads();
    /* dBm, dCm sum over channels: one private copy per thread, added up at the end. */
    double *privB = (double *)calloc((size_t)nthreads * nBC, sizeof(double));
    double *privC = (double *)calloc((size_t)nthreads * nBC, sizeof(double));
    if (!privB || !privC) { free(privB); free(privC); return 2; }

#pragma omp parallel for schedule(static)
    for (int d = 0; d < D; ++d) {           /* dA, dD, dbias are per channel: no race */
#ifdef _OPENMP
        int tid = omp_get_thread_num();
#else
        int tid = 0;
#endif
        double *pB = privB + (size_t)tid * nBC, *pC = privC + (size_t)tid * nBC;
        double *xs = (double *)malloc(sizeof(double) * (size_t)(L + 1) * N); /* xs[(l+1)*N+n] = x_l, xs[n] = x_{-1} */
        double *h = (double *)malloc(sizeof(double) * N);
        for (int b = 0; b < B; ++b) {
            long row = (long)b * D + d;
            long bg = (long)b * G + d / (D / G);      /* row of Bm, Cm, dBm, dCm of this channel's group */
            for (int n = 0; n < N; ++n) xs[n] = x0 ? x0[row * N + n] : 0.0;
            for (long l = 0; l < L; ++l) {                      /* forward sweep, states kept */
                double s = delta[row * L + l] + (delta_bias ? delta_bias[d] : 0.0);
                double dt = delta_softplus ? softplus(s) : s;
                double uu = u[row * L + l];
                for (int n = 0; n < N; ++n) {
                    double a, g;
                    disc_eval(disc, dt, A[(long)d * N + n], &a, &g, 0, 0, 0, 0);
                    xs[(l + 1) * N + n] = a * xs[l * N + n] + g * Bm[(bg * L + l) * N + n] * uu;
                }
            }
            for (int n = 0; n < N; ++n) h[n] = 0.0;            /* h[n] = a_{l+1} * (dLoss/dx_{l+1}), zero past the end */
            for (long l = L - 1; l >= 0; --l) {                 /* reverse sweep */
                double s = delta[row * L + l] + (delta_bias ? delta_bias[d] : 0.0);
                double dt = delta_softplus ? softplus(s) : s;
                double uu = u[row * L + l];
                double acc = 0.0;
                for (int n = 0; n < N; ++n) acc += Cm[(bg * L + l) * N + n] * xs[(l + 1) * N + n];
                double ypre = acc + (Dskip ? Dskip[d] * uu : 0.0);
                double dypre = dy[row * L + l];
                if (z) {
                    double zz = z[row * L + l], sg = sigmoid(zz);
                    if (dz) dz[row * L + l] = dypre * ypre * sg * (1.0 + zz * (1.0 - sg));
                    dypre *= zz * sg;
                }
                if (dD && Dskip) dD[d] += dypre * uu;
                double du_l = Dskip ? dypre * Dskip[d] : 0.0;
                double ddt = 0.0;
                for (int n = 0; n < N; ++n) {
                    long bc = (bg * L + l) * N + n;
                    double a, g, a_t, a_A, g_t, g_A;
                    disc_eval(disc, dt, A[(long)d * N + n], &a, &g, &a_t, &a_A, &g_t, &g_A);
                    double hx = Cm[bc] * dypre + h[n];           /* dLoss/dx_l */
                    pC[bc] += dypre * xs[(l + 1) * N + n];
                    double da = hx * xs[l * N + n];              /* x_l = a x_{l-1} + g Bm u */
                    double dg = hx * Bm[bc] * uu;
                    pB[bc] += hx * g * uu;
                    du_l += hx * g * Bm[bc];
                    ddt += da * a_t + dg * g_t;
                    dA[(long)d * N + n] += da * a_A + dg * g_A;
                    h[n] = a * hx;
                }
                double ds = delta_softplus ? ddt * sigmoid(s) : ddt;   /* d softplus / ds = sigmoid */
                ddelta[row * L + l] = ds;
                if (dbias && delta_bias) dbias[d] += ds;
                du[row * L + l] = du_l;
            }
            if (dx0) for (int n = 0; n < N; ++n) dx0[row * N + n] = h[n];
        }
        free(xs); free(h);
    }
    for (int t = 0; t < nthreads; ++t)
        for (long i = 0; i < nBC; ++i) {
            dBm[i] += privB[(size_t)t * nBC + i];
            dCm[i] += privC[(size_t)t * nBC + i];
        }
    free(privB); free(privC);
    return 0;
}

/* Complex discretisation with its partial derivatives.  a and g are holomorphic in A and differentiable in the real
 * step dt; the four partials are ordinary complex derivatives (d/d dt along the real axis, d/dA complex).      */
static void disc_eval_cd(int disc, double dt, double complex A, double complex *a, double complex *g,
                         double complex *a_t, double complex *a_A, double complex *g_t, double complex *g_A)
{
    if (disc == DISC_BILINEAR) {
        double complex q = 1.0 / (1.0 - 0.5 * dt * A);
        *a = (1.0 + 0.5 * dt * A) * q;
        *g = dt * q;
        *a_t = A * q * q;
        *a_A = dt * q * q;
        *g_t = q * q;
        *g_A = 0.5 * dt * dt * q * q;
        return;
    }
    double complex zc = dt * A;
    *a = cexp(zc);
    *a_t = A * (*a);
    *a_A = dt * (*a);
    if (disc == DISC_ZOH_S6) { *g = dt; *g_t = 1.0; *g_A = 0.0; }
    else if (disc == DISC_DIRAC) { *g = 1.0; *g_t = 0.0; *g_A = 0.0; }
    else {                                   /* exact ZOH: g = (a - 1) / A = dt (e^z - 1) / z */
        *g_t = *a;
        if (cabs(zc) < 1e-3) {
            /* (e^z - 1)/z = 1 + z/2 + z^2/6 + z^3/24 + ...;  d/dA of g = dt^2 (z e^z - e^z + 1)/z^2
             * = dt^2 (1/2 + z/3 + z^2/8 + z^3/30 + ...): the omitted terms are below 1e-14 relative here */
            *g = dt * (1.0 + zc * (0.5 + zc * (1.0 / 6.0 + zc * (1.0 / 24.0 + zc / 120.0))));
            *g_A = dt * dt * (0.5 + zc * (1.0 / 3.0 + zc * (0.125 + zc * (1.0 / 30.0 + zc / 144.0))));
        } else {
            *g = (*a - 1.0) / A;
            *g_A = (zc * (*a) - (*a - 1.0)) / (A * A);
        }
    }
}

/* Expose the complex discretisation so the tests can pin it: out = (a, g, a_t, a_A, g_t, g_A) as (re, im) pairs. */
void lrnnx_oracle_disc_complex(int disc, double dt, double Ar, double Ai, double *out12)
{
    double complex v[6];
    disc_eval_cd(disc, dt, Ar + Ai * I, &v[0], &v[1], &v[2], &v[3], &v[4], &v[5]);
    for (int i = 0; i < 6; ++i) { out12[2 * i] = creal(v[i]); out12[2 * i + 1] = cimag(v[i]); }
}

/* Reverse-mode derivative of lrnnx_oracle_selective_scan_fwd_complex for a given upstream dy (real).
 * The gradient of the real loss with respect to a complex quantity q is written dLoss/dRe q + i dLoss/dIm q
 * (the convention of complex automatic differentiation); with it, for w = p q (complex product),
 * grad p = grad w * conj(q), and for y = Re(c x), grad x = dy conj(c), grad c = dy conj(x).  A real input that
 * enters a complex expression receives the real part.
 * Complex ((re, im) pairs): A, dA [D,N]; Bm, Cm, dBm, dCm [B,G,L,N] (G = 1: [B,L,N]); x0, dx0 [B,D,N].  Real: u, delta, z, dy, du,
 * ddelta, dz [B,D,L]; Dskip, delta_bias, dD, dbias [D].  dA, dBm, dCm, dD, dbias are overwritten.
 * Optional (may be NULL): Dskip, delta_bias, z, x0, dD, dbias, dz, dx0.                                        */
int lrnnx_oracle_selective_scan_bwd_complex(
    int B, int D, int N, int G, long L, int disc, int delta_softplus,
    const double *u, const double *delta, const double *A_,
    const double *Bm_, const double *Cm_, const double *Dskip,
    const double *delta_bias, const double *z, const double *x0_,
    const double *dy,
    double *du, double *ddelta, double *dA_, double *dBm_, double *dCm_,
    double *dD, double *dbias, double *dz, double *dx0_)
{
    if (B < 0 || D < 0 || N < 1 || L < 0 || disc < 0 || disc > 3 || G < 1 || D % G) return 1;
    const double complex *A = (const double complex *)A_, *Bm = (const double complex *)Bm_;
    const double complex *Cm = (const double complex *)Cm_, *x0 = (const double complex *)x0_;
    double complex *dA = (double complex *)dA_, *dBm = (double complex *)dBm_;
    double complex *dCm = (double complex *)dCm_, *dx0 = (double complex *)dx0_;
    long nBC = (long)B * G * L * N;
    for (long i = 0; i < (long)D * N; ++i) dA[i] = 0.0;
    for (long i = 0; i < nBC; ++i) { dBm[i] = 0.0; dCm[i] = 0.0; }
    if (dD) memset(dD, 0, sizeof(double) * (size_t)D);
    if (dbias) memset(dbias, 0, sizeof(double) * (size_t)D);

    int nthreads = lrnnx_oracle_num_threads();
    double complex *privB = (double complex *)calloc((size_t)nthreads * nBC + 1, sizeof(double complex));
    double complex *privC = (double complex *)calloc((size_t)nthreads * nBC + 1, sizeof(double complex));
    if (!privB || !privC) { free(privB); free(privC); return 2; }

#pragma omp parallel for schedule(static)
    for (int d = 0; d < D; ++d) {
#ifdef _OPENMP
        int tid = omp_get_thread_num();
#else
        int tid = 0;
#endif
        double complex *pB = privB + (size_t)tid * nBC, *pC = privC + (size_t)tid * nBC;
        double complex *xs = (double complex *)malloc(sizeof(double complex) * (size_t)(L + 1) * N); /* xs[(l+1)N+n] = x_l */
        double complex *h = (double complex *)malloc(sizeof(double complex) * N);
        for (int b = 0; b < B; ++b) {
            long row = (long)b * D + d;
            long bg = (long)b * G + d / (D / G);      /* row of Bm, Cm, dBm, dCm of this channel's group */
            for (int n = 0; n < N; ++n) xs[n] = x0 ? x0[row * N + n] : 0.0;
            for (long l = 0; l < L; ++l) {                      /* forward sweep, states kept */
                double s = delta[row * L + l] + (delta_bias ? delta_bias[d] : 0.0);
                double dt = delta_softplus ? softplus(s) : s;
                double uu = u[row * L + l];
                for (int n = 0; n < N; ++n) {
                    double complex a, g, t0, t1, t2, t3;
                    disc_eval_cd(disc, dt, A[(long)d * N + n], &a, &g, &t0, &t1, &t2, &t3);
                    xs[(l + 1) * N + n] = a * xs[l * N + n] + g * Bm[(bg * L + l) * N + n] * uu;
                }
            }
            for (int n = 0; n < N; ++n) h[n] = 0.0;            /* h[n] = conj(a_{l+1}) grad x_{l+1}, zero past the end */
            for (long l = L - 1; l >= 0; --l) {                 /* reverse sweep */
                double s = delta[row * L + l] + (delta_bias ? delta_bias[d] : 0.0);
                double dt = delta_softplus ? softplus(s) : s;
                double uu = u[row * L + l];
                double acc = 0.0;
                for (int n = 0; n < N; ++n) acc += creal(Cm[(bg * L + l) * N + n] * xs[(l + 1) * N + n]);
                double ypre = acc + (Dskip ? Dskip[d] * uu : 0.0);
                double dypre = dy[row * L + l];
                if (z) {
                    double zz = z[row * L + l], sg = sigmoid(zz);
                    if (dz) dz[row * L + l] = dypre * ypre * sg * (1.0 + zz * (1.0 - sg));
                    dypre *= zz * sg;
                }
                if (dD && Dskip) dD[d] += dypre * uu;
                double du_l = Dskip ? dypre * Dskip[d] : 0.0;
                double ddt = 0.0;
                for (int n = 0; n < N; ++n) {
                    long bc = (bg * L + l) * N + n;
                    double complex a, g, a_t, a_A, g_t, g_A;
                    disc_eval_cd(disc, dt, A[(long)d * N + n], &a, &g, &a_t, &a_A, &g_t, &g_A);
                    double complex hx = dypre * conj(Cm[bc]) + h[n];        /* grad x_l */
                    pC[bc] += dypre * conj(xs[(l + 1) * N + n]);
                    double complex ga = hx * conj(xs[l * N + n]);           /* grad a_l:  x_l = a x_{l-1} + g Bm u */
                    double complex gg = hx * conj(Bm[bc]) * uu;             /* grad g_l */
                    pB[bc] += hx * conj(g) * uu;
                    du_l += creal(hx * conj(g * Bm[bc]));
                    ddt += creal(ga * conj(a_t)) + creal(gg * conj(g_t));
                    dA[(long)d * N + n] += ga * conj(a_A) + gg * conj(g_A);
                    h[n] = conj(a) * hx;
                }
                double ds = delta_softplus ? ddt * sigmoid(s) : ddt;
                ddelta[row * L + l] = ds;
                if (dbias && delta_bias) dbias[d] += ds;
                du[row * L + l] = du_l;
            }
            if (dx0) for (int n = 0; n < N; ++n) dx0[row * N + n] = h[n];
        }
        free(xs); free(h);
    }
    for (int t = 0; t < nthreads; ++t)
        for (long i = 0; i < nBC; ++i) {
            dBm[i] += privB[(size_t)t * nBC + i];
            dCm[i] += privC[(size_t)t * nBC + i];
        }
    free(privB); free(privC);
    return 0;
}

/* Time-invariant complex-diagonal recurrence (S5 / LRU, Sec. 2.2.1):
 *     x_k = lambda (.) x_{k-1} + v_k,   v_k = Bbar u_k supplied by the caller.
 * Complex numbers are (re, im) pairs of doubles.  x0 may be NULL (zero).      */
int lrnnx_oracle_lti_diag_scan(int B, long L, int P,
                               const double *lambda, const double *v,
                               const double *x0, double *x)
{
    if (B < 0 || L < 0 || P < 0) return 1;
    long rows = (long)B * P;
#pragma omp parallel for schedule(static)
    for (long row = 0; row < rows; ++row) {
        int b = (int)(row / P), p = (int)(row % P);
        double lr = lambda[2 * p], li = lambda[2 * p + 1];
        double xr = x0 ? x0[2 * row] : 0.0, xi = x0 ? x0[2 * row + 1] : 0.0;
        for (long k = 0; k < L; ++k) {
            long idx = 2 * (((long)b * L + k) * P + p);
            double nr = lr * xr - li * xi + v[idx];
            double ni = lr * xi + li * xr + v[idx + 1];
            xr = nr; xi = ni;
            x[idx] = xr; x[idx + 1] = xi;
        }
    }
    return 0;
}

/* Time-varying diagonal recurrence with the per-step coefficients supplied by the caller:
 *     x_k = a_k (.) x_{k-1} + b_k          (Eq. 2 with A(k) = diag(a_k) and b_k = B(k) u_k already formed)
 * the form shared by the time-varying S5-style layers of Sec. 2.2.2 (S7), the gated real recurrence (RG-LRU)
 * and event-driven discretisation (Sec. 3), whose gates and step sizes are computed by the caller.
 * a, b, x: [B, L, P]; x0: [B, P] or NULL.  is_complex = 0: doubles; 1: (re, im) pairs of doubles.            */
int lrnnx_oracle_diag_scan(int B, long L, int P, int is_complex,
                           const double *a, const double *b, const double *x0, double *x)
{
    if (B < 0 || L < 0 || P < 0) return 1;
    long rows = (long)B * P;
#pragma omp parallel for schedule(static)
    for (long row = 0; row < rows; ++row) {
        int bb = (int)(row / P), p = (int)(row % P);
        if (!is_complex) {
            double xr = x0 ? x0[row] : 0.0;
            for (long k = 0; k < L; ++k) {
                long idx = ((long)bb * L + k) * P + p;
                xr = a[idx] * xr + b[idx];
                x[idx] = xr;
            }
        } else {
            double xr = x0 ? x0[2 * row] : 0.0, xi = x0 ? x0[2 * row + 1] : 0.0;
            for (long k = 0; k < L; ++k) {
                long idx = 2 * (((long)bb * L + k) * P + p);
                double nr = a[idx] * xr - a[idx + 1] * xi + b[idx];
                double ni = a[idx] * xi + a[idx + 1] * xr + b[idx + 1];
                xr = nr; xi = ni;
                x[idx] = xr; x[idx + 1] = xi;
            }
        }
    }
    return 0;
}

/* Backward of the recurrence with caller-supplied coefficients x_k = a_k x_{k-1} + b_k.  gx_k is the gradient of a
 * real loss reaching x_k (for complex data: dLoss/dRe + i dLoss/dIm, and the chain rule multiplies by conjugates):
 *     g_k  = gx_k + conj(a_{k+1}) g_{k+1},  g_{L+1} = 0
 *     db_k = g_k,   da_k = conj(x_{k-1}) g_k,   dx0 = conj(a_1) g_1            (k = 1..L, x_0 the initial state)
 * The states are recomputed here from (a, b, x0).                                                              */
int lrnnx_oracle_diag_scan_bwd(int B, long L, int P, int is_complex,
                               const double *a, const double *b, const double *x0, const double *gx,
                               double *da, double *db, double *dx0)
{
    if (B < 0 || L < 0 || P < 0) return 1;
    long rows = (long)B * P;
    int c = is_complex ? 2 : 1;
#pragma omp parallel
    {
        double *xs = (double *)malloc(sizeof(double) * 2 * (size_t)(L + 1));
#pragma omp for schedule(static)
        for (long row = 0; row < rows; ++row) {
            int bb = (int)(row / P), p = (int)(row % P);
            xs[0] = x0 ? x0[c * row] : 0.0;
            xs[1] = (x0 && is_complex) ? x0[c * row + 1] : 0.0;
            for (long k = 0; k < L; ++k) {                          /* x after step k in slot k+1 */
                long idx = c * (((long)bb * L + k) * P + p);
                double ar = a[idx], ai = is_complex ? a[idx + 1] : 0.0;
                double br = b[idx], bi = is_complex ? b[idx + 1] : 0.0;
                xs[2 * (k + 1)]     = ar * xs[2 * k] - ai * xs[2 * k + 1] + br;
                xs[2 * (k + 1) + 1] = ar * xs[2 * k + 1] + ai * xs[2 * k] + bi;
            }
            double hr = 0.0, hi = 0.0;                               /* conj(a_{k+1}) g_{k+1}, carried backwards */
            for (long k = L - 1; k >= 0; --k) {
                long idx = c * (((long)bb * L + k) * P + p);
                double gr = gx[idx] + hr, gi = (is_complex ? gx[idx + 1] : 0.0) + hi;
                db[idx] = gr;
                da[idx] = xs[2 * k] * gr + xs[2 * k + 1] * gi;       /* conj(x_{k-1}) g_k */
                if (is_complex) {
                    db[idx + 1] = gi;
                    da[idx + 1] = xs[2 * k] * gi - xs[2 * k + 1] * gr;
                }
                double ar = a[idx], ai = is_complex ? a[idx + 1] : 0.0;
                hr = ar * gr + ai * gi;                              /* conj(a_k) g_k */
                hi = ar * gi - ai * gr;
            }
            if (dx0) { dx0[c * row] = hr; if (is_complex) dx0[c * row + 1] = hi; }
        }
        free(xs);
    }
    return 0;
}

/* Backward of the time-invariant complex-diagonal recurrence (the adjoint recurrence of Sec. 2.2.1's
 * x_k = lambda x_{k-1} + v_k).  A real loss depends on x through gx_k = dLoss/dRe(x_k) + i dLoss/dIm(x_k);
 * gradients of complex quantities follow the same convention.  Because x_k is holomorphic in x_{k-1}, v_k and
 * lambda, the chain rule multiplies by the CONJUGATE of the holomorphic derivative:
 *     g_k   = gx_k + conj(lambda) g_{k+1},  g_{L+1} = 0     (total gradient reaching x_k)
 *     dv_k  = g_k
 *     dx0   = conj(lambda) g_1
 *     dlam  = sum_b sum_k conj(x_{k-1}) g_k
 * The states are recomputed here from (lambda, v, x0); xs is a scratch row of L+1 complex numbers per thread.  */
int lrnnx_oracle_lti_diag_scan_bwd(int B, long L, int P,
                                   const double *lambda, const double *v, const double *x0,
                                   const double *gx, double *dv, double *dlambda, double *dx0)
{
    if (B < 0 || L < 0 || P < 0) return 1;
#pragma omp parallel
    {
        double *xs = (double *)malloc(sizeof(double) * 2 * (size_t)(L + 1));
#pragma omp for schedule(static)
        for (int p = 0; p < P; ++p) {
            double lr = lambda[2 * p], li = lambda[2 * p + 1];
            double dlr = 0.0, dli = 0.0;
            for (int b = 0; b < B; ++b) {
                long row = (long)b * P + p;
                xs[0] = x0 ? x0[2 * row] : 0.0;
                xs[1] = x0 ? x0[2 * row + 1] : 0.0;
                for (long k = 0; k < L; ++k) {                      /* x_{k+1} in slot k+1 */
                    long idx = 2 * (((long)b * L + k) * P + p);
                    xs[2 * (k + 1)]     = lr * xs[2 * k] - li * xs[2 * k + 1] + v[idx];
                    xs[2 * (k + 1) + 1] = lr * xs[2 * k + 1] + li * xs[2 * k] + v[idx + 1];
                }
                double gr = 0.0, gi = 0.0;                          /* conj(lambda) g_{k+1}, carried backwards */
                for (long k = L - 1; k >= 0; --k) {
                    long idx = 2 * (((long)b * L + k) * P + p);
                    double tr = gx[idx] + gr, ti = gx[idx + 1] + gi;   /* g_k */
                    dv[idx] = tr; dv[idx + 1] = ti;
                    /* conj(x_{k-1}) g_k : (xr - i xi)(tr + i ti) */
                    dlr += xs[2 * k] * tr + xs[2 * k + 1] * ti;
                    dli += xs[2 * k] * ti - xs[2 * k + 1] * tr;
                    /* conj(lambda) g_k : (lr - i li)(tr + i ti) */
                    gr = lr * tr + li * ti;
                    gi = lr * ti - li * tr;
                }
                if (dx0) { dx0[2 * row] = gr; dx0[2 * row + 1] = gi; }
            }
            dlambda[2 * p] = dlr; dlambda[2 * p + 1] = dli;
        }
        free(xs);
    }
    return 0;
}

/* Single-token update (the `step` method of Sec. 3, "Library Design"): one application of
 * Eq. 2 to a carried state.  x[B,D,N] is updated in place; u, delta, z, y are [B,D];
 * Bm, Cm are [B,G,N] (channel d reads group d / (D/G); G = 1: [B,N]).  Optional (NULL allowed): Dskip,
 * delta_bias, z.                                                                      */
int lrnnx_oracle_selective_step(
    int B, int D, int N, int G, int disc, int delta_softplus,
    double *x, const double *u, const double *delta, const double *A,
    const double *Bm, const double *Cm, const double *Dskip,
    const double *delta_bias, const double *z, double *y)
{
    if (B < 0 || D < 0 || N < 1 || disc < 0 || disc > 3 || G < 1 || D % G) return 1;
    for (int b = 0; b < B; ++b)
        for (int d = 0; d < D; ++d) {
            long row = (long)b * D + d;
            long bg = (long)b * G + d / (D / G);
            double s = delta[row] + (delta_bias ? delta_bias[d] : 0.0);
            double dt = delta_softplus ? softplus(s) : s;
            double acc = 0.0;
            for (int n = 0; n < N; ++n) {
                double a, g;
                disc_eval(disc, dt, A[(long)d * N + n], &a, &g, 0, 0, 0, 0);
                x[row * N + n] = a * x[row * N + n] + g * Bm[bg * N + n] * u[row];
                acc += Cm[bg * N + n] * x[row * N + n];
            }
            double ypre = acc + (Dskip ? Dskip[d] * u[row] : 0.0);
            if (z) ypre *= z[row] * sigmoid(z[row]);
            y[row] = ypre;
        }
    return 0;
}

/* Single-token update with a complex diagonal A (the `step` method for the complex-A selective scan): one
 * application of the recurrence of lrnnx_oracle_selective_scan_fwd_complex to a carried complex state.  x[B,D,N]
 * complex, updated in place; u, delta, z, y [B,D] real; A [D,N], Bm, Cm [B,G,N] complex (G = 1: [B,N]).  Optional: Dskip,
 * delta_bias, z.                                                                                              */
int lrnnx_oracle_selective_step_complex(
    int B, int D, int N, int G, int disc, int delta_softplus,
    double *x_, const double *u, const double *delta, const double *A_,
    const double *Bm_, const double *Cm_, const double *Dskip,
    const double *delta_bias, const double *z, double *y)
{
    if (B < 0 || D < 0 || N < 1 || disc < 0 || disc > 3 || G < 1 || D % G) return 1;
    double complex *x = (double complex *)x_;
    const double complex *A = (const double complex *)A_, *Bm = (const double complex *)Bm_;
    const double complex *Cm = (const double complex *)Cm_;
    for (int b = 0; b < B; ++b)
        for (int d = 0; d < D; ++d) {
            long row = (long)b * D + d;
            double s = delta[row] + (delta_bias ? delta_bias[d] : 0.0);
            double dt = delta_softplus ? softplus(s) : s;
            double acc = 0.0;
            for (int n = 0; n < N; ++n) {
                double complex a, g, t0, t1, t2, t3;
                disc_eval_cd(disc, dt, A[(long)d * N + n], &a, &g, &t0, &t1, &t2, &t3);
                long bg = (long)b * G + d / (D / G);
                x[row * N + n] = a * x[row * N + n] + g * Bm[bg * N + n] * u[row];
                acc += creal(Cm[bg * N + n] * x[row * N + n]);
            }
            double ypre = acc + (Dskip ? Dskip[d] * u[row] : 0.0);
            if (z) ypre *= z[row] * sigmoid(z[row]);
            y[row] = ypre;
        }
    return 0;
}

/* Single-token update of the LTI complex-diagonal recurrence: x[B,P] <- lambda (.) x + v[B,P]. */
int lrnnx_oracle_lti_step(int B, int P, const double *lambda, double *x, const double *v)
{
    if (B < 0 || P < 0) return 1;
    for (int b = 0; b < B; ++b)
        for (int p = 0; p < P; ++p) {
            long i = 2 * ((long)b * P + p);
            double nr = lambda[2 * p] * x[i] - lambda[2 * p + 1] * x[i + 1] + v[i];
            double ni = lambda[2 * p] * x[i + 1] + lambda[2 * p + 1] * x[i] + v[i + 1];
            x[i] = nr; x[i + 1] = ni;
        }
    return 0;
}
