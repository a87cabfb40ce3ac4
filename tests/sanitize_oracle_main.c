/* Driver for the sanitizer build of the CPU oracle (tests/test_sanitizers.py compiles this file together with
 * oracle/lrnnx_oracle.c under -fsanitize=address,undefined).  Every exported oracle function is called on small
 * ragged shapes with heap buffers of exactly the documented sizes, so that an access past a buffer, a use of an
 * uninitialised output slot as input or any undefined arithmetic ends the run with a report.  Results are only
 * checked to be finite: what the oracle computes is pinned elsewhere (tests/test_oracle_pins.py).            */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

int lrnnx_oracle_selective_scan_fwd(int, int, int, int, long, int, int, const double *, const double *, const double *,
                                    const double *, const double *, const double *, const double *, const double *,
                                    const double *, double *, double *, double *);
int lrnnx_oracle_selective_scan_fwd_complex(int, int, int, int, long, int, int, const double *, const double *,
                                            const double *, const double *, const double *, const double *,
                                            const double *, const double *, const double *, double *, double *);
int lrnnx_oracle_selective_scan_bwd(int, int, int, int, long, int, int, const double *, const double *, const double *,
                                    const double *, const double *, const double *, const double *, const double *,
                                    const double *, const double *, double *, double *, double *, double *, double *,
                                    double *, double *, double *, double *);
int lrnnx_oracle_selective_scan_bwd_complex(int, int, int, int, long, int, int, const double *, const double *,
                                            const double *, const double *, const double *, const double *,
                                            const double *, const double *, const double *, const double *, double *,
                                            double *, double *, double *, double *, double *, double *, double *,
                                            double *);
int lrnnx_oracle_lti_diag_scan(int, long, int, const double *, const double *, const double *, double *);
int lrnnx_oracle_lti_diag_scan_bwd(int, long, int, const double *, const double *, const double *, const double *,
                                   double *, double *, double *);
int lrnnx_oracle_diag_scan(int, long, int, int, const double *, const double *, const double *, double *);
int lrnnx_oracle_diag_scan_bwd(int, long, int, int, const double *, const double *, const double *, const double *,
                               double *, double *, double *);
int lrnnx_oracle_selective_step(int, int, int, int, int, int, double *, const double *, const double *, const double *,
                                const double *, const double *, const double *, const double *, const double *,
                                double *);
int lrnnx_oracle_selective_step_complex(int, int, int, int, int, int, double *, const double *, const double *,
                                        const double *, const double *, const double *, const double *, const double *,
                                        const double *, double *);
int lrnnx_oracle_lti_step(int, int, const double *, double *, const double *);
void lrnnx_oracle_disc(int, double, double, double *);
void lrnnx_oracle_disc_complex(int, double, double, double, double *);
double lrnnx_oracle_softplus(double);

static unsigned long long rng_state = 0x9E3779B97F4A7C15ull;
static double rnd(void) {                       /* xorshift, uniform in (-1, 1) */
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
    return (double)(rng_state >> 11) / 4503599627370496.0 - 1.0;
}
static double *fresh(size_t n, double scale, double shift) {
    double *p = (double *)malloc((n ? n : 1) * sizeof(double));
    if (!p) exit(3);
    for (size_t i = 0; i < n; ++i) p[i] = shift + scale * rnd();
    return p;
}
static double *blank(size_t n) {                /* outputs start as NaN: a slot the oracle forgets to write is seen */
    double *p = (double *)malloc((n ? n : 1) * sizeof(double));
    if (!p) exit(3);
    for (size_t i = 0; i < n; ++i) p[i] = NAN;
    return p;
}
static int finite_all(const double *p, size_t n, const char *what) {
    for (size_t i = 0; i < n; ++i)
        if (!isfinite(p[i])) { fprintf(stderr, "%s[%zu] is not finite\n", what, i); return 0; }
    return 1;
}
#define CHECK(x) do { if (!(x)) { fprintf(stderr, "failed: %s (line %d)\n", #x, __LINE__); return 1; } } while (0)

static int selective(int B, int D, int N, int G, long L, int disc, int softplus, int cplx) {
    const size_t c = cplx ? 2 : 1, bdl = (size_t)B * D * L, bgln = (size_t)B * G * L * N * c, dn = (size_t)D * N * c,
                 bdn = (size_t)B * D * N * c;
    double *u = fresh(bdl, 1, 0), *dl = fresh(bdl, softplus ? 1 : 0.05, softplus ? 0 : 0.06), *A = fresh(dn, 0.4, -0.6);
    double *Bm = fresh(bgln, 1, 0), *Cm = fresh(bgln, 1, 0), *Dk = fresh(D, 1, 0), *bias = fresh(D, 1, -2), *z = fresh(bdl, 1, 0);
    double *x0 = fresh(bdn, 1, 0), *dy = fresh(bdl, 1, 0);
    double *y = blank(bdl), *xl = blank(bdn), *xs = cplx ? NULL : blank(bdl * N);
    double *du = blank(bdl), *dd = blank(bdl), *dA = blank(dn), *dB = blank(bgln), *dC = blank(bgln), *dD = blank(D),
           *db = blank(D), *dz = blank(bdl), *dx0 = blank(bdn);
    int rc;
    if (cplx) {
        rc = lrnnx_oracle_selective_scan_fwd_complex(B, D, N, G, L, disc, softplus, u, dl, A, Bm, Cm, Dk, bias, z, x0, y, xl);
        CHECK(rc == 0);
        rc = lrnnx_oracle_selective_scan_bwd_complex(B, D, N, G, L, disc, softplus, u, dl, A, Bm, Cm, Dk, bias, z, x0, dy,
                                                     du, dd, dA, dB, dC, dD, db, dz, dx0);
    } else {
        rc = lrnnx_oracle_selective_scan_fwd(B, D, N, G, L, disc, softplus, u, dl, A, Bm, Cm, Dk, bias, z, x0, y, xl, xs);
        CHECK(rc == 0 && finite_all(xs, bdl * N, "xs"));
        rc = lrnnx_oracle_selective_scan_bwd(B, D, N, G, L, disc, softplus, u, dl, A, Bm, Cm, Dk, bias, z, x0, dy,
                                             du, dd, dA, dB, dC, dD, db, dz, dx0);
    }
    CHECK(rc == 0);
    CHECK(finite_all(y, bdl, "y") && finite_all(xl, bdn, "x_last") && finite_all(du, bdl, "du") && finite_all(dd, bdl, "ddelta"));
    CHECK(finite_all(dA, dn, "dA") && finite_all(dB, bgln, "dBm") && finite_all(dC, bgln, "dCm") && finite_all(dD, D, "dD"));
    CHECK(finite_all(db, D, "dbias") && finite_all(dz, bdl, "dz") && finite_all(dx0, bdn, "dx0"));
    /* one token through the step functions, on the [B,D] slice at time 0 of contiguous copies */
    {
        double *us = fresh((size_t)B * D, 1, 0), *ds = fresh((size_t)B * D, 1, 0), *zs = fresh((size_t)B * D, 1, 0);
        double *Bs = fresh((size_t)B * G * N * c, 1, 0), *Cs = fresh((size_t)B * G * N * c, 1, 0), *ys = blank((size_t)B * D);
        rc = cplx ? lrnnx_oracle_selective_step_complex(B, D, N, G, disc, softplus, x0, us, ds, A, Bs, Cs, Dk, bias, zs, ys)
                  : lrnnx_oracle_selective_step(B, D, N, G, disc, softplus, x0, us, ds, A, Bs, Cs, Dk, bias, zs, ys);
        CHECK(rc == 0 && finite_all(ys, (size_t)B * D, "step y") && finite_all(x0, bdn, "step x"));
        free(us); free(ds); free(zs); free(Bs); free(Cs); free(ys);
    }
    /* optional inputs absent */
    if (!cplx) {
        rc = lrnnx_oracle_selective_scan_fwd(B, D, N, G, L, disc, softplus, u, dl, A, Bm, Cm, NULL, NULL, NULL, NULL, y, xl, NULL);
        CHECK(rc == 0);
        rc = lrnnx_oracle_selective_scan_bwd(B, D, N, G, L, disc, softplus, u, dl, A, Bm, Cm, NULL, NULL, NULL, NULL, dy,
                                             du, dd, dA, dB, dC, NULL, NULL, NULL, dx0);
        CHECK(rc == 0);
    }
    free(u); free(dl); free(A); free(Bm); free(Cm); free(Dk); free(bias); free(z); free(x0); free(dy);
    free(y); free(xl); free(xs); free(du); free(dd); free(dA); free(dB); free(dC); free(dD); free(db); free(dz); free(dx0);
    return 0;
}

static int chained(int B, long L, int P, int cplx) {
    const size_t c = cplx ? 2 : 1, blp = (size_t)B * L * P * c, bp = (size_t)B * P * c;
    double *a = fresh(blp, 0.45, 0.5), *b = fresh(blp, 1, 0), *x0 = fresh(bp, 1, 0), *gx = fresh(blp, 1, 0);
    double *x = blank(blp), *da = blank(blp), *db = blank(blp), *dx0 = blank(bp);
    CHECK(lrnnx_oracle_diag_scan(B, L, P, cplx, a, b, x0, x) == 0 && finite_all(x, blp, "diag x"));
    CHECK(lrnnx_oracle_diag_scan_bwd(B, L, P, cplx, a, b, x0, gx, da, db, dx0) == 0);
    CHECK(finite_all(da, blp, "da") && finite_all(db, blp, "db") && finite_all(dx0, bp, "diag dx0"));
    CHECK(lrnnx_oracle_diag_scan(B, L, P, cplx, a, b, NULL, x) == 0);
    if (cplx) {
        double *lam = fresh((size_t)P * 2, 0.6, 0), *dv = blank(blp), *dlam = blank((size_t)P * 2);
        CHECK(lrnnx_oracle_lti_diag_scan(B, L, P, lam, b, x0, x) == 0 && finite_all(x, blp, "lti x"));
        CHECK(lrnnx_oracle_lti_diag_scan_bwd(B, L, P, lam, b, x0, gx, dv, dlam, dx0) == 0);
        CHECK(finite_all(dv, blp, "dv") && finite_all(dlam, (size_t)P * 2, "dlambda") && finite_all(dx0, bp, "lti dx0"));
        CHECK(lrnnx_oracle_lti_step(B, P, lam, x0, b) == 0 && finite_all(x0, bp, "lti step"));
        free(lam); free(dv); free(dlam);
    }
    free(a); free(b); free(x0); free(gx); free(x); free(da); free(db); free(dx0);
    return 0;
}

int main(void) {
    double out[12];
    for (int disc = 0; disc < 4; ++disc) {
        lrnnx_oracle_disc(disc, 0.3, -0.7, out);
        lrnnx_oracle_disc(disc, 0.3, 0.0, out);
        lrnnx_oracle_disc_complex(disc, 0.3, -0.7, 2.0, out);
        lrnnx_oracle_disc_complex(disc, 0.3, 0.0, 0.0, out);
        for (int softplus = 0; softplus < 2; ++softplus)
            for (int cplx = 0; cplx < 2; ++cplx) {
                if (selective(2, 6, 4, 1, 37, disc, softplus, cplx)) return 1;
                if (selective(1, 6, 3, 3, 1, disc, softplus, cplx)) return 1;      /* grouped maps, one step */
            }
    }
    if (selective(3, 1, 16, 1, 300, 0, 1, 0)) return 1;
    for (int cplx = 0; cplx < 2; ++cplx)
        if (chained(2, 41, 5, cplx) || chained(1, 1, 1, cplx)) return 1;
    if (!isfinite(lrnnx_oracle_softplus(-800.0)) || !isfinite(lrnnx_oracle_softplus(800.0))) return 1;
    puts("sanitized oracle run ok");
    return 0;
}
