/*
 * heinsen_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, float64 CPU evaluation of the first-order linear recurrence
 *
 *        x_t = a_t * x_{t-1} + b_t ,   t = 1..n ,   x_0 given          (paper, Abstract / Sec. 3)
 *
 * in two independent ways:
 *
 *   O1  the definition itself, one step at a time (Sec. 3, first sentence), and the same loop taken
 *       in the log domain for strictly positive data;
 *   O2  the paper's closed form, Eq. (1)-(2) as stabilised in Sec. 4 (the LCSE expression), followed
 *       step by step with complex logarithms so that negative a_t, b_t, x_0 are legal (Sec. 1, last
 *       paragraph).
 *
 * Nothing here is blocked, fused or reordered beyond what those passages state.  This file shares no
 * code with the GPU library and is never linked into it; only tests, the smoke check and the CPU leg
 * of the benchmark may call it.
 *
 * Pins (see tests/test_oracle_pins.py): exact rational expansion of Eq. (4) for n <= 16, geometric
 * closed form, running product, running sum, numpy.logaddexp.accumulate for the LCSE step, the
 * "imaginary part is a multiple of pi" identity, split invariance, and O1 == O2.
 *
 * Build:  gcc -O2 -ffp-contract=off -fno-fast-math -fopenmp -shared -fPIC heinsen_oracle.c -lm
 */
#include <complex.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

#define ORACLE_LAYOUT_BND 0 /* [B, n, D]: element (b,t,d) at ((b*n + t)*D + d) */
#define ORACLE_LAYOUT_BDN 1 /* [B, D, n]: element (b,t,d) at ((b*D + d)*n + t) */

/* ---------------------------------------------------------------------------------------------
 * O1, single sequence, float64 inputs.  Sec. 3: x_t = a_t x_{t-1} + b_t.
 * out[t-1] = x_t for t = 1..n (x_0 is an input and is not emitted, matching tail() in Sec. 4).
 * ------------------------------------------------------------------------------------------- */
void oracle_seq_f64(const double *a, const double *b, double x0, double *out, int64_t n)
{
    double x = x0;
    for (int64_t t = 0; t < n; ++t) {
        double prod = a[t] * x; /* product and sum rounded separately (-ffp-contract=off) */
        x = prod + b[t];
        out[t] = x;
    }
}

static void channel_geometry(int layout, int64_t D, int64_t n, int64_t ch, int64_t *base, int64_t *stride)
{
    int64_t bb = ch / D, d = ch % D;
    if (layout == ORACLE_LAYOUT_BND) {
        *base = bb * n * D + d;
        *stride = D;
    } else {
        *base = (bb * D + d) * n;
        *stride = 1;
    }
}

/* ---------------------------------------------------------------------------------------------
 * O1, batched: B*D independent sequences stored as float32 in either layout, widened exactly to
 * float64.  x0 has B*D entries (or one, if x0_scalar).  out has the layout of a and b, in float64.
 * threads <= 1 means a single thread; channels are independent so they may be split over threads.
 * ------------------------------------------------------------------------------------------- */
void oracle_sequential_f32in(const float *a, const float *b, const float *x0, double *out, int64_t B,
                             int64_t D, int64_t n, int layout, int x0_scalar, int threads)
{
    int64_t C = B * D;
    if (threads < 1) threads = 1;
#pragma omp parallel for num_threads(threads) schedule(static)
    for (int64_t ch = 0; ch < C; ++ch) {
        int64_t base, stride;
        channel_geometry(layout, D, n, ch, &base, &stride);
        double x = (double)(x0_scalar ? x0[0] : x0[ch]);
        for (int64_t t = 0; t < n; ++t) {
            int64_t i = base + t * stride;
            double prod = (double)a[i] * x;
            x = prod + (double)b[i];
            out[i] = x;
        }
    }
}

/* log(e^p + e^q) for real p, q (either may be -inf).  Sec. 4: the log-sum-exp trick. */
static double lae_f64(double p, double q)
{
    double m = p > q ? p : q;
    double lo = p > q ? q : p;
    if (m == -INFINITY) return -INFINITY;
    if (m == INFINITY) return INFINITY;
    return m + log1p(exp(lo - m));
}

/* ---------------------------------------------------------------------------------------------
 * O1 in the log domain, for strictly positive data given as logarithms:
 *   log x_t = log( e^{log a_t + log x_{t-1}} + e^{log b_t} )
 * which is the logarithm of the definition in Sec. 3 term by term.  Inputs float32 logs (widened
 * exactly), output float64 log x_t, same layouts as above.
 * ------------------------------------------------------------------------------------------- */
void oracle_sequential_log_f32in(const float *log_a, const float *log_b, const float *log_x0,
                                 double *out_log, int64_t B, int64_t D, int64_t n, int layout,
                                 int x0_scalar, int threads)
{
    int64_t C = B * D;
    if (threads < 1) threads = 1;
#pragma omp parallel for num_threads(threads) schedule(static)
    for (int64_t ch = 0; ch < C; ++ch) {
        int64_t base, stride;
        channel_geometry(layout, D, n, ch, &base, &stride);
        double lx = (double)(x0_scalar ? log_x0[0] : log_x0[ch]);
        for (int64_t t = 0; t < n; ++t) {
            int64_t i = base + t * stride;
            lx = lae_f64(lx + (double)log_a[i], (double)log_b[i]);
            out_log[i] = lx;
        }
    }
}

/* ---------------------------------------------------------------------------------------------
 * O2 building blocks (complex128).
 * ------------------------------------------------------------------------------------------- */

/* principal complex log of a real number: log|v| + i*pi for v < 0, -inf + 0i for v == 0 */
static double complex clog_real(double v)
{
    if (v == 0.0) return CMPLX(-INFINITY, 0.0);
    if (v < 0.0) return CMPLX(log(-v), M_PI);
    return CMPLX(log(v), 0.0);
}

/* complex exp that maps real part -inf to exactly 0 (cexp(-inf + iy) may carry signed zeros/NaN) */
static double complex cexp_safe(double complex z)
{
    if (creal(z) == -INFINITY) return 0.0;
    return cexp(z);
}

/* log(e^p + e^q) for complex p, q, shifted by the operand of larger real part */
static double complex clae(double complex p, double complex q)
{
    double complex m = creal(p) >= creal(q) ? p : q;
    if (creal(m) == -INFINITY) return CMPLX(-INFINITY, 0.0);
    double complex s = cexp_safe(p - m) + cexp_safe(q - m);
    if (s == 0.0) return CMPLX(-INFINITY, 0.0);
    return m + clog(s);
}

/* Sec. 4: LCSE(z) := log cumsum exp(z), running and max-shifted at every step.
 * in/out are interleaved (re, im) pairs; out[k] = log sum_{j<=k} exp(z_j). */
void oracle_lcse_c128(const double *z_re_im, double *out_re_im, int64_t n)
{
    double complex acc = CMPLX(-INFINITY, 0.0);
    for (int64_t k = 0; k < n; ++k) {
        double complex z = CMPLX(z_re_im[2 * k], z_re_im[2 * k + 1]);
        acc = (k == 0) ? z : clae(acc, z);
        out_re_im[2 * k] = creal(acc);
        out_re_im[2 * k + 1] = cimag(acc);
    }
}

/* ---------------------------------------------------------------------------------------------
 * O2, single sequence: Sec. 4,
 *     x_t = exp( a*_t + tail( LCSE( cat( log x_0, log b_t - a*_t ) ) ) ),
 *     a*_t = cumsum_t log a_t                                   (Eq. (2), first line)
 * with every logarithm taken in C (Sec. 1, last paragraph).
 * Outputs (each of length n, any may be NULL): x = Re exp(log x_t); logx_re, logx_im = log x_t.
 * Returns 0, or 1 if allocation failed.
 * ------------------------------------------------------------------------------------------- */
int oracle_logspace_c128(const double *a, const double *b, double x0, double *x, double *logx_re,
                         double *logx_im, int64_t n)
{
    double complex *astar = (double complex *)malloc((size_t)(n > 0 ? n : 1) * sizeof(double complex));
    double *z = (double *)malloc((size_t)(n + 1) * 2 * sizeof(double));
    double *l = (double *)malloc((size_t)(n + 1) * 2 * sizeof(double));
    if (!astar || !z || !l) {
        free(astar); free(z); free(l);
        return 1;
    }
    /* first prefix sum: a*_t */
    double complex run = 0.0;
    for (int64_t t = 0; t < n; ++t) {
        run = run + clog_real(a[t]);
        astar[t] = run;
    }
    /* cat(log x_0, log b_t - a*_t) */
    double complex lx0 = clog_real(x0);
    z[0] = creal(lx0);
    z[1] = cimag(lx0);
    for (int64_t t = 0; t < n; ++t) {
        double complex lb = clog_real(b[t]);
        double complex zt = (creal(lb) == -INFINITY) ? CMPLX(-INFINITY, 0.0) : lb - astar[t];
        if (creal(astar[t]) == -INFINITY && creal(lb) != -INFINITY) {
            /* a product of zero: b_t / 0 has no finite logarithm.  The closed form does not cover
             * this case (it divides by the running product, Eq. (4)); report NaN so a test that
             * feeds a_t = 0 to O2 fails loudly instead of comparing garbage. */
            zt = CMPLX(NAN, NAN);
        }
        z[2 * (t + 1)] = creal(zt);
        z[2 * (t + 1) + 1] = cimag(zt);
    }
    /* second prefix sum in the log domain */
    oracle_lcse_c128(z, l, n + 1);
    /* tail(), add a*_t, exponentiate */
    for (int64_t t = 0; t < n; ++t) {
        double complex lx = astar[t] + CMPLX(l[2 * (t + 1)], l[2 * (t + 1) + 1]);
        if (logx_re) logx_re[t] = creal(lx);
        if (logx_im) logx_im[t] = cimag(lx);
        if (x) x[t] = creal(cexp_safe(lx));
    }
    free(astar); free(z); free(l);
    return 0;
}

int oracle_max_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
