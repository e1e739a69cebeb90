/*
 * goom_oracle.c -- plain CPU oracle for generalized orders of magnitude (GOOMs).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement of
 * what the GPU library must compute.  It is not part of the product: nothing in the
 * product path may include, link, import or call it, and it shares no code, header,
 * table or constant with the HIP sources.
 *
 * Everything here is written from the paper's definitions:
 *   - a GOOM is a complex logarithm x' with exp(x') real; Re = log|x|, Im = an even
 *     multiple of pi for x >= 0 and an odd multiple for x < 0; zero is non-negative
 *     (Section 2, eq. 1 and the paragraph after it);
 *   - float -> GOOM and GOOM -> float maps (Section 3.1);
 *   - LMME(A', B') = log(exp(A') exp(B')) = LSE_j(A'_ij + B'_jk) (Section 3.2, eq. 9),
 *     written here in its definitional signed log-sum-exp form (Example 2), never the
 *     scaled-matmul shortcut of eq. 10;
 *   - matrix-product chains S'_t = LMME(A'_t, S'_{t-1}) (Section 4.1);
 *   - the linear recurrence with bias used for non-diagonal state-space models
 *     (Section 4.3, eqs. 25 and 26);
 *   - sequential QR estimation of Lyapunov spectra (Section 4.2.1, eqs. 19-20) and
 *     the selectively reset recurrence (Section 5; Appendix C);
 *   - backward passes: the redefined finite derivatives of the codecs (Section 3.1,
 *     eqs. 5, 6 and 8) and the adjoint recurrence of the linear recurrence with bias.
 *
 * Arithmetic: log-magnitudes are held in IEEE double, signs as one byte (0 = +, 1 = -).
 * Sums of exponentials accumulate in long double.  Codecs evaluate log/exp in
 * __float128 and round once to the component type, so they are correctly rounded for
 * every practical purpose.  OpenMP is used only across independent outputs of one
 * combine or across independent problems; every chain is walked strictly left to
 * right in t.
 *
 * Pins (tests/test_oracle_*.py, run without a GPU): closed forms and the paper's
 * printed examples for the codecs; brute-force extended-precision real products,
 * the exp(1000) dot-product example, shift/permutation invariances and d = 1 for
 * LMME; brute force, the worked scan of Appendix C and the Gaussian growth-rate
 * closed form for the scan; brute force and degenerate cases for the affine
 * recurrence; the Appendix C reset example, S == 0, the log|det| sum rule and the
 * Gaussian closed-form spectrum for the reset recurrence and the QR estimator;
 * central finite differences of a long-double evaluation over reals, the sum rule of
 * log-domain gradients and scalar closed forms for the backward passes.
 */
#include <math.h>
#include <quadmath.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <float.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_API __attribute__((visibility("default")))

/* ------------------------------------------------------------------------- */
/* threads                                                                    */
/* ------------------------------------------------------------------------- */

ORACLE_API int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

ORACLE_API void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ------------------------------------------------------------------------- */
/* codecs (Section 3.1)                                                       */
/* ------------------------------------------------------------------------- */

/* Sign of the real number a GOOM stands for: negative iff Im is an odd multiple of
 * pi (Section 2).  Rounding Im/pi to the nearest integer accepts any representative. */
static inline uint8_t sign_from_imag(double im)
{
    long long k = llround(im / M_PI);
    return (uint8_t)(k & 1LL);
}

/* Finite floor for log 0: twice the log of the smallest normal number of the
 * component format (Section 3.1, footnote on the configurable real log). */
static float floor_f32(void) { return (float)(2.0Q * logq((__float128)FLT_MIN)); }
static double floor_f64(void) { return (double)(2.0Q * logq((__float128)DBL_MIN)); }

ORACLE_API float oracle_floor_f32(void) { return floor_f32(); }
ORACLE_API double oracle_floor_f64(void) { return floor_f64(); }

/* x -> (log|x|, 0 or pi), interleaved (re, im).  zero_floor = 0: log 0 = -inf;
 * zero_floor = 1: log 0 = the finite floor.  -0.0 counts as non-negative. */
ORACLE_API void oracle_to_goom_f32(const float *x, float *y, size_t n, int zero_floor)
{
    const float pi_f = (float)M_PIq;
    const float fl = floor_f32();
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) {
        float v = x[i];
        float re;
        if (v == 0.0f)
            re = zero_floor ? fl : -INFINITY;
        else
            re = (float)logq(fabsq((__float128)v)); /* NaN -> NaN, +-inf -> +inf */
        y[2 * i] = re;
        y[2 * i + 1] = (v < 0.0f) ? pi_f : 0.0f;
    }
}

ORACLE_API void oracle_to_goom_f64(const double *x, double *y, size_t n, int zero_floor)
{
    const double pi_d = (double)M_PIq;
    const double fl = floor_f64();
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) {
        double v = x[i];
        double re;
        if (v == 0.0)
            re = zero_floor ? fl : -INFINITY;
        else
            re = (double)logq(fabsq((__float128)v));
        y[2 * i] = re;
        y[2 * i + 1] = (v < 0.0) ? pi_d : 0.0;
    }
}

/* (re, im) -> Re(exp(re + i im)) = +-exp(re); the imaginary part of the complex
 * exponential is dropped (Section 3.1, eq. 7). */
ORACLE_API void oracle_from_goom_f32(const float *y, float *x, size_t n)
{
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) {
        __float128 e = expq((__float128)y[2 * i]);
        float mag = (float)e;
        x[i] = sign_from_imag((double)y[2 * i + 1]) ? -mag : mag;
    }
}

ORACLE_API void oracle_from_goom_f64(const double *y, double *x, size_t n)
{
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) {
        __float128 e = expq((__float128)y[2 * i]);
        double mag = (double)e;
        x[i] = sign_from_imag(y[2 * i + 1]) ? -mag : mag;
    }
}

/* Widen interleaved complex GOOMs to the oracle's working form: double
 * log-magnitude plus a sign byte. */
ORACLE_API void oracle_split_c64(const float *z, double *re, uint8_t *sg, size_t n)
{
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) {
        re[i] = (double)z[2 * i];
        sg[i] = sign_from_imag((double)z[2 * i + 1]);
    }
}

ORACLE_API void oracle_split_c128(const double *z, double *re, uint8_t *sg, size_t n)
{
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) {
        re[i] = z[2 * i];
        sg[i] = sign_from_imag(z[2 * i + 1]);
    }
}

/* ------------------------------------------------------------------------- */
/* signed log-sum-exp (Example 2) and LMME (Section 3.2, eq. 9)               */
/* ------------------------------------------------------------------------- */

/* log of sum_j (+-)exp(z_j).  Returns the log-magnitude, the sign, and
 * kappa = sum_j exp(z_j) / |sum_j (+-)exp(z_j)|, the cancellation factor of the sum
 * (1 = no cancellation).  An empty or all -inf sum is zero: (-inf, +). */
static void signed_lse(int d, const double *z, const uint8_t *s, double *out_re,
                       uint8_t *out_sg, double *out_kappa)
{
    double m = -INFINITY;
    for (int j = 0; j < d; ++j)
        if (z[j] > m) m = z[j];
    if (!(m > -INFINITY)) {
        *out_re = -INFINITY;
        *out_sg = 0;
        if (out_kappa) *out_kappa = 1.0;
        return;
    }
    long double acc = 0.0L, mass = 0.0L;
    for (int j = 0; j < d; ++j) {
        long double e = expl((long double)(z[j] - m));
        mass += e;
        acc += s[j] ? -e : e;
    }
    if (acc == 0.0L) {
        *out_re = -INFINITY;
        *out_sg = 0;
        if (out_kappa) *out_kappa = INFINITY;
        return;
    }
    *out_re = m + (double)logl(fabsl(acc));
    *out_sg = acc < 0.0L;
    if (out_kappa) *out_kappa = (double)(mass / fabsl(acc));
}

/* C' = LMME(A', B'):  C'_ik = LSE_j(A'_ij + B'_jk), A' is n x d, B' is d x m, all
 * row-major.  Adding two GOOMs adds log-magnitudes and xors signs (Example 1).
 * kappa may be NULL. */
ORACLE_API void oracle_lmme(const double *are, const uint8_t *asg, const double *bre,
                            const uint8_t *bsg, double *cre, uint8_t *csg, double *kappa,
                            int n, int d, int m)
{
#pragma omp parallel
    {
        double *z = (double *)malloc(sizeof(double) * (size_t)(d > 0 ? d : 1));
        uint8_t *s = (uint8_t *)malloc((size_t)(d > 0 ? d : 1));
#pragma omp for collapse(2) schedule(static)
        for (int i = 0; i < n; ++i) {
            for (int k = 0; k < m; ++k) {
                for (int j = 0; j < d; ++j) {
                    z[j] = are[(size_t)i * d + j] + bre[(size_t)j * m + k];
                    /* (-inf) + (+inf) would be NaN; a zero factor makes the term zero */
                    if (are[(size_t)i * d + j] == -INFINITY || bre[(size_t)j * m + k] == -INFINITY)
                        z[j] = -INFINITY;
                    s[j] = asg[(size_t)i * d + j] ^ bsg[(size_t)j * m + k];
                }
                signed_lse(d, z, s, &cre[(size_t)i * m + k], &csg[(size_t)i * m + k],
                           kappa ? &kappa[(size_t)i * m + k] : NULL);
            }
        }
        free(z);
        free(s);
    }
}

/* batch of independent LMMEs, leading index first (Section 3: functions broadcast
 * over preceding indices). */
ORACLE_API void oracle_lmme_batched(const double *are, const uint8_t *asg, const double *bre,
                                    const uint8_t *bsg, double *cre, uint8_t *csg,
                                    double *kappa, long batch, int n, int d, int m)
{
    for (long b = 0; b < batch; ++b)
        oracle_lmme(are + (size_t)b * n * d, asg + (size_t)b * n * d, bre + (size_t)b * d * m,
                    bsg + (size_t)b * d * m, cre + (size_t)b * n * m, csg + (size_t)b * n * m,
                    kappa ? kappa + (size_t)b * n * m : NULL, n, d, m);
}

/* ------------------------------------------------------------------------- */
/* chain of matrix products (Section 4.1, eqs. 14-15)                         */
/* ------------------------------------------------------------------------- */

/* Inclusive prefix products, newer factor on the left:
 *   P_1 = M_1 (or LMME(M_1, init) when init is given, init being d x m),
 *   P_t = LMME(M_t, P_{t-1}),  t = 2..T.
 * M is [T, d, d]; P is [T, d, m] (m = d when init is NULL); kappa (nullable, same
 * shape as P) receives the cancellation factor of the last sum that produced each
 * entry (1 for entries copied from M_1). */
ORACLE_API void oracle_scan(const double *mre, const uint8_t *msg, const double *ire,
                            const uint8_t *isg, double *pre, uint8_t *psg, double *kappa,
                            long T, int d, int m)
{
    size_t dd = (size_t)d * d, dm = (size_t)d * m;
    for (long t = 0; t < T; ++t) {
        const double *pr_prev;
        const uint8_t *ps_prev;
        if (t == 0) {
            if (!ire) {
                memcpy(pre, mre, sizeof(double) * dd);
                memcpy(psg, msg, dd);
                if (kappa)
                    for (size_t e = 0; e < dd; ++e) kappa[e] = 1.0;
                continue;
            }
            pr_prev = ire;
            ps_prev = isg;
        } else {
            pr_prev = pre + (size_t)(t - 1) * dm;
            ps_prev = psg + (size_t)(t - 1) * dm;
        }
        oracle_lmme(mre + (size_t)t * dd, msg + (size_t)t * dd, pr_prev, ps_prev,
                    pre + (size_t)t * dm, psg + (size_t)t * dm,
                    kappa ? kappa + (size_t)t * dm : NULL, d, d, m);
    }
}

/* Same chain, but only the running state is kept; the caller passes the state in
 * (state_valid != 0) or starts a fresh chain (state_valid == 0: the state becomes
 * M_1).  After the call the state is P_T.  Steps listed in sample_t (0-based,
 * ascending, nsample entries) are copied to out (nsample x d x m).  Lets a long chain
 * be walked block by block without holding every prefix. */
ORACLE_API void oracle_scan_stream(const double *mre, const uint8_t *msg, double *state_re,
                                   uint8_t *state_sg, int state_valid, const long *sample_t,
                                   long nsample, double *out_re, uint8_t *out_sg,
                                   double *out_kappa, long T, int d, int m)
{
    size_t dd = (size_t)d * d, dm = (size_t)d * m;
    double *nre = (double *)malloc(sizeof(double) * dm);
    uint8_t *nsg = (uint8_t *)malloc(dm);
    double *nk = (double *)malloc(sizeof(double) * dm);
    long si = 0;
    for (long t = 0; t < T; ++t) {
        if (t == 0 && !state_valid) {
            memcpy(nre, mre, sizeof(double) * dd);
            memcpy(nsg, msg, dd);
            for (size_t e = 0; e < dd; ++e) nk[e] = 1.0;
        } else {
            oracle_lmme(mre + (size_t)t * dd, msg + (size_t)t * dd, state_re, state_sg, nre,
                        nsg, nk, d, d, m);
        }
        memcpy(state_re, nre, sizeof(double) * dm);
        memcpy(state_sg, nsg, dm);
        while (si < nsample && sample_t[si] == t) {
            memcpy(out_re + (size_t)si * dm, nre, sizeof(double) * dm);
            memcpy(out_sg + (size_t)si * dm, nsg, dm);
            if (out_kappa) memcpy(out_kappa + (size_t)si * dm, nk, sizeof(double) * dm);
            ++si;
        }
    }
    free(nre);
    free(nsg);
    free(nk);
}

/* ------------------------------------------------------------------------- */
/* second chain oracle: scaled real products in double                        */
/* ------------------------------------------------------------------------- */

/* The same chain computed another way, for chains too long for d^3 exponentials per
 * step: the state is a real double matrix W with one power-of-two exponent per
 * column, P_t[:, k] = W[:, k] * 2^e_k.  Each step exponentiates the incoming factor
 * (entries of M_t must themselves be in double range, which holds for GOOMs of
 * ordinary floats), multiplies, and renormalises every column by an exact power of
 * two.  It is trusted only after tests show it agrees with oracle_scan; it also
 * reports kappa like oracle_scan.  State arrays: w [d*m] doubles, e [m] doubles
 * (integer valued).  state_valid == 0 starts from P_1 = M_1 (needs m == d). */
ORACLE_API void oracle_scan_scaled_stream(const double *mre, const uint8_t *msg, double *w,
                                          double *e, int state_valid, const long *sample_t,
                                          long nsample, double *out_re, uint8_t *out_sg,
                                          double *out_kappa, long T, int d, int m)
{
    size_t dd = (size_t)d * d, dm = (size_t)d * m;
    double *a = (double *)malloc(sizeof(double) * dd);
    double *nw = (double *)malloc(sizeof(double) * dm);
    double *nk = (double *)malloc(sizeof(double) * dm);
    long si = 0;
    for (long t = 0; t < T; ++t) {
        const double *re = mre + (size_t)t * dd;
        const uint8_t *sg = msg + (size_t)t * dd;
        for (size_t q = 0; q < dd; ++q) {
            double v = exp(re[q]);
            a[q] = sg[q] ? -v : v;
        }
        if (t == 0 && !state_valid) {
            memcpy(nw, a, sizeof(double) * dd);
            for (size_t q = 0; q < dm; ++q) nk[q] = 1.0;
            for (int k = 0; k < m; ++k) e[k] = 0.0;
        } else {
#pragma omp parallel for collapse(2) schedule(static)
            for (int i = 0; i < d; ++i) {
                for (int k = 0; k < m; ++k) {
                    long double acc = 0.0L, mass = 0.0L;
                    for (int j = 0; j < d; ++j) {
                        long double p = (long double)a[(size_t)i * d + j] * w[(size_t)j * m + k];
                        acc += p;
                        mass += fabsl(p);
                    }
                    nw[(size_t)i * m + k] = (double)acc;
                    nk[(size_t)i * m + k] = acc != 0.0L ? (double)(mass / fabsl(acc)) : INFINITY;
                }
            }
        }
        /* exact power-of-two renormalisation of every column */
        for (int k = 0; k < m; ++k) {
            double cmax = 0.0;
            for (int i = 0; i < d; ++i) {
                double v = fabs(nw[(size_t)i * m + k]);
                if (v > cmax) cmax = v;
            }
            if (cmax > 0.0 && isfinite(cmax)) {
                int ex;
                frexp(cmax, &ex);
                for (int i = 0; i < d; ++i) nw[(size_t)i * m + k] = ldexp(nw[(size_t)i * m + k], -ex);
                e[k] += (double)ex;
            }
        }
        memcpy(w, nw, sizeof(double) * dm);
        while (si < nsample && sample_t[si] == t) {
            for (int i = 0; i < d; ++i)
                for (int k = 0; k < m; ++k) {
                    double v = w[(size_t)i * m + k];
                    size_t o = (size_t)si * dm + (size_t)i * m + k;
                    out_re[o] = (v == 0.0) ? -INFINITY : log(fabs(v)) + e[k] * M_LN2;
                    out_sg[o] = v < 0.0;
                    if (out_kappa) out_kappa[o] = nk[(size_t)i * m + k];
                }
            ++si;
        }
    }
    free(a);
    free(nw);
    free(nk);
}

/* ------------------------------------------------------------------------- */
/* linear recurrence with bias over GOOMs (Section 4.3, eqs. 25 and 26)       */
/* ------------------------------------------------------------------------- */

/* h_t = A_t h_{t-1} + b_t, t = 1..T, h_0 given (NULL = zero vector).
 * In GOOM form each entry of h_t is the signed log-sum-exp of the d products
 * A'_t[i, j] + h'_{t-1}[j] together with b'_t[i]; that is eq. 26 with the inner LMMEs
 * written out.  A is [T, d, d], b is [T, d], h is [T, d]. */
ORACLE_API void oracle_affine_scan(const double *are, const uint8_t *asg, const double *bre,
                                   const uint8_t *bsg, const double *h0re, const uint8_t *h0sg,
                                   double *hre, uint8_t *hsg, double *kappa, long T, int d)
{
    double *pre = (double *)malloc(sizeof(double) * (size_t)d);
    uint8_t *psg = (uint8_t *)malloc((size_t)d);
    double *z = (double *)malloc(sizeof(double) * (size_t)(d + 1));
    uint8_t *s = (uint8_t *)malloc((size_t)(d + 1));
    for (int j = 0; j < d; ++j) {
        pre[j] = h0re ? h0re[j] : -INFINITY;
        psg[j] = h0sg ? h0sg[j] : 0;
    }
    for (long t = 0; t < T; ++t) {
        const double *ar = are + (size_t)t * d * d;
        const uint8_t *as = asg + (size_t)t * d * d;
        for (int i = 0; i < d; ++i) {
            for (int j = 0; j < d; ++j) {
                z[j] = ar[(size_t)i * d + j] + pre[j];
                if (ar[(size_t)i * d + j] == -INFINITY || pre[j] == -INFINITY) z[j] = -INFINITY;
                s[j] = as[(size_t)i * d + j] ^ psg[j];
            }
            z[d] = bre[(size_t)t * d + i];
            s[d] = bsg[(size_t)t * d + i];
            signed_lse(d + 1, z, s, &hre[(size_t)t * d + i], &hsg[(size_t)t * d + i],
                       kappa ? &kappa[(size_t)t * d + i] : NULL);
        }
        memcpy(pre, hre + (size_t)t * d, sizeof(double) * (size_t)d);
        memcpy(psg, hsg + (size_t)t * d, (size_t)d);
    }
    free(pre);
    free(psg);
    free(z);
    free(s);
}

/* Independent sequences, leading index first: A [batch, T, d, d], b [batch, T, d],
 * h0 [batch, d] (nullable), h [batch, T, d].  Threads split the sequences; each
 * sequence is still walked left to right. */
ORACLE_API void oracle_affine_scan_batched(const double *are, const uint8_t *asg,
                                           const double *bre, const uint8_t *bsg,
                                           const double *h0re, const uint8_t *h0sg, double *hre,
                                           uint8_t *hsg, double *kappa, long batch, long T, int d)
{
#pragma omp parallel for schedule(dynamic)
    for (long q = 0; q < batch; ++q) {
        size_t oa = (size_t)q * T * d * d, ob = (size_t)q * T * d;
        oracle_affine_scan(are + oa, asg + oa, bre + ob, bsg + ob,
                           h0re ? h0re + (size_t)q * d : NULL, h0sg ? h0sg + (size_t)q * d : NULL,
                           hre + ob, hsg + ob, kappa ? kappa + ob : NULL, T, d);
    }
}

/* ------------------------------------------------------------------------- */
/* QR (Householder, R_ii > 0) on small real matrices                          */
/* ------------------------------------------------------------------------- */

/* a: d x d row-major, overwritten by Q (orthonormal columns); r receives the upper
 * triangular factor with positive diagonal.  Householder reflections, then Q is
 * accumulated explicitly; signs are flipped at the end so that diag(R) > 0. */
static void qr_householder(double *a, double *r, int d)
{
    double *q = (double *)calloc((size_t)d * d, sizeof(double));
    double *v = (double *)malloc(sizeof(double) * (size_t)d);
    for (int i = 0; i < d; ++i) q[(size_t)i * d + i] = 1.0;
    /* reduce a to upper triangular in place: a <- H_k ... H_1 a ; q <- q H_1 ... H_k */
    for (int k = 0; k < d; ++k) {
        long double nrm = 0.0L;
        for (int i = k; i < d; ++i) nrm += (long double)a[(size_t)i * d + k] * a[(size_t)i * d + k];
        double alpha = (double)sqrtl(nrm);
        if (alpha == 0.0) continue;
        if (a[(size_t)k * d + k] > 0.0) alpha = -alpha;
        for (int i = 0; i < d; ++i) v[i] = 0.0;
        for (int i = k; i < d; ++i) v[i] = a[(size_t)i * d + k];
        v[k] -= alpha;
        long double vn = 0.0L;
        for (int i = k; i < d; ++i) vn += (long double)v[i] * v[i];
        if (vn == 0.0L) continue;
        for (int j = 0; j < d; ++j) { /* a <- (I - 2 v v^T / v^T v) a */
            long double dot = 0.0L;
            for (int i = k; i < d; ++i) dot += (long double)v[i] * a[(size_t)i * d + j];
            double f = (double)(2.0L * dot / vn);
            for (int i = k; i < d; ++i) a[(size_t)i * d + j] -= f * v[i];
        }
        for (int i = 0; i < d; ++i) { /* q <- q (I - 2 v v^T / v^T v) */
            long double dot = 0.0L;
            for (int j = k; j < d; ++j) dot += (long double)q[(size_t)i * d + j] * v[j];
            double f = (double)(2.0L * dot / vn);
            for (int j = k; j < d; ++j) q[(size_t)i * d + j] -= f * v[j];
        }
    }
    for (int i = 0; i < d; ++i)
        for (int j = 0; j < d; ++j) r[(size_t)i * d + j] = (j >= i) ? a[(size_t)i * d + j] : 0.0;
    for (int k = 0; k < d; ++k) {
        if (r[(size_t)k * d + k] < 0.0) {
            for (int j = 0; j < d; ++j) r[(size_t)k * d + j] = -r[(size_t)k * d + j];
            for (int i = 0; i < d; ++i) q[(size_t)i * d + k] = -q[(size_t)i * d + k];
        }
    }
    memcpy(a, q, sizeof(double) * (size_t)d * d);
    free(q);
    free(v);
}

ORACLE_API void oracle_qr(const double *a, double *q, double *r, int d)
{
    memcpy(q, a, sizeof(double) * (size_t)d * d);
    qr_householder(q, r, d);
}

/* ------------------------------------------------------------------------- */
/* Lyapunov spectrum, sequential QR (Section 4.2.1, eqs. 19-20)               */
/* ------------------------------------------------------------------------- */

/* J: [T, d, d] real Jacobians (double).  Q_0 = I.  S_t = J_t Q_{t-1};
 * Q_t, R_t = QR(S_t); lambda = sum_t log|diag R_t| / (dt T). */
ORACLE_API void oracle_lyapunov_qr(const double *J, long T, int d, double dt, double *lambda)
{
    size_t dd = (size_t)d * d;
    double *q = (double *)calloc(dd, sizeof(double));
    double *s = (double *)malloc(sizeof(double) * dd);
    double *r = (double *)malloc(sizeof(double) * dd);
    long double *acc = (long double *)calloc((size_t)d, sizeof(long double));
    for (int i = 0; i < d; ++i) q[(size_t)i * d + i] = 1.0;
    for (long t = 0; t < T; ++t) {
        const double *jt = J + (size_t)t * dd;
        for (int i = 0; i < d; ++i)
            for (int k = 0; k < d; ++k) {
                long double a = 0.0L;
                for (int j = 0; j < d; ++j) a += (long double)jt[(size_t)i * d + j] * q[(size_t)j * d + k];
                s[(size_t)i * d + k] = (double)a;
            }
        qr_householder(s, r, d);
        memcpy(q, s, sizeof(double) * dd);
        for (int k = 0; k < d; ++k) acc[k] += logl(fabsl((long double)r[(size_t)k * d + k]));
    }
    for (int k = 0; k < d; ++k) lambda[k] = (double)(acc[k] / ((long double)dt * (long double)T));
    free(q);
    free(s);
    free(r);
    free(acc);
}

/* ------------------------------------------------------------------------- */
/* selectively reset recurrence (Section 5; Section 4.2.1 item (a))           */
/* ------------------------------------------------------------------------- */

/* Log-normalise the columns of a GOOM matrix to unit norm, exponentiate, and
 * return the real matrix plus each column's log-norm (Section 4.2.1 (a): states are
 * log-scaled to log-unit norms over GOOMs before QR).  A zero column keeps
 * log-norm -inf and exponentiates to zeros. */
static void normalise_columns(const double *xre, const uint8_t *xsg, double *n, double *lognorm,
                              int d)
{
    for (int k = 0; k < d; ++k) {
        double m = -INFINITY;
        for (int i = 0; i < d; ++i)
            if (xre[(size_t)i * d + k] > m) m = xre[(size_t)i * d + k];
        if (!(m > -INFINITY)) {
            lognorm[k] = -INFINITY;
            for (int i = 0; i < d; ++i) n[(size_t)i * d + k] = 0.0;
            continue;
        }
        long double ss = 0.0L;
        for (int i = 0; i < d; ++i) ss += expl(2.0L * (long double)(xre[(size_t)i * d + k] - m));
        lognorm[k] = m + 0.5 * (double)logl(ss);
        for (int i = 0; i < d; ++i) {
            double v = exp(xre[(size_t)i * d + k] - lognorm[k]);
            n[(size_t)i * d + k] = xsg[(size_t)i * d + k] ? -v : v;
        }
    }
}

/* Selection function of Section 4.2.1 (a): 1 when the absolute cosine similarity of
 * any pair of (unit) columns exceeds the threshold. */
static int near_colinear(const double *n, int d, double threshold)
{
    for (int a = 0; a < d; ++a)
        for (int b = a + 1; b < d; ++b) {
            long double dot = 0.0L;
            for (int i = 0; i < d; ++i) dot += (long double)n[(size_t)i * d + a] * n[(size_t)i * d + b];
            if (fabsl(dot) > threshold) return 1;
        }
    return 0;
}

/* X_t = J_t X_{t-1}, t = 1..T, over GOOMs, with the state examined at every step t
 * that is a multiple of check_every: when policy == 1 (always) or, for policy == 0,
 * when the columns are near-colinear, the state is replaced by the orthonormal
 * factor Q of its column-normalised real form (Section 5: X_t <- R(X_t); Section
 * 4.2.1 (a) for this particular S and R).  With R_ii > 0, the log-growth removed by a
 * reset from column k is log R_kk + lognorm_k; those accumulate in growth[k].  At
 * the end the same factorisation is applied once to the final state (without
 * replacing it) so that growth / (dt T) estimates the spectrum.  policy == -1: never
 * reset (plain chain).
 *   J' : [T, d, d] GOOMs;  X0 : [d, d] GOOM (NULL = identity)
 *   states : [T, d, d] (after any reset at that step);  reset_flag : [T] bytes
 *   growth : [d] */
ORACLE_API void oracle_reset_scan(const double *jre, const uint8_t *jsg, const double *x0re,
                                  const uint8_t *x0sg, double *sre, uint8_t *ssg,
                                  uint8_t *reset_flag, double *growth, long T, int d,
                                  long check_every, int policy, double cos_threshold)
{
    size_t dd = (size_t)d * d;
    double *cre = (double *)malloc(sizeof(double) * dd);
    uint8_t *csg = (uint8_t *)malloc(dd);
    double *n = (double *)malloc(sizeof(double) * dd);
    double *r = (double *)malloc(sizeof(double) * dd);
    double *ln = (double *)malloc(sizeof(double) * (size_t)d);
    long double *acc = (long double *)calloc((size_t)d, sizeof(long double));
    for (int i = 0; i < d; ++i)
        for (int k = 0; k < d; ++k) {
            cre[(size_t)i * d + k] = x0re ? x0re[(size_t)i * d + k] : (i == k ? 0.0 : -INFINITY);
            csg[(size_t)i * d + k] = x0sg ? x0sg[(size_t)i * d + k] : 0;
        }
    for (long t = 0; t < T; ++t) {
        double *ore = sre + (size_t)t * dd;
        uint8_t *osg = ssg + (size_t)t * dd;
        oracle_lmme(jre + (size_t)t * dd, jsg + (size_t)t * dd, cre, csg, ore, osg, NULL, d, d, d);
        int did = 0;
        if (policy >= 0 && check_every > 0 && ((t + 1) % check_every) == 0) {
            normalise_columns(ore, osg, n, ln, d);
            if (policy == 1 || near_colinear(n, d, cos_threshold)) {
                qr_householder(n, r, d); /* n <- Q */
                for (int k = 0; k < d; ++k) acc[k] += logl(fabsl((long double)r[(size_t)k * d + k])) + ln[k];
                for (size_t q = 0; q < dd; ++q) {
                    ore[q] = n[q] == 0.0 ? -INFINITY : log(fabs(n[q]));
                    osg[q] = n[q] < 0.0;
                }
                did = 1;
            }
        }
        if (reset_flag) reset_flag[t] = (uint8_t)did;
        memcpy(cre, ore, sizeof(double) * dd);
        memcpy(csg, osg, dd);
    }
    if (growth) {
        normalise_columns(cre, csg, n, ln, d);
        qr_householder(n, r, d);
        for (int k = 0; k < d; ++k) {
            long double g = acc[k] + logl(fabsl((long double)r[(size_t)k * d + k])) + ln[k];
            growth[k] = (double)g;
        }
    }
    free(cre);
    free(csg);
    free(n);
    free(r);
    free(ln);
    free(acc);
}

/* ------------------------------------------------------------------------- */
/* the literal tuple combine of Section 5, eq. 28, over plain reals           */
/* ------------------------------------------------------------------------- */

/* One application of the selective-resetting transformation to a pair of tuples
 * (A_prev, B_prev), (A_curr, B_curr) of real d x d matrices (double, row-major).
 * select_prev is the value of S(A_prev) decided by the caller; reset_value is
 * R(A_prev) (used only when the reset fires).  prev is updated in place by the
 * reset, curr by the recurrence.  The bias update uses A_curr as it was before
 * this step's update of A_curr, which is what the worked example in Appendix C
 * shows (A_3 B_2 + B_3). */
ORACLE_API void oracle_reset_combine_real(double *a_prev, double *b_prev, double *a_curr,
                                          double *b_curr, int select_prev,
                                          const double *reset_value, int d)
{
    size_t dd = (size_t)d * d;
    int b_is_zero = 1;
    for (size_t q = 0; q < dd; ++q)
        if (b_prev[q] != 0.0) { b_is_zero = 0; break; }
    if (select_prev && b_is_zero) {
        memcpy(b_prev, reset_value, sizeof(double) * dd);
        memset(a_prev, 0, sizeof(double) * dd);
    }
    double *na = (double *)malloc(sizeof(double) * dd);
    double *nb = (double *)malloc(sizeof(double) * dd);
    for (int i = 0; i < d; ++i)
        for (int k = 0; k < d; ++k) {
            long double sa = 0.0L, sb = 0.0L;
            for (int j = 0; j < d; ++j) {
                sa += (long double)a_curr[(size_t)i * d + j] * a_prev[(size_t)j * d + k];
                sb += (long double)a_curr[(size_t)i * d + j] * b_prev[(size_t)j * d + k];
            }
            na[(size_t)i * d + k] = (double)sa;
            nb[(size_t)i * d + k] = (double)(sb + (long double)b_curr[(size_t)i * d + k]);
        }
    memcpy(a_curr, na, sizeof(double) * dd);
    memcpy(b_curr, nb, sizeof(double) * dd);
    free(na);
    free(nb);
}

/* ------------------------------------------------------------------------- */
/* Lyapunov spectrum from given input states (Section 4.2.1, groups (b)-(d))  */
/* ------------------------------------------------------------------------- */

/* For every step t = 1..T: the input state S_{t-1} (a GOOM matrix, working form: log-magnitudes
 * and sign bytes; prev_re/prev_sg hold S_0 .. S_{T-1} back to back) is log-scaled to unit column
 * norms and exponentiated, QR gives its orthonormal basis Q_{t-1} (group (b)); the real Jacobian
 * J_t is applied to it (group (c)); QR of the result gives R_t, and log|diag R_t| is stored in
 * steplog[t-1][:] (group (d)).  lambda[k] = mean_t steplog[t][k] / dt.  steplog may be NULL. */
ORACLE_API void oracle_lyapunov_from_states(const double *prev_re, const uint8_t *prev_sg, const double *J,
                                            double *steplog, double *lambda, long T, int d, double dt)
{
    size_t dd = (size_t)d * d;
    long double *acc = (long double *)calloc((size_t)d, sizeof(long double));
#pragma omp parallel
    {
        double *n = (double *)malloc(sizeof(double) * dd);
        double *r = (double *)malloc(sizeof(double) * dd);
        double *z = (double *)malloc(sizeof(double) * dd);
        double *ln = (double *)malloc(sizeof(double) * (size_t)d);
        long double *mine = (long double *)calloc((size_t)d, sizeof(long double));
#pragma omp for schedule(static)
        for (long t = 0; t < T; ++t) {
            normalise_columns(prev_re + (size_t)t * dd, prev_sg + (size_t)t * dd, n, ln, d);
            qr_householder(n, r, d); /* n <- Q_{t-1} */
            const double *jt = J + (size_t)t * dd;
            for (int i = 0; i < d; ++i)
                for (int k = 0; k < d; ++k) {
                    long double a = 0.0L;
                    for (int j = 0; j < d; ++j) a += (long double)jt[(size_t)i * d + j] * n[(size_t)j * d + k];
                    z[(size_t)i * d + k] = (double)a;
                }
            qr_householder(z, r, d);
            for (int k = 0; k < d; ++k) {
                double v = log(fabs(r[(size_t)k * d + k]));
                if (steplog) steplog[(size_t)t * d + k] = v;
                mine[k] += v;
            }
        }
#pragma omp critical
        for (int k = 0; k < d; ++k) acc[k] += mine[k];
        free(n);
        free(r);
        free(z);
        free(ln);
        free(mine);
    }
    for (int k = 0; k < d; ++k) lambda[k] = (double)(acc[k] / ((long double)dt * (long double)T));
    free(acc);
}

/* ------------------------------------------------------------------------- */
/* largest Lyapunov exponent (Section 4.2.2)                                  */
/* ------------------------------------------------------------------------- */

/* The standard method (eqs. 21-22): s_t = J_t u_{t-1}, u_t = s_t / |s_t|,
 * LLE = sum_t log(|s_t| / |u_{t-1}|) / (dt T).  Real Jacobians, double. */
ORACLE_API double oracle_lle_standard(const double *J, const double *u0, long T, int d, double dt)
{
    double *u = (double *)malloc(sizeof(double) * (size_t)d);
    double *s = (double *)malloc(sizeof(double) * (size_t)d);
    long double acc = 0.0L;
    memcpy(u, u0, sizeof(double) * (size_t)d);
    for (long t = 0; t < T; ++t) {
        const double *jt = J + (size_t)t * d * d;
        long double nu = 0.0L, ns = 0.0L;
        for (int i = 0; i < d; ++i) nu += (long double)u[i] * u[i];
        for (int i = 0; i < d; ++i) {
            long double a = 0.0L;
            for (int j = 0; j < d; ++j) a += (long double)jt[(size_t)i * d + j] * u[j];
            s[i] = (double)a;
            ns += a * a;
        }
        acc += 0.5L * (logl(ns) - logl(nu));
        long double inv = 1.0L / sqrtl(ns);
        for (int i = 0; i < d; ++i) u[i] = (double)(s[i] * inv);
    }
    free(u);
    free(s);
    return (double)(acc / ((long double)dt * (long double)T));
}

/* The un-normalised form over GOOMs (eq. 24): LSE(2 * log-magnitudes of J_T ... J_1 u_0) / (2 dt T),
 * given the final vector of that product in working form (from the scan oracle). */
ORACLE_API double oracle_lle_from_final(const double *fre, long T, int d, double dt)
{
    double m = -INFINITY;
    for (int i = 0; i < d; ++i)
        if (2.0 * fre[i] > m) m = 2.0 * fre[i];
    if (!(m > -INFINITY)) return -INFINITY;
    long double acc = 0.0L;
    for (int i = 0; i < d; ++i) acc += expl((long double)(2.0 * fre[i] - m));
    return (double)(((long double)m + logl(acc)) / (2.0L * (long double)dt * (long double)T));
}

/* ------------------------------------------------------------------------- */
/* scaled exponentiation of recurrence states (Section 4.3, eq. 27)           */
/* ------------------------------------------------------------------------- */

/* For each of n vectors of length d in working form: c = max of the log-magnitudes,
 * scaled_i = (+-) exp(re_i - c + 2), so every scaled entry lies in [-e^2, e^2].  A vector of
 * zeros has c = -inf and scaled = 0. */
ORACLE_API void oracle_scaled_exp(const double *re, const uint8_t *sg, double *scaled, double *c, long n, int d)
{
    for (long v = 0; v < n; ++v) {
        const double *r = re + (size_t)v * d;
        double m = -INFINITY;
        for (int i = 0; i < d; ++i)
            if (r[i] > m) m = r[i];
        c[v] = m;
        for (int i = 0; i < d; ++i) {
            double x = (m > -INFINITY) ? (double)expl((long double)r[i] - (long double)m + 2.0L) : 0.0;
            scaled[(size_t)v * d + i] = sg[(size_t)v * d + i] ? -x : x;
        }
    }
}

/* Backward of the scaled exponentiation: the log-scaling constant c is computed without altering gradients (Section 4.3:
 * detached), so scaled_i = (+-) exp(re_i - c + 2) depends on re_i alone with d scaled_i / d re_i = scaled_i, also for the
 * entry that sets c.  g: gradients with respect to the scaled values; gre: with respect to the log-magnitudes. */
ORACLE_API void oracle_scaled_exp_backward(const double *re, const uint8_t *sg, const double *g, double *gre, long n, int d)
{
    for (long v = 0; v < n; ++v) {
        const double *r = re + (size_t)v * d;
        double m = -INFINITY;
        for (int i = 0; i < d; ++i)
            if (r[i] > m) m = r[i];
        for (int i = 0; i < d; ++i) {
            const long double x = (m > -INFINITY) ? expl((long double)r[i] - (long double)m + 2.0L) : 0.0L;
            gre[(size_t)v * d + i] = (double)((long double)g[(size_t)v * d + i] * (sg[(size_t)v * d + i] ? -x : x));
        }
    }
}

/* ------------------------------------------------------------------------- */
/* signed log-add of two GOOM arrays: log(exp(x') + exp(y')) (Section 2, Example 2; */
/* the bias step of Section 4.3, eq. 26)                                      */
/* ------------------------------------------------------------------------- */

/* Elementwise.  With m the larger and l the smaller log-magnitude, delta = m - l >= 0:
 * same signs: m + log1p(exp(-delta)); opposite signs: m + log(-expm1(-delta)), sign of the
 * larger; equal magnitudes with opposite signs give zero (-inf, +). */
ORACLE_API void oracle_log_add_exp(const double *xre, const uint8_t *xsg, const double *yre, const uint8_t *ysg,
                                   double *ore, uint8_t *osg, long n)
{
#pragma omp parallel for schedule(static)
    for (long i = 0; i < n; ++i) {
        double a = xre[i], b = yre[i];
        uint8_t sa = xsg[i], sb = ysg[i];
        if (b > a || (b == a && sb < sa)) { double t = a; a = b; b = t; uint8_t u = sa; sa = sb; sb = u; }
        if (!(a > -INFINITY)) { ore[i] = -INFINITY; osg[i] = 0; continue; }       /* 0 + 0 */
        if (!(b > -INFINITY)) { ore[i] = a; osg[i] = sa; continue; }               /* x + 0 */
        long double delta = (long double)a - (long double)b;
        if (sa == sb) {
            ore[i] = (double)((long double)a + log1pl(expl(-delta)));
            osg[i] = sa;
        } else if (delta == 0.0L) {
            ore[i] = -INFINITY;
            osg[i] = 0;
        } else {
            ore[i] = (double)((long double)a + logl(-expm1l(-delta)));
            osg[i] = sa;
        }
    }
}

/* ------------------------------------------------------------------------- */
/* backward passes (Section 3.1: the redefined finite derivatives of the real  */
/* absolute value, the real logarithm and the complex exponential; Section 3.2:*/
/* log-scaling constants take no part in gradients; Section 4.3: the recurrence)*/
/* ------------------------------------------------------------------------- */

/* float -> GOOM, backward: the log-magnitude is log(abs(x)) with d abs(x) / dx := +1 for x >= 0 and -1 for
 * x < 0 (never zero), and d log(u) / du := 1 / (u + eps) (always finite); so an upstream gradient g with
 * respect to the log-magnitude gives gx = g * s(x) / (|x| + eps).  The phase is piecewise constant. */
ORACLE_API void oracle_to_goom_backward(const double *x, const double *g, double *gx, double eps, long n)
{
    for (long i = 0; i < n; ++i) {
        const long double s = x[i] < 0.0 ? -1.0L : 1.0L;
        gx[i] = (double)((long double)g[i] * s / (fabsl((long double)x[i]) + (long double)eps));
    }
}

/* GOOM -> float, backward: x = Re(exp(x')) and d exp(x') / d x' := exp(x') + eps for x >= 0, exp(x') - eps
 * for x < 0 (never zero); so an upstream gradient gx with respect to x gives, for the log-magnitude,
 * g = gx * (x + s(x) eps).  Inputs in working form (log-magnitude, sign). */
ORACLE_API void oracle_from_goom_backward(const double *re, const uint8_t *sg, const double *gx, double *g, double eps, long n)
{
    for (long i = 0; i < n; ++i) {
        const long double mag = expl((long double)re[i]);
        const long double v = sg[i] ? -mag : mag;
        g[i] = (double)((long double)gx[i] * (v + (v < 0.0L ? -(long double)eps : (long double)eps)));
    }
}

/* Backward pass of h_t = A_t h_{t-1} + b_t over GOOMs, in the limit eps -> 0 of the redefined derivatives (they
 * differ from the ordinary ones only where a value is within eps of zero; a state entry that is exactly zero
 * passes no gradient here).  Given the upstream gradients G_t[i] = dL / d Re h'_t[i], the adjoint of the value
 * h_t[i] receives G_t[i] / h_t[i] directly, and adjoints run backwards through the transposed matrices:
 *     lam_t = G_t / h_t + A_{t+1}^T lam_{t+1},        lam_{T-1} = G_{T-1} / h_{T-1},
 * a recurrence of the same kind in reverse time, walked here over GOOMs (the adjoints shrink as fast as the
 * states grow).  The gradients with respect to log-magnitudes follow with d v / d log|v| = v:
 *     dL / d Re A'_t[i, j] = lam_t[i] A_t[i, j] h_{t-1}[j],     dL / d Re b'_t[i] = lam_t[i] b_t[i],
 *     dL / d Re h'_{-1}[j] = h_{-1}[j] sum_i lam_0[i] A_0[i, j]                       (the initial state).
 * A [T, d, d], b [T, d], h0 [d] or NULL (zero), h [T, d] the forward states, G [T, d] reals.  Outputs: gA
 * [T, d, d], gb [T, d], gh0 [d] or NULL, and the adjoints themselves as GOOMs lam [T, d]. */
ORACLE_API void oracle_affine_backward(const double *are, const uint8_t *asg, const double *bre, const uint8_t *bsg,
                                       const double *h0re, const uint8_t *h0sg, const double *hre, const uint8_t *hsg,
                                       const double *G, double *gA, double *gb, double *gh0, double *lre, uint8_t *lsg,
                                       long T, int d)
{
    double *z = (double *)malloc(sizeof(double) * (size_t)(d + 1));
    uint8_t *s = (uint8_t *)malloc((size_t)(d + 1));
    for (long t = T - 1; t >= 0; --t) {
        for (int i = 0; i < d; ++i) {
            int n = 0;
            const double g = G[(size_t)t * d + i], hr = hre[(size_t)t * d + i];
            if (g != 0.0 && hr > -INFINITY) {
                z[n] = log(fabs(g)) - hr;
                s[n] = (uint8_t)((g < 0.0) ^ hsg[(size_t)t * d + i]);
                ++n;
            }
            if (t + 1 < T) {
                const double *ar = are + (size_t)(t + 1) * d * d;
                const uint8_t *as = asg + (size_t)(t + 1) * d * d;
                for (int j = 0; j < d; ++j) { /* (A_{t+1}^T lam_{t+1})[i] = sum_j A_{t+1}[j, i] lam_{t+1}[j] */
                    const double a = ar[(size_t)j * d + i], l = lre[(size_t)(t + 1) * d + j];
                    if (a == -INFINITY || l == -INFINITY) continue;
                    z[n] = a + l;
                    s[n] = as[(size_t)j * d + i] ^ lsg[(size_t)(t + 1) * d + j];
                    ++n;
                }
            }
            signed_lse(n, z, s, &lre[(size_t)t * d + i], &lsg[(size_t)t * d + i], NULL);
        }
    }
    for (long t = 0; t < T; ++t) {
        for (int i = 0; i < d; ++i) {
            const double l = lre[(size_t)t * d + i];
            const uint8_t ls = lsg[(size_t)t * d + i];
            const double br = bre[(size_t)t * d + i];
            double v = (l > -INFINITY && br > -INFINITY) ? (double)expl((long double)l + (long double)br) : 0.0;
            gb[(size_t)t * d + i] = (ls ^ bsg[(size_t)t * d + i]) ? -v : v;
            for (int j = 0; j < d; ++j) {
                const double a = are[((size_t)t * d + i) * d + j];
                const double pr = t > 0 ? hre[(size_t)(t - 1) * d + j] : (h0re ? h0re[j] : -INFINITY);
                const uint8_t ps = t > 0 ? hsg[(size_t)(t - 1) * d + j] : (h0sg ? h0sg[j] : 0);
                v = (l > -INFINITY && a > -INFINITY && pr > -INFINITY) ? (double)expl((long double)l + (long double)a + (long double)pr) : 0.0;
                gA[((size_t)t * d + i) * d + j] = (ls ^ asg[((size_t)t * d + i) * d + j] ^ ps) ? -v : v;
            }
        }
    }
    if (gh0) {
        for (int j = 0; j < d; ++j) {
            long double acc = 0.0L;
            for (int i = 0; i < d; ++i) acc += (long double)gA[(size_t)i * d + j]; /* lam_0[i] A_0[i, j] h_{-1}[j], summed over i */
            gh0[j] = h0re ? (double)acc : 0.0;
        }
    }
    free(z);
    free(s);
}

/* Backward pass of C' = LMME(A', B') over GOOMs (Section 3.2 with the derivatives of Section 3.1 in the limit
 * eps -> 0, as for the recurrence above).  With C = A B over reals and upstream gradients G_ik = dL / d Re C'_ik,
 * d log|C_ik| / d A_ij = B_jk / C_ik and d A_ij / d log|A_ij| = A_ij, so
 *     dL / d Re A'_ij = sum_k G_ik A_ij B_jk / C_ik,      dL / d Re B'_jk = sum_i G_ik A_ij B_jk / C_ik,
 * each term evaluated as (+-) exp(A'_ij + B'_jk - C'_ik + log|G_ik|) and the sums taken relative to their largest
 * term in long double.  An output C_ik that is exactly zero passes no gradient.  A [n, d], B [d, m], C = LMME(A, B)
 * [n, m] in working form, G [n, m] reals; gA [n, d], gB [d, m] reals. */
ORACLE_API void oracle_lmme_backward(const double *are, const uint8_t *asg, const double *bre, const uint8_t *bsg,
                                     const double *cre, const uint8_t *csg, const double *g, double *gA, double *gB,
                                     int n, int d, int m)
{
    const int len = n > m ? n : m;
    double *z = (double *)malloc(sizeof(double) * (size_t)(len > 0 ? len : 1));
    uint8_t *s = (uint8_t *)malloc((size_t)(len > 0 ? len : 1));
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < d; ++j) {
            for (int k = 0; k < m; ++k) {
                const double a = are[(size_t)i * d + j], b = bre[(size_t)j * m + k], c = cre[(size_t)i * m + k], gv = g[(size_t)i * m + k];
                const int live = a > -INFINITY && b > -INFINITY && c > -INFINITY && gv != 0.0;
                z[k] = live ? (double)((long double)a + (long double)b - (long double)c + logl(fabsl((long double)gv))) : -INFINITY;
                s[k] = (uint8_t)(asg[(size_t)i * d + j] ^ bsg[(size_t)j * m + k] ^ csg[(size_t)i * m + k] ^ (gv < 0.0));
            }
            double re;
            uint8_t sg;
            signed_lse(m, z, s, &re, &sg, NULL);
            const double v = re > -INFINITY ? (double)expl((long double)re) : 0.0;
            gA[(size_t)i * d + j] = sg ? -v : v;
        }
    for (int j = 0; j < d; ++j)
        for (int k = 0; k < m; ++k) {
            for (int i = 0; i < n; ++i) {
                const double a = are[(size_t)i * d + j], b = bre[(size_t)j * m + k], c = cre[(size_t)i * m + k], gv = g[(size_t)i * m + k];
                const int live = a > -INFINITY && b > -INFINITY && c > -INFINITY && gv != 0.0;
                z[i] = live ? (double)((long double)a + (long double)b - (long double)c + logl(fabsl((long double)gv))) : -INFINITY;
                s[i] = (uint8_t)(asg[(size_t)i * d + j] ^ bsg[(size_t)j * m + k] ^ csg[(size_t)i * m + k] ^ (gv < 0.0));
            }
            double re;
            uint8_t sg;
            signed_lse(n, z, s, &re, &sg, NULL);
            const double v = re > -INFINITY ? (double)expl((long double)re) : 0.0;
            gB[(size_t)j * m + k] = sg ? -v : v;
        }
    free(z);
    free(s);
}

/* Backward pass of the prefix scan P_t = M_t P_{t-1} over GOOMs (Section 4.1; derivatives of Section 3.1 in the
 * limit eps -> 0, as above).  P_{-1} is the initial state S0 (d x m) or, without one, the identity (m = d, so that
 * P_0 = M_0).  Given G_t[i, k] = dL / d Re P'_t[i, k], the adjoints of the values are d x m matrices that run
 * backwards through the transposed factors,
 *     Lam_t = G_t / P_t (entry by entry) + M_{t+1}^T Lam_{t+1},        Lam_{T-1} = G_{T-1} / P_{T-1},
 * and with d v / d log|v| = v
 *     dL / d Re M'_t[i, j] = M_t[i, j] sum_k Lam_t[i, k] P_{t-1}[j, k],
 *     dL / d Re S0'[j, k] = S0[j, k] sum_i M_0[i, j] Lam_0[i, k].
 * An entry of a state that is exactly zero passes no gradient.  M [T, d, d], S0 [d, m] or NULL, P [T, d, m] the
 * forward states, G [T, d, m] reals.  Outputs: gM [T, d, d], gS0 [d, m] or NULL, the adjoints as GOOMs lam [T, d, m]. */
ORACLE_API void oracle_scan_backward(const double *mre, const uint8_t *msg, const double *s0re, const uint8_t *s0sg,
                                     const double *pre, const uint8_t *psg, const double *G, double *gM, double *gS0,
                                     double *lre, uint8_t *lsg, long T, int d, int m)
{
    const size_t dd = (size_t)d * d, dm = (size_t)d * m;
    const int len = (d > m ? d : m) + 1;
    double *z = (double *)malloc(sizeof(double) * (size_t)len);
    uint8_t *s = (uint8_t *)malloc((size_t)len);
    for (long t = T - 1; t >= 0; --t)
        for (int i = 0; i < d; ++i)
            for (int k = 0; k < m; ++k) {
                int n = 0;
                const size_t e = (size_t)t * dm + (size_t)i * m + k;
                if (G[e] != 0.0 && pre[e] > -INFINITY) {
                    z[n] = log(fabs(G[e])) - pre[e];
                    s[n] = (uint8_t)((G[e] < 0.0) ^ psg[e]);
                    ++n;
                }
                if (t + 1 < T)
                    for (int j = 0; j < d; ++j) { /* (M_{t+1}^T Lam_{t+1})[i, k] = sum_j M_{t+1}[j, i] Lam_{t+1}[j, k] */
                        const double a = mre[(size_t)(t + 1) * dd + (size_t)j * d + i], l = lre[(size_t)(t + 1) * dm + (size_t)j * m + k];
                        if (a == -INFINITY || l == -INFINITY) continue;
                        z[n] = a + l;
                        s[n] = msg[(size_t)(t + 1) * dd + (size_t)j * d + i] ^ lsg[(size_t)(t + 1) * dm + (size_t)j * m + k];
                        ++n;
                    }
                signed_lse(n, z, s, &lre[e], &lsg[e], NULL);
            }
    for (long t = 0; t < T; ++t)
        for (int i = 0; i < d; ++i)
            for (int j = 0; j < d; ++j) {
                const double a = mre[(size_t)t * dd + (size_t)i * d + j];
                int n = 0;
                for (int k = 0; k < m; ++k) {
                    double pr;
                    uint8_t ps;
                    if (t > 0) {
                        pr = pre[(size_t)(t - 1) * dm + (size_t)j * m + k];
                        ps = psg[(size_t)(t - 1) * dm + (size_t)j * m + k];
                    } else if (s0re) {
                        pr = s0re[(size_t)j * m + k];
                        ps = s0sg[(size_t)j * m + k];
                    } else {
                        pr = j == k ? 0.0 : -INFINITY; /* the identity */
                        ps = 0;
                    }
                    const double l = lre[(size_t)t * dm + (size_t)i * m + k];
                    if (pr == -INFINITY || l == -INFINITY || a == -INFINITY) continue;
                    z[n] = (double)((long double)a + (long double)l + (long double)pr);
                    s[n] = (uint8_t)(msg[(size_t)t * dd + (size_t)i * d + j] ^ lsg[(size_t)t * dm + (size_t)i * m + k] ^ ps);
                    ++n;
                }
                double re;
                uint8_t sg;
                signed_lse(n, z, s, &re, &sg, NULL);
                const double v = re > -INFINITY ? (double)expl((long double)re) : 0.0;
                gM[(size_t)t * dd + (size_t)i * d + j] = sg ? -v : v;
            }
    if (gS0)
        for (int j = 0; j < d; ++j)
            for (int k = 0; k < m; ++k) {
                int n = 0;
                const double sr = s0re ? s0re[(size_t)j * m + k] : -INFINITY;
                for (int i = 0; i < d && sr > -INFINITY; ++i) {
                    const double a = mre[(size_t)i * d + j], l = lre[(size_t)i * m + k];
                    if (a == -INFINITY || l == -INFINITY) continue;
                    z[n] = (double)((long double)sr + (long double)a + (long double)l);
                    s[n] = (uint8_t)(s0sg[(size_t)j * m + k] ^ msg[(size_t)i * d + j] ^ lsg[(size_t)i * m + k]);
                    ++n;
                }
                double re;
                uint8_t sg;
                signed_lse(n, z, s, &re, &sg, NULL);
                const double v = re > -INFINITY ? (double)expl((long double)re) : 0.0;
                gS0[(size_t)j * m + k] = sg ? -v : v;
            }
    free(z);
    free(s);
}
