/*
 * TEST INFRASTRUCTURE -- CPU oracle, selection arithmetic of noisy top-k gating.
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call this.
 * It shares no code with the HIP library.
 *
 * What it computes (Section 2.1, noisy top-k gating, the equation defining H(x)):
 *     clean_i = (x . W_g)_i            raw_i = (x . W_noise)_i
 *     H_i     = clean_i (+ bias_i) + eps_i * Softplus(raw_i)
 *
 * The paper fixes no floating-point format or summation order.  Because the top-k choice
 * is an integer decision taken on H, "bit-exact top-k" only has a meaning once the fp32
 * arithmetic of H is pinned.  The reading used on both sides of the parity tests is:
 *
 *   (R1) dot products: one fp32 accumulator per (token, expert) starting at +0.0f,
 *        acc = fma(x[t][j], W[j][i], acc) for j = 0 .. d-1 in ascending order
 *        (single rounding per step, no partial sums, no reassociation).
 *   (R2) Softplus(z) = max(z,0) + log1p(exp(-|z|)), evaluated in binary64 with the fixed
 *        sequence of IEEE operations written out in softplus_f32() below and rounded
 *        once to binary32.  |z| is clipped at 64 (softplus(-64) ~ 1.6e-28), so the result
 *        is always a normal, strictly positive fp32 number.
 *   (R3) H = fma(eps, softplus, clean + bias): the bias add is one fp32 add (absent when
 *        there is no bias), the noise term one fused multiply-add.
 *
 * Build: gcc -O2 -mfma -ffp-contract=off -fopenmp -shared -fPIC  (see oracle/build.py).
 * -ffp-contract=off matters: every fused operation below is spelled fma()/fmaf().
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

/* (R2) binary64 evaluation of softplus, one final rounding to binary32. */
float oracle_softplus_f32(float zf)
{
    const double LOG2E = 1.4426950408889634;   /* 1/ln 2, nearest binary64 */
    const double LN2 = 0.6931471805599453;     /* ln 2, nearest binary64   */
    double z = (double)zf;
    double a = fabs(z);
    if (a > 64.0) a = 64.0;

    /* E = exp(-a): a = q*ln2 + r with q = rint(a*log2e), |r| <= ~0.35 */
    double q = rint(a * LOG2E);
    double r = fma(-q, LN2, a);                /* r >= -0.35, exp(-a) = 2^-q * exp(-r) */
    double m = -r;
    /* exp(m) by its Taylor polynomial of degree 13, Horner form */
    double p = 1.0 / 6227020800.0;             /* 1/13! */
    p = fma(p, m, 1.0 / 479001600.0);          /* 1/12! */
    p = fma(p, m, 1.0 / 39916800.0);
    p = fma(p, m, 1.0 / 3628800.0);
    p = fma(p, m, 1.0 / 362880.0);
    p = fma(p, m, 1.0 / 40320.0);
    p = fma(p, m, 1.0 / 5040.0);
    p = fma(p, m, 1.0 / 720.0);
    p = fma(p, m, 1.0 / 120.0);
    p = fma(p, m, 1.0 / 24.0);
    p = fma(p, m, 1.0 / 6.0);
    p = fma(p, m, 0.5);
    p = fma(p, m, 1.0);
    p = fma(p, m, 1.0);
    double E = ldexp(p, -(int)q);              /* exact scaling, E in (0, 1] */

    /* L = log1p(E) = 2*atanh(s), s = E/(2+E) in (0, 1/3].
       The reciprocal of v = 2+E in (2,3] is built from a linear guess and four Newton
       steps so that no division's rounding is involved. */
    double v = 2.0 + E;
    double y = fma(-1.0 / 6.0, v, 5.0 / 6.0);  /* exact at v=2 and v=3 */
    double e;
    e = fma(-v, y, 1.0); y = fma(y, e, y);
    e = fma(-v, y, 1.0); y = fma(y, e, y);
    e = fma(-v, y, 1.0); y = fma(y, e, y);
    e = fma(-v, y, 1.0); y = fma(y, e, y);
    double s = E * y;
    double s2 = s * s;
    /* atanh(s)/s = sum_{j>=0} s2^j / (2j+1), truncated after j = 13 (s2 <= 1/9) */
    double t = 1.0 / 27.0;
    t = fma(t, s2, 1.0 / 25.0);
    t = fma(t, s2, 1.0 / 23.0);
    t = fma(t, s2, 1.0 / 21.0);
    t = fma(t, s2, 1.0 / 19.0);
    t = fma(t, s2, 1.0 / 17.0);
    t = fma(t, s2, 1.0 / 15.0);
    t = fma(t, s2, 1.0 / 13.0);
    t = fma(t, s2, 1.0 / 11.0);
    t = fma(t, s2, 1.0 / 9.0);
    t = fma(t, s2, 1.0 / 7.0);
    t = fma(t, s2, 1.0 / 5.0);
    t = fma(t, s2, 1.0 / 3.0);
    t = fma(t, s2, 1.0);
    double L = 2.0 * (s * t);

    double zpos = z > 0.0 ? z : 0.0;
    return (float)(zpos + L);
}

void oracle_softplus_array(const float *z, float *out, size_t count)
{
#pragma omp parallel for schedule(static)
    for (ptrdiff_t i = 0; i < (ptrdiff_t)count; ++i) out[i] = oracle_softplus_f32(z[i]);
}

/* (R1) clean[t][i] = sum_j x[rows[t]][j] * W[j][i] with the sequential fp32 fma chain.
 * x is [*, d] row-major; `rows` (may be NULL = identity) selects T rows; W is [d, n]
 * row-major; out is [T, n]. */
void oracle_dot_chain_f32(const float *x, const int32_t *rows, const float *W,
                          int64_t T, int64_t d, int64_t n, float *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        const float *xt = x + (rows ? (int64_t)rows[t] : t) * d;
        float *acc = out + t * n;
        for (int64_t i = 0; i < n; ++i) acc[i] = 0.0f;
        for (int64_t j = 0; j < d; ++j) {
            const float xj = xt[j];
            const float *Wj = W + j * n;
            for (int64_t i = 0; i < n; ++i) acc[i] = fmaf(xj, Wj[i], acc[i]);
        }
    }
}

/* (R3) sp = Softplus(raw); cleanb = clean (+ bias); H = fma(eps, sp, cleanb).  eps == NULL
 * means the noise-free gate H = cleanb.  All arrays [T, n]; bias [n] or NULL. */
void oracle_noisy_logits_f32(const float *clean, const float *raw, const float *bias,
                             const float *eps, int64_t T, int64_t n, float *cleanb, float *sp,
                             float *H)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        for (int64_t i = 0; i < n; ++i) {
            const int64_t o = t * n + i;
            float base = clean[o];
            if (bias) base = base + bias[i];
            const float s = oracle_softplus_f32(raw[o]);
            sp[o] = s;
            cleanb[o] = base;
            H[o] = eps ? fmaf(eps[o], s, base) : base;
        }
    }
}
