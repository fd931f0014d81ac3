/*
 * CPU oracle for the arithmetic reduction R(X) = sum_{i=1..n} x_i of the paper
 * (Section 4, the equation that defines R(X)), for fp16 inputs.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is what the GPU library is checked
 * against; nothing in the product path may call it.  It shares no code, header,
 * table or helper with the HIP sources and includes nothing from them.
 *
 * The ones-matrix MMA encoding (Section 4.1, eqs. MMA1/MMA2; Section 4.3, the
 * chained form C_r = 1 x M_r + C_{r-1}) is a re-association of this same sum,
 * not an approximation of it, so the oracle is the plain definition evaluated
 * serially (the one-accumulator algorithm of Section 4) in binary64 (the
 * precision of the CPU reference in Section 5.4), strengthened with
 * Kahan compensation so that its own rounding error is far below one fp32 ulp
 * of the result.
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math (fast-math would delete the
 * compensation term).  Pins: see tests/test_oracle_*.py (closed forms, brute
 * force, exact integer arithmetic, numpy's half decoder for all 65536 codes).
 */
#include <math.h>
#include <pthread.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>

/* IEEE 754 binary16 -> binary64, from the bit fields: 1 sign, 5 exponent
 * (bias 15), 10 fraction.  Subnormals are honoured (value = frac * 2^-24). */
double oracle_fp16_to_f64(uint16_t h)
{
    const int sign = (h >> 15) & 1;
    const int e = (h >> 10) & 0x1f;
    const int f = h & 0x3ff;
    double v;
    if (e == 0) {
        v = ldexp((double)f, -24);              /* zero or subnormal */
    } else if (e == 31) {
        v = f ? NAN : INFINITY;                 /* NaN payload is not kept */
    } else {
        v = ldexp((double)(1024 + f), e - 25);  /* (1 + f/1024) * 2^(e-15) */
    }
    return sign ? -v : v;
}

/* bfloat16 -> binary64: 1 sign, 8 exponent (bias 127), 7 fraction bits. */
double oracle_bf16_to_f64(uint16_t h)
{
    const int sign = (h >> 15) & 1;
    const int e = (h >> 7) & 0xff;
    const int f = h & 0x7f;
    double v;
    if (e == 0) {
        v = ldexp((double)f, -133);             /* zero or subnormal: f * 2^-7 * 2^-126 */
    } else if (e == 255) {
        v = f ? NAN : INFINITY;
    } else {
        v = ldexp((double)(128 + f), e - 134);  /* (1 + f/128) * 2^(e-127) */
    }
    return sign ? -v : v;
}

/* binary32 -> binary64 from the bit fields: 1 sign, 8 exponent (bias 127), 23 fraction. */
double oracle_f32_bits_to_f64(uint32_t w)
{
    const int sign = (int)(w >> 31);
    const int e = (int)((w >> 23) & 0xff);
    const uint32_t f = w & 0x7fffffu;
    double v;
    if (e == 0) {
        v = ldexp((double)f, -149);
    } else if (e == 255) {
        v = f ? NAN : INFINITY;
    } else {
        v = ldexp((double)(0x800000u + f), e - 150);
    }
    return sign ? -v : v;
}

enum { ORACLE_F16 = 0, ORACLE_BF16 = 1, ORACLE_F32 = 2 };

static double value_at(const void *x, size_t i, int dtype)
{
    switch (dtype) {
    case ORACLE_BF16: return oracle_bf16_to_f64(((const uint16_t *)x)[i]);
    case ORACLE_F32: return oracle_f32_bits_to_f64(((const uint32_t *)x)[i]);
    default: return oracle_fp16_to_f64(((const uint16_t *)x)[i]);
    }
}

/* Kahan-compensated serial sum of x[0..n) and plain serial sum of |x_i|.
 * sum_abs feeds the acceptance tolerance |gpu - sum| <= 1e-5 * sum_abs. */
void oracle_sum_typed(const void *x, size_t n, int dtype, double *sum, double *sum_abs)
{
    double s = 0.0, c = 0.0, a = 0.0, ca = 0.0, plain = 0.0;
    for (size_t i = 0; i < n; ++i) {
        const double v = value_at(x, i, dtype);
        plain += v;
        const double y = v - c;
        const double t = s + y;
        c = (t - s) - y;
        s = t;
        const double av = fabs(v);
        const double ya = av - ca;
        const double ta = a + ya;
        ca = (ta - a) - ya;
        a = ta;
    }
    /* Inf/NaN inputs: the compensation term turns Inf into NaN, so report the
     * plain IEEE sum (NaN if any NaN or both infinities, else the infinity). */
    if (!isfinite(plain)) { s = plain; a = isnan(plain) ? plain : INFINITY; }
    if (sum) *sum = s;
    if (sum_abs) *sum_abs = a;
}

void oracle_sum_f16(const uint16_t *x, size_t n, double *sum, double *sum_abs)
{
    oracle_sum_typed(x, n, ORACLE_F16, sum, sum_abs);
}

/* bfloat16 and binary32 span far more than 53 bits of dynamic range, where
 * plain Kahan loses a small term that follows a huge one; the sums of those
 * types use the Kahan-Babuska (Neumaier) form, which keeps it.  Same serial
 * order, same definition R(X) = sum x_i. */
static void neumaier_sum_typed(const void *x, size_t n, int dtype, double *sum, double *sum_abs)
{
    double s = 0.0, c = 0.0, a = 0.0, ca = 0.0, plain = 0.0;
    for (size_t i = 0; i < n; ++i) {
        const double v = value_at(x, i, dtype);
        plain += v;
        const double t = s + v;
        if (fabs(s) >= fabs(v)) c += (s - t) + v; else c += (v - t) + s;
        s = t;
        const double av = fabs(v);
        const double ta = a + av;
        ca += (a - ta) + av;          /* a >= av >= 0 except at the start, where the other form is exact too */
        a = ta;
    }
    s += c;
    a += ca;
    if (!isfinite(plain)) { s = plain; a = isnan(plain) ? plain : INFINITY; }
    if (sum) *sum = s;
    if (sum_abs) *sum_abs = a;
}

void oracle_sum_bf16(const uint16_t *x, size_t n, double *sum, double *sum_abs)
{
    neumaier_sum_typed(x, n, ORACLE_BF16, sum, sum_abs);
}

void oracle_sum_f32(const uint32_t *x, size_t n, double *sum, double *sum_abs)
{
    neumaier_sum_typed(x, n, ORACLE_F32, sum, sum_abs);
}

/* Uncompensated serial binary64 sum with one running total: the serial
 * algorithm of Section 4 in double precision, which is the CPU comparison of
 * Section 5.4. */
void oracle_sum_f16_naive(const uint16_t *x, size_t n, double *sum)
{
    double s = 0.0;
    for (size_t i = 0; i < n; ++i) s += oracle_fp16_to_f64(x[i]);
    *sum = s;
}

/* The same oracle, blocked over host threads: thread t Kahan-sums the
 * contiguous chunk [t*n/T, (t+1)*n/T); chunk sums are Kahan-combined in index
 * order.  Used only to report a multi-core CPU baseline. */
struct chunk { const uint16_t *x; size_t n; double s, a; };

static void *chunk_main(void *p)
{
    struct chunk *c = (struct chunk *)p;
    oracle_sum_f16(c->x, c->n, &c->s, &c->a);
    return NULL;
}

int oracle_sum_f16_blocked(const uint16_t *x, size_t n, int threads,
                           double *sum, double *sum_abs)
{
    if (threads < 1) threads = 1;
    if (threads > 256) threads = 256;
    struct chunk *ch = (struct chunk *)calloc((size_t)threads, sizeof *ch);
    pthread_t *th = (pthread_t *)calloc((size_t)threads, sizeof *th);
    if (!ch || !th) { free(ch); free(th); return -1; }
    for (int t = 0; t < threads; ++t) {
        const size_t lo = (size_t)(((__uint128_t)n * (unsigned)t) / (unsigned)threads);
        const size_t hi = (size_t)(((__uint128_t)n * (unsigned)(t + 1)) / (unsigned)threads);
        ch[t].x = x + lo;
        ch[t].n = hi - lo;
    }
    int started = 0;
    for (; started < threads; ++started)
        if (pthread_create(&th[started], NULL, chunk_main, &ch[started])) break;
    for (int t = 0; t < started; ++t) pthread_join(th[t], NULL);
    for (int t = started; t < threads; ++t) chunk_main(&ch[t]);   /* fall back inline */
    double s = 0.0, c = 0.0, a = 0.0, ca = 0.0, plain = 0.0;
    for (int t = 0; t < threads; ++t) {
        plain += ch[t].s;
        double y = ch[t].s - c, u = s + y;
        c = (u - s) - y; s = u;
        y = ch[t].a - ca; u = a + y;
        ca = (u - a) - y; a = u;
    }
    free(ch); free(th);
    if (!isfinite(plain)) { s = plain; a = isnan(plain) ? plain : INFINITY; }
    if (sum) *sum = s;
    if (sum_abs) *sum_abs = a;
    return started;   /* threads actually created */
}
