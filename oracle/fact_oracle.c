/*
 * CPU oracle for bf16 GEMM with fp64 accumulation.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain reference that the GPU library is checked
 * against.  It shares no code, header, table or helper with the HIP path and
 * must never be linked into, or called from, the product library.
 *
 * What it computes (paper, Section 5.1 "Benchmark problems": C = A x B for the
 * square, batched and large-K problems; Section 5.2.4 / 5.2.5: the linear
 * projections of the MLP and SwiGLU patterns):
 *
 *   acc[i][j]   = sum_{k=0}^{K-1} a[i][k] * b[k][j]        (fp64, ascending k)
 *   bound[i][j] = sum_{k=0}^{K-1} |a[i][k]| * |b[k][j]|    (fp64, ascending k)
 *
 * on inputs stored as bf16 bit patterns, each widened exactly to fp64 first.
 * A product of two bf16 values has at most 16 significant bits, so every
 * product is exact in fp64 and only the additions round.
 *
 * Precision reading: the paper's kernels use reduced-precision inputs with an
 * fp32 accumulator (Listing 1, "fp16 with fp32 accumulator"; Section 5.2.3 on
 * the overflow that forced fp32 accumulation and output).  The oracle
 * accumulates in fp64 so that it is strictly more accurate than any kernel it
 * judges.
 *
 * The epilogue (bias, activation, residual) is written out in oracle/ref.py
 * with numpy fp64 operations; this file supplies only the contraction, the
 * bf16 <-> fp64 conversions and the single final rounding.
 *
 * A second input format, IEEE binary16 ("fp16", the precision the paper's own
 * kernels compute in: Listing 1; Sections 5.2.3 - 5.2.5), goes through the same
 * contraction: orc_gemm_f64_f16 differs from orc_gemm_f64 only in how a 16-bit
 * pattern is widened.  A product of two binary16 values has at most 22
 * significant bits and lies between 2^-48 and 2^32, so it is exact in fp64 too.
 * Its pins are in tests/test_oracle_pins_f16.py.
 *
 * Pins (tests/test_oracle_pins.py): identity and permutation matrices, K = 1
 * outer products on rounding ties, exact small-integer inputs, all-ones closed
 * forms, exact rational brute force on tiny shapes, an exactly rounded sum
 * (math.fsum) on long K, and torch's bfloat16 conversion as a library
 * cross-check of the rounding routine.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

/* ---- bf16 <-> wider types ------------------------------------------------ */

/* A bf16 value is the upper 16 bits of the IEEE-754 binary32 with the same
 * value, so widening is exact. */
static inline double widen(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

double orc_bf16_to_f64(uint16_t h) { return widen(h); }

/* Round an fp64 value to the nearest bf16, ties to even, in ONE rounding.
 * bf16: 1 sign, 8 exponent, 7 fraction bits; normal range 2^-126 .. below
 * 2^128; subnormal quantum 2^-133.  The value is scaled so that one unit is
 * the bf16 quantum at its magnitude, rounded to an integer with nearbyint()
 * (round-half-even in the default rounding mode), and scaled back. */
uint16_t orc_bf16_from_f64(double x)
{
    if (isnan(x)) return 0x7FC0;                       /* canonical quiet NaN */
    uint16_t sign = signbit(x) ? 0x8000 : 0;
    double ax = fabs(x);
    if (isinf(ax)) return sign | 0x7F80;
    if (ax == 0.0) return sign;

    int e;                      /* ax = m * 2^e with m in [0.5, 1) */
    (void)frexp(ax, &e);
    int exp2 = e - 1;           /* ax in [2^exp2, 2^(exp2+1)) */
    if (exp2 < -126) exp2 = -126;   /* subnormal range shares quantum 2^-133 */
    int qexp = exp2 - 7;            /* bf16 quantum at this magnitude */
    double q = nearbyint(ldexp(ax, -qexp));   /* exact scaling, one rounding */
    double r = ldexp(q, qexp);                /* exact */
    if (r >= ldexp(1.0, 128)) return sign | 0x7F80;    /* rounded up past max */
    float f = (float)r;                       /* exact: r has <= 8 sig. bits */
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    return sign | (uint16_t)(u >> 16);
}

void orc_bf16_from_f64_array(const double *in, uint16_t *out, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) out[i] = orc_bf16_from_f64(in[i]);
}

void orc_bf16_to_f64_array(const uint16_t *in, double *out, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) out[i] = widen(in[i]);
}

/* ---- IEEE binary16 <-> fp64 --------------------------------------------- */

/* binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits.  Exponent field 0:
 * subnormal, value = fraction * 2^-24; field 31: infinity or NaN; otherwise
 * (1024 + fraction) * 2^(field - 25).  Every case is exact in binary32, which
 * is built bit by bit here (the contraction calls this once per term), then in
 * fp64. */
static inline double widen_f16(uint16_t h)
{
    const uint32_t sign = (uint32_t)(h & 0x8000) << 16;
    const uint32_t field = (h >> 10) & 31, frac = h & 1023;
    uint32_t u;
    float f;
    if (field == 0) {                       /* fraction * 2^-24: at most 10 bits, exact in binary32 */
        f = (float)frac * 0x1p-24f;
        memcpy(&u, &f, sizeof u);
        u |= sign;
    } else if (field == 31) {               /* infinity (fraction 0) or NaN */
        u = sign | 0x7F800000u | (frac << 13);
    } else {                                /* the binary32 with the same value: exponent bias 127 - 15, fraction moved up 13 bits */
        u = sign | ((field + 112) << 23) | (frac << 13);
    }
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

double orc_f16_to_f64(uint16_t h) { return widen_f16(h); }

/* Round an fp64 value to the nearest binary16, ties to even, in ONE rounding
 * (the same scheme as orc_bf16_from_f64): normal range 2^-14 .. below 2^16,
 * quantum 2^(exponent - 10); subnormal quantum 2^-24; a result that rounds up
 * to 2^16 is infinity. */
uint16_t orc_f16_from_f64(double x)
{
    if (isnan(x)) return 0x7E00;                       /* canonical quiet NaN */
    uint16_t sign = signbit(x) ? 0x8000 : 0;
    double ax = fabs(x);
    if (isinf(ax)) return sign | 0x7C00;
    if (ax == 0.0) return sign;

    int e;
    (void)frexp(ax, &e);
    int exp2 = e - 1;               /* ax in [2^exp2, 2^(exp2+1)) */
    if (exp2 < -14) exp2 = -14;     /* subnormal range shares quantum 2^-24 */
    int qexp = exp2 - 10;
    double q = nearbyint(ldexp(ax, -qexp));   /* exact scaling, one rounding */
    double r = ldexp(q, qexp);                /* exact */
    if (r >= 65536.0) return sign | 0x7C00;            /* rounded up past max */
    if (r < ldexp(1.0, -14)) return sign | (uint16_t)q;   /* subnormal: q quanta of 2^-24 (0 .. 1023) */
    int e2;
    (void)frexp(r, &e2);
    int E = e2 - 1;                 /* r in [2^E, 2^(E+1)), -14 <= E <= 15 */
    int frac = (int)ldexp(r, 10 - E) - 1024;  /* exact integer in 0 .. 1023 */
    return sign | (uint16_t)(((E + 15) << 10) | frac);
}

void orc_f16_from_f64_array(const double *in, uint16_t *out, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) out[i] = orc_f16_from_f64(in[i]);
}

void orc_f16_to_f64_array(const uint16_t *in, double *out, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) out[i] = widen_f16(in[i]);
}

/* A 16-bit pattern of either format, widened exactly. */
static inline double widen_as(uint16_t h, int f16) { return f16 ? widen_f16(h) : widen(h); }

/* ---- the contraction ----------------------------------------------------- */

/*
 * acc and bound are [nrows][N] row-major fp64.  rows == NULL selects rows
 * 0..nrows-1 (then nrows must equal M for a full product); otherwise rows[r]
 * names the row of A (and of C) that output row r holds.
 *
 * trans_b == 0 : B is [K][N] row-major, leading dimension ldb (C = A * B).
 * trans_b == 1 : B is [N][K] row-major, leading dimension ldb (C = A * B^T,
 *                the weight layout of a linear projection).
 *
 * Every output element is the plain ascending-k sum.  For trans_b == 0 the
 * k loop is outside the j loop so that memory is walked along rows of B;
 * each acc[r][j] still receives its terms in the order k = 0, 1, ..., K-1.
 *
 * Returns 0, or -1 on a bad argument.  bound may be NULL.  f16 selects how the
 * 16-bit patterns of A and B are widened (0: bf16, 1: binary16); nothing else
 * depends on it.
 */
static inline int gemm_f64_as(int f16, int64_t M, int64_t N, int64_t K,
                              const uint16_t *A, int64_t lda,
                              const uint16_t *B, int64_t ldb, int trans_b,
                              const int64_t *rows, int64_t nrows,
                              double *acc, double *bound)
{
    if (M <= 0 || N <= 0 || K <= 0 || !A || !B || !acc || nrows < 0) return -1;
    if (lda < K) return -1;
    if (trans_b ? (ldb < K) : (ldb < N)) return -1;
    if (rows) {
        for (int64_t r = 0; r < nrows; ++r)
            if (rows[r] < 0 || rows[r] >= M) return -1;
    } else if (nrows > M) {
        return -1;
    }

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < nrows; ++r) {
        const int64_t i = rows ? rows[r] : r;
        const uint16_t *a = A + i * lda;
        double *c = acc + r * N;
        double *d = bound ? bound + r * N : 0;
        for (int64_t j = 0; j < N; ++j) c[j] = 0.0;
        if (d) for (int64_t j = 0; j < N; ++j) d[j] = 0.0;

        if (!trans_b) {
            for (int64_t k = 0; k < K; ++k) {
                const double aik = widen_as(a[k], f16);
                const uint16_t *b = B + k * ldb;
                for (int64_t j = 0; j < N; ++j) c[j] += aik * widen_as(b[j], f16);
                if (d) {
                    const double abs_aik = fabs(aik);
                    for (int64_t j = 0; j < N; ++j) d[j] += abs_aik * fabs(widen_as(b[j], f16));
                }
            }
        } else {
            for (int64_t j = 0; j < N; ++j) {
                const uint16_t *w = B + j * ldb;
                double s = 0.0, t = 0.0;
                for (int64_t k = 0; k < K; ++k) {
                    const double p = widen_as(a[k], f16) * widen_as(w[k], f16);
                    s += p;
                    t += fabs(p);       /* |a||b| = |ab| exactly: p is exact */
                }
                c[j] = s;
                if (d) d[j] = t;
            }
        }
    }
    return 0;
}

/* bf16 inputs */
int orc_gemm_f64(int64_t M, int64_t N, int64_t K,
                 const uint16_t *A, int64_t lda,
                 const uint16_t *B, int64_t ldb, int trans_b,
                 const int64_t *rows, int64_t nrows,
                 double *acc, double *bound)
{
    return gemm_f64_as(0, M, N, K, A, lda, B, ldb, trans_b, rows, nrows, acc, bound);
}

/* binary16 inputs */
int orc_gemm_f64_f16(int64_t M, int64_t N, int64_t K,
                     const uint16_t *A, int64_t lda,
                     const uint16_t *B, int64_t ldb, int trans_b,
                     const int64_t *rows, int64_t nrows,
                     double *acc, double *bound)
{
    return gemm_f64_as(1, M, N, K, A, lda, B, ldb, trans_b, rows, nrows, acc, bound);
}

/* Number of threads the parallel loop above will use (for reporting). */
#ifdef _OPENMP
#include <omp.h>
int orc_num_threads(void) { return omp_get_max_threads(); }
#else
int orc_num_threads(void) { return 1; }
#endif
