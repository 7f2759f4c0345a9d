/*
 * redux_oracle.c -- plain, slow CPU oracle for the arithmetic
 * reduction R(X) = sum_{i=1..n} x_i (paper Section III, the definition of the
 * arithmetic reduction).
 *
 * THIS IS TEST INFRASTRUCTURE.  It exists so that the GPU library can be
 * checked against something that is obviously correct.  It shares no code,
 * header, table or helper with the GPU library, and the GPU library never
 * calls it.  Only the test-suite, the smoke check and the "cpu_baseline" leg
 * of the benchmark may load it.
 *
 * The method of the paper (Section IV-A: two matrix-multiply-accumulate
 * operations against an all-ones operand, applied hierarchically) only
 * re-associates the additions of the definition and multiplies by one, so in
 * exact arithmetic it reaches the plain sum.  The oracle is therefore the
 * definition written out, in arithmetic wide enough that its own rounding is
 * far below the tolerance that the GPU result is held to:
 *
 *   binary16 input  -> every value is decoded exactly to binary64, then
 *       summed in binary64 four independent ways:
 *         serial   : one accumulator, elements taken left to right (the
 *                    sequential algorithm that Section III starts from);
 *         pairwise : recursive halving with a 128-element serial base case;
 *         neumaier : Kahan-Babuska compensated serial sum (compensated
 *                    summation is the remedy named in Section II);
 *         exact    : every finite binary16 is an integer multiple of 2^-24
 *                    with |multiple| < 2^41, so the sum of multiples is
 *                    accumulated exactly in a 128-bit integer (n < 2^86) and
 *                    converted once.
 *   int8 input      -> int64 serial sum (exact for n < 2^56).
 *   bfloat16, binary32, and the two 8-bit floating-point formats of the OCP
 *   8-bit floating point specification (E4M3: no infinities, one NaN pattern per
 *   sign; E5M2: IEEE-like) -> each value decoded exactly to binary64, then the
 *   same pairwise and Neumaier sums; the 8-bit formats also have an exact
 *   fixed-point sum (every value is a multiple of 2^-9 resp. 2^-16).
 *
 * Every routine also returns sum |x_i|, which the tolerance for cancelling
 * sums is stated against.
 *
 * Non-finite inputs follow IEEE-754 addition: NaN, or +Inf together with
 * -Inf, gives NaN; otherwise an infinity dominates.  The exact routine
 * reports their presence through *nonfinite and leaves them out of the
 * integer sum.
 *
 * Many-core form (the *_chunks routines): the array is cut into contiguous
 * chunks, chunk t of T being elements [t*n/T, (t+1)*n/T); every chunk is summed
 * by the single-threaded routine above (one OpenMP thread per chunk) and the
 * chunk sums are added in chunk order, so the result depends on T but never on
 * scheduling.  It exists so that the CPU baseline can be timed on all host cores.
 *
 * Build: gcc -O2 -std=c11 -fopenmp -shared -fPIC -o libredux_oracle.so redux_oracle.c -lm
 * (without -fopenmp the chunks are summed one after the other, with the same result)
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_ERR_NULL (-1)

/* ---- binary16 decode ---------------------------------------------------- */

/* IEEE-754 binary16: 1 sign bit, 5 exponent bits (bias 15), 10 fraction bits. */
double redux_oracle_f16_decode(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int f = h & 0x3ff;
    double v;
    if (e == 0) {
        v = ldexp((double)f, -24);            /* zero and subnormals: f * 2^-24 */
    } else if (e == 31) {
        v = (f == 0) ? INFINITY : NAN;
    } else {
        v = ldexp((double)(1024 + f), e - 25); /* (1 + f/1024) * 2^(e-15) */
    }
    return sign ? -v : v;
}

/* All 65536 decoded values; filled from redux_oracle_f16_decode on first use. */
static double g_decode[65536];
static int g_decode_ready = 0;

static const double *decode_table(void)
{
    if (!g_decode_ready) {
        for (uint32_t h = 0; h < 65536u; ++h)
            g_decode[h] = redux_oracle_f16_decode((uint16_t)h);
        g_decode_ready = 1;
    }
    return g_decode;
}

/* ---- binary16 sums ------------------------------------------------------ */

/* Section III: one accumulator, elements taken in index order. */
int redux_oracle_sum_f16_serial(const uint16_t *x, size_t n, double *sum, double *sum_abs)
{
    if ((n && !x) || !sum || !sum_abs) return ORACLE_ERR_NULL;
    const double *t = decode_table();
    double s = 0.0, a = 0.0;
    for (size_t i = 0; i < n; ++i) {
        double v = t[x[i]];
        s += v;
        a += fabs(v);
    }
    *sum = s;
    *sum_abs = a;
    return ORACLE_OK;
}

static void pairwise(const double *t, const uint16_t *x, size_t n, double *s, double *a)
{
    if (n <= 128) {
        double ss = 0.0, aa = 0.0;
        for (size_t i = 0; i < n; ++i) {
            double v = t[x[i]];
            ss += v;
            aa += fabs(v);
        }
        *s = ss;
        *a = aa;
        return;
    }
    size_t half = n / 2;
    double s0, a0, s1, a1;
    pairwise(t, x, half, &s0, &a0);
    pairwise(t, x + half, n - half, &s1, &a1);
    *s = s0 + s1;
    *a = a0 + a1;
}

/* Primary oracle: binary64 pairwise summation. */
int redux_oracle_sum_f16(const uint16_t *x, size_t n, double *sum, double *sum_abs)
{
    if ((n && !x) || !sum || !sum_abs) return ORACLE_ERR_NULL;
    pairwise(decode_table(), x, n, sum, sum_abs);
    return ORACLE_OK;
}

/* Cross-check: Neumaier's variant of Kahan's compensated summation. */
int redux_oracle_sum_f16_neumaier(const uint16_t *x, size_t n, double *sum, double *sum_abs)
{
    if ((n && !x) || !sum || !sum_abs) return ORACLE_ERR_NULL;
    const double *t = decode_table();
    double s = 0.0, c = 0.0;            /* never build this file with -ffast-math */
    double a = 0.0;
    int nonfinite = 0;
    for (size_t i = 0; i < n; ++i) {
        double v = t[x[i]];
        if (!isfinite(v)) nonfinite = 1;
        double tt = s + v;
        if (fabs(s) >= fabs(v)) c += (s - tt) + v;
        else                    c += (v - tt) + s;
        s = tt;
        a += fabs(v);
    }
    /* The compensation term is meaningless (Inf - Inf) once a non-finite value came in. */
    *sum = nonfinite ? s : s + c;
    *sum_abs = a;
    return ORACLE_OK;
}

/*
 * Cross-check: exact fixed-point sum in units of 2^-24.
 * The integer total is returned as hi:lo (two's complement, 128 bits) and
 * rounded once to binary64 in *sum.  *nonfinite is 1 if an Inf or NaN was
 * seen (such elements are skipped in the integer sums).
 */
int redux_oracle_sum_f16_exact(const uint16_t *x, size_t n, double *sum, double *sum_abs,
                               int64_t *hi, uint64_t *lo, int *nonfinite)
{
    if ((n && !x) || !sum || !sum_abs || !hi || !lo || !nonfinite) return ORACLE_ERR_NULL;
    __int128 s = 0, a = 0;
    int nf = 0;
    for (size_t i = 0; i < n; ++i) {
        uint16_t h = x[i];
        int e = (h >> 10) & 0x1f;
        int64_t f = h & 0x3ff;
        int64_t units;
        if (e == 31) { nf = 1; continue; }
        if (e == 0) units = f;                          /* f * 2^-24 */
        else        units = (1024 + f) << (e - 1);      /* (1024+f) * 2^(e-25) = ((1024+f) << (e-1)) * 2^-24 */
        a += units;
        s += (h & 0x8000) ? -units : units;
    }
    *hi = (int64_t)(s >> 64);
    *lo = (uint64_t)s;
    /* __int128 -> double conversion rounds to nearest; scaling by 2^-24 is exact. */
    *sum = ldexp((double)s, -24);
    *sum_abs = ldexp((double)a, -24);
    *nonfinite = nf;
    return ORACLE_OK;
}

/* ---- int8 sum ----------------------------------------------------------- */

int redux_oracle_sum_i8(const int8_t *x, size_t n, int64_t *sum, int64_t *sum_abs)
{
    if ((n && !x) || !sum || !sum_abs) return ORACLE_ERR_NULL;
    int64_t s = 0, a = 0;
    for (size_t i = 0; i < n; ++i) {
        int64_t v = x[i];
        s += v;
        a += v < 0 ? -v : v;
    }
    *sum = s;
    *sum_abs = a;
    return ORACLE_OK;
}

/* ---- segmented forms: the same sums, one per contiguous segment ---------- */

int redux_oracle_sum_segmented_f16(const uint16_t *x, size_t nseg, size_t seglen,
                                   double *sum, double *sum_abs)
{
    if ((nseg && seglen && !x) || (nseg && (!sum || !sum_abs))) return ORACLE_ERR_NULL;
    for (size_t s = 0; s < nseg; ++s) {
        int rc = redux_oracle_sum_f16(x + s * seglen, seglen, &sum[s], &sum_abs[s]);
        if (rc) return rc;
    }
    return ORACLE_OK;
}

int redux_oracle_sum_segmented_i8(const int8_t *x, size_t nseg, size_t seglen,
                                  int64_t *sum, int64_t *sum_abs)
{
    if ((nseg && seglen && !x) || (nseg && (!sum || !sum_abs))) return ORACLE_ERR_NULL;
    for (size_t s = 0; s < nseg; ++s) {
        int rc = redux_oracle_sum_i8(x + s * seglen, seglen, &sum[s], &sum_abs[s]);
        if (rc) return rc;
    }
    return ORACLE_OK;
}

/* ---- other floating-point element types: decode exactly, then the same sums ------------------------ */

#define ORACLE_BF16 2
#define ORACLE_F32 3
#define ORACLE_F8E4M3 4
#define ORACLE_F8E5M2 5
#define ORACLE_ERR_DTYPE (-2)

/* bfloat16: the upper 16 bits of a binary32 (1 sign, 8 exponent bits with bias 127, 7 fraction bits). */
double redux_oracle_bf16_decode(uint16_t h)
{
    int sign = (h >> 15) & 1, e = (h >> 7) & 0xff, f = h & 0x7f;
    double v;
    if (e == 0) v = ldexp((double)f, -133);                  /* subnormal: f * 2^-7 * 2^-126 */
    else if (e == 255) v = (f == 0) ? INFINITY : NAN;
    else v = ldexp((double)(128 + f), e - 134);              /* (1 + f/128) * 2^(e-127) */
    return sign ? -v : v;
}

/* binary32 from its bit pattern (1, 8 with bias 127, 23). */
double redux_oracle_f32_decode(uint32_t w)
{
    int sign = (w >> 31) & 1, e = (w >> 23) & 0xff;
    uint32_t f = w & 0x7fffffu;
    double v;
    if (e == 0) v = ldexp((double)f, -149);
    else if (e == 255) v = (f == 0) ? INFINITY : NAN;
    else v = ldexp((double)(0x800000u + f), e - 150);
    return sign ? -v : v;
}

/* OCP E4M3: 1 sign, 4 exponent bits (bias 7), 3 fraction bits; no infinities; S.1111.111 is NaN;
 * largest finite value 448 = 1.75 * 2^8. */
double redux_oracle_f8e4m3_decode(uint8_t b)
{
    int sign = (b >> 7) & 1, e = (b >> 3) & 0xf, f = b & 7;
    double v;
    if (e == 15 && f == 7) v = NAN;
    else if (e == 0) v = ldexp((double)f, -9);               /* f/8 * 2^-6 */
    else v = ldexp((double)(8 + f), e - 10);                 /* (1 + f/8) * 2^(e-7) */
    return sign ? -v : v;
}

/* OCP E5M2: 1 sign, 5 exponent bits (bias 15), 2 fraction bits; IEEE-like infinities and NaNs. */
double redux_oracle_f8e5m2_decode(uint8_t b)
{
    int sign = (b >> 7) & 1, e = (b >> 2) & 0x1f, f = b & 3;
    double v;
    if (e == 31) v = (f == 0) ? INFINITY : NAN;
    else if (e == 0) v = ldexp((double)f, -16);              /* f/4 * 2^-14 */
    else v = ldexp((double)(4 + f), e - 17);                 /* (1 + f/4) * 2^(e-15) */
    return sign ? -v : v;
}

static double decode_at(const void *x, size_t i, int dtype)
{
    switch (dtype) {
    case ORACLE_BF16: return redux_oracle_bf16_decode(((const uint16_t *)x)[i]);
    case ORACLE_F32: return redux_oracle_f32_decode(((const uint32_t *)x)[i]);
    case ORACLE_F8E4M3: return redux_oracle_f8e4m3_decode(((const uint8_t *)x)[i]);
    default: return redux_oracle_f8e5m2_decode(((const uint8_t *)x)[i]);
    }
}

static void pairwise_any(const void *x, size_t lo, size_t n, int dtype, double *s, double *a)
{
    if (n <= 128) {
        double ss = 0.0, aa = 0.0;
        for (size_t i = 0; i < n; ++i) {
            double v = decode_at(x, lo + i, dtype);
            ss += v;
            aa += fabs(v);
        }
        *s = ss;
        *a = aa;
        return;
    }
    size_t half = n / 2;
    double s0, a0, s1, a1;
    pairwise_any(x, lo, half, dtype, &s0, &a0);
    pairwise_any(x, lo + half, n - half, dtype, &s1, &a1);
    *s = s0 + s1;
    *a = a0 + a1;
}

/* Primary oracle for dtype 2..5: binary64 pairwise sum and sum of |x|. */
int redux_oracle_sum_any(const void *x, size_t n, int dtype, double *sum, double *sum_abs)
{
    if (dtype < ORACLE_BF16 || dtype > ORACLE_F8E5M2) return ORACLE_ERR_DTYPE;
    if ((n && !x) || !sum || !sum_abs) return ORACLE_ERR_NULL;
    pairwise_any(x, 0, n, dtype, sum, sum_abs);
    return ORACLE_OK;
}

/* Cross-check for dtype 2..5: Neumaier-compensated serial sum. */
int redux_oracle_sum_any_neumaier(const void *x, size_t n, int dtype, double *sum, double *sum_abs)
{
    if (dtype < ORACLE_BF16 || dtype > ORACLE_F8E5M2) return ORACLE_ERR_DTYPE;
    if ((n && !x) || !sum || !sum_abs) return ORACLE_ERR_NULL;
    double s = 0.0, c = 0.0, a = 0.0;
    int nonfinite = 0;
    for (size_t i = 0; i < n; ++i) {
        double v = decode_at(x, i, dtype);
        if (!isfinite(v)) nonfinite = 1;
        double tt = s + v;
        if (fabs(s) >= fabs(v)) c += (s - tt) + v;
        else                    c += (v - tt) + s;
        s = tt;
        a += fabs(v);
    }
    *sum = nonfinite ? s : s + c;
    *sum_abs = a;
    return ORACLE_OK;
}

/* Exact fixed-point sum for the 8-bit formats, in units of 2^-9 (E4M3) or 2^-16 (E5M2); NaN/Inf are
 * skipped and reported.  |units| <= 448 * 2^9 resp. 57344 * 2^16 per element, so int64 holds any n < 2^31. */
int redux_oracle_sum_f8_exact(const uint8_t *x, size_t n, int dtype, int64_t *units, int64_t *units_abs, int *nonfinite)
{
    if (dtype != ORACLE_F8E4M3 && dtype != ORACLE_F8E5M2) return ORACLE_ERR_DTYPE;
    if ((n && !x) || !units || !units_abs || !nonfinite) return ORACLE_ERR_NULL;
    int64_t s = 0, a = 0;
    int nf = 0;
    for (size_t i = 0; i < n; ++i) {
        uint8_t b = x[i];
        int64_t u;
        if (dtype == ORACLE_F8E4M3) {
            int e = (b >> 3) & 0xf, f = b & 7;
            if (e == 15 && f == 7) { nf = 1; continue; }
            u = e == 0 ? f : (int64_t)(8 + f) << (e - 1);      /* (8+f) * 2^(e-10) = ((8+f) << (e-1)) * 2^-9 */
        } else {
            int e = (b >> 2) & 0x1f, f = b & 3;
            if (e == 31) { nf = 1; continue; }
            u = e == 0 ? f : (int64_t)(4 + f) << (e - 1);      /* (4+f) * 2^(e-17) = ((4+f) << (e-1)) * 2^-16 */
        }
        a += u;
        s += (b & 0x80) ? -u : u;
    }
    *units = s;
    *units_abs = a;
    *nonfinite = nf;
    return ORACLE_OK;
}

int redux_oracle_sum_segmented_any(const void *x, size_t nseg, size_t seglen, int dtype, double *sum, double *sum_abs)
{
    if (dtype < ORACLE_BF16 || dtype > ORACLE_F8E5M2) return ORACLE_ERR_DTYPE;
    if ((nseg && seglen && !x) || (nseg && (!sum || !sum_abs))) return ORACLE_ERR_NULL;
    for (size_t s = 0; s < nseg; ++s) pairwise_any(x, s * seglen, seglen, dtype, &sum[s], &sum_abs[s]);
    return ORACLE_OK;
}

/* ---- many-core form: contiguous chunks, one thread each, combined in chunk order ---------- */

#define ORACLE_ERR_CHUNKS (-2)
#define ORACLE_MAX_CHUNKS 4096

/* Threads an OpenMP parallel region would get (1 when built without OpenMP). */
int redux_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* first element of chunk t when n elements are cut into T chunks; chunk T starts at n */
static size_t chunk_begin(size_t n, size_t t, size_t T)
{
    return (size_t)(((unsigned __int128)n * t) / T);
}

int redux_oracle_sum_f16_chunks(const uint16_t *x, size_t n, int chunks, double *sum, double *sum_abs)
{
    if ((n && !x) || !sum || !sum_abs) return ORACLE_ERR_NULL;
    if (chunks < 1 || chunks > ORACLE_MAX_CHUNKS) return ORACLE_ERR_CHUNKS;
    static double ps[ORACLE_MAX_CHUNKS], pa[ORACLE_MAX_CHUNKS];
    const double *t = decode_table();       /* filled before the threads start */
    const size_t T = (size_t)chunks;
#pragma omp parallel for num_threads(chunks) schedule(static, 1)
    for (int c = 0; c < chunks; ++c) {
        const size_t lo = chunk_begin(n, (size_t)c, T), hi = chunk_begin(n, (size_t)c + 1, T);
        pairwise(t, x + lo, hi - lo, &ps[c], &pa[c]);
    }
    double s = 0.0, a = 0.0;
    for (int c = 0; c < chunks; ++c) {      /* chunk order, whatever order the threads finished in */
        s += ps[c];
        a += pa[c];
    }
    *sum = s;
    *sum_abs = a;
    return ORACLE_OK;
}

int redux_oracle_sum_i8_chunks(const int8_t *x, size_t n, int chunks, int64_t *sum, int64_t *sum_abs)
{
    if ((n && !x) || !sum || !sum_abs) return ORACLE_ERR_NULL;
    if (chunks < 1 || chunks > ORACLE_MAX_CHUNKS) return ORACLE_ERR_CHUNKS;
    static int64_t ps[ORACLE_MAX_CHUNKS], pa[ORACLE_MAX_CHUNKS];
    const size_t T = (size_t)chunks;
#pragma omp parallel for num_threads(chunks) schedule(static, 1)
    for (int c = 0; c < chunks; ++c) {
        const size_t lo = chunk_begin(n, (size_t)c, T), hi = chunk_begin(n, (size_t)c + 1, T);
        (void)redux_oracle_sum_i8(x + lo, hi - lo, &ps[c], &pa[c]);
    }
    int64_t s = 0, a = 0;
    for (int c = 0; c < chunks; ++c) {
        s += ps[c];
        a += pa[c];
    }
    *sum = s;
    *sum_abs = a;
    return ORACLE_OK;
}

/* Segmented: segments are independent, so chunk t takes segments [t*nseg/T, (t+1)*nseg/T) whole;
 * every segment's sum is exactly the single-threaded one. */
int redux_oracle_sum_segmented_f16_chunks(const uint16_t *x, size_t nseg, size_t seglen, int chunks,
                                          double *sum, double *sum_abs)
{
    if ((nseg && seglen && !x) || (nseg && (!sum || !sum_abs))) return ORACLE_ERR_NULL;
    if (chunks < 1 || chunks > ORACLE_MAX_CHUNKS) return ORACLE_ERR_CHUNKS;
    const double *t = decode_table();
    const size_t T = (size_t)chunks;
#pragma omp parallel for num_threads(chunks) schedule(static, 1)
    for (int c = 0; c < chunks; ++c) {
        const size_t lo = chunk_begin(nseg, (size_t)c, T), hi = chunk_begin(nseg, (size_t)c + 1, T);
        for (size_t sgm = lo; sgm < hi; ++sgm) pairwise(t, x + sgm * seglen, seglen, &sum[sgm], &sum_abs[sgm]);
    }
    return ORACLE_OK;
}
