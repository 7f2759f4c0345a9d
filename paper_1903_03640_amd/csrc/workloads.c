/*
 * workloads.c -- seeded synthetic input generators (host side).
 *
 * These routines only produce bytes.  They hold none of the reduction's
 * arithmetic and are the one piece of code that both the GPU tests and the
 * CPU oracle's tests draw inputs from.
 *
 * Generator: counter based, so any sub-range can be produced independently
 * and in parallel:
 *     z(seed, i) = mix64(seed * 0x9E3779B97F4A7C15 + i)       (mod 2^64)
 * with mix64 the finaliser of the public-domain SplitMix64 generator, and
 *     u24(seed, i) = (z >> 40) * 2^-24   in [0, 1), exact in binary32.
 *
 * Build: gcc -O2 -std=c11 -fopenmp -shared -fPIC -o libredux_workloads.so workloads.c -lm
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

static inline uint64_t mix64(uint64_t z)
{
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

static inline uint64_t z_of(uint64_t seed, uint64_t i)
{
    return mix64(seed * 0x9E3779B97F4A7C15ull + i);
}

static inline double u24_of(uint64_t seed, uint64_t i)
{
    return (double)(z_of(seed, i) >> 40) * 0x1p-24;
}

/* binary64 -> binary16 bit pattern, round to nearest even, one rounding. */
static uint16_t f64_to_f16(double v)
{
    uint16_t sign = signbit(v) ? 0x8000u : 0;
    double a = fabs(v);
    if (isnan(a)) return (uint16_t)(sign | 0x7e00u);
    if (a >= 65520.0) return (uint16_t)(sign | 0x7c00u);     /* rounds to infinity */
    if (a < 0x1p-14) {
        /* subnormal range: spacing 2^-24; rint() rounds to nearest even.  A value that
         * rounds up to 1024 units is the smallest normal, whose pattern is also 1024. */
        return (uint16_t)(sign | (uint16_t)rint(a * 0x1p24));
    }
    int e;
    double m = frexp(a, &e);                 /* a = m * 2^e, m in [0.5, 1) */
    int mant = (int)rint(m * 2048.0);        /* 11 significant bits, in [1024, 2048] */
    if (mant == 2048) { mant = 1024; e += 1; }
    int field = e + 14;                      /* a = (mant/1024) * 2^(e-1), bias 15 */
    return (uint16_t)(sign | (uint16_t)(field << 10) | (uint16_t)(mant - 1024));
}

/*
 * out[k] = binary16(u24(seed, start + k))            if symmetric == 0   -> [0, 1)
 *        = binary16(2 * u24(seed, start + k) - 1)    if symmetric != 0   -> [-1, 1)
 * A value that rounds up to 1.0 is replaced by the largest binary16 below 1
 * (0x3BFF), so the stated half-open range holds after rounding.
 */
void redux_gen_uniform_f16(uint16_t *out, uint64_t seed, uint64_t start, uint64_t count, int symmetric)
{
#pragma omp parallel for schedule(static)
    for (uint64_t k = 0; k < count; ++k) {
        double u = u24_of(seed, start + k);
        uint16_t h = f64_to_f16(symmetric ? 2.0 * u - 1.0 : u);
        if (h == 0x3c00u) h = 0x3bffu;
        out[k] = h;
    }
}

/*
 * out[k] = binary16(N(0,1)) by the Box-Muller transform in binary64:
 *   u1 = u24(seed, 2i), u2 = u24(seed, 2i+1), i = start + k
 *   x  = sqrt(-2 ln(1 - u1)) * cos(2 pi u2)        (1 - u1 is in (0, 1], so the log is finite)
 */
void redux_gen_normal_f16(uint16_t *out, uint64_t seed, uint64_t start, uint64_t count)
{
    const double two_pi = 6.283185307179586476925286766559;
#pragma omp parallel for schedule(static)
    for (uint64_t k = 0; k < count; ++k) {
        uint64_t i = start + k;
        double u1 = u24_of(seed, 2 * i);
        double u2 = u24_of(seed, 2 * i + 1);
        double r = sqrt(-2.0 * log(1.0 - u1));
        out[k] = f64_to_f16(r * cos(two_pi * u2));
    }
}

/* out[k] = top byte of z(seed, start + k) read as int8: uniform on [-128, 127]. */
void redux_gen_uniform_i8(int8_t *out, uint64_t seed, uint64_t start, uint64_t count)
{
#pragma omp parallel for schedule(static)
    for (uint64_t k = 0; k < count; ++k)
        out[k] = (int8_t)(uint8_t)(z_of(seed, start + k) >> 56);
}

/* Sum of the raw storage patterns mod 2^64: lets two runs prove that they saw the same bytes. */
uint64_t redux_checksum_u16(const uint16_t *x, uint64_t count)
{
    uint64_t s = 0;
#pragma omp parallel for schedule(static) reduction(+ : s)
    for (uint64_t k = 0; k < count; ++k) s += x[k];
    return s;
}

uint64_t redux_checksum_u8(const uint8_t *x, uint64_t count)
{
    uint64_t s = 0;
#pragma omp parallel for schedule(static) reduction(+ : s)
    for (uint64_t k = 0; k < count; ++k) s += x[k];
    return s;
}
