/* Host check of the two short sequences the SQ encoder kernel uses in place of the hardware's
 * division (Sec. 2.2, Eq. "SQ": s = (max - min) / 7, z = -min / s, q = rne(w / s + z), every
 * division a correctly rounded binary32 one):
 *   reciprocal: r0 within a few units in the last place of 1 / s,  r = fma(fma(-s, r0, 1), r0, r0)
 *   quotient:   q = v * r,  then STEPS times  q = fma(fma(-s, q, v), r, q)
 * against the C compiler's IEEE division, for every finite non-zero fp16 divisor s and
 *   - every bf16 and every fp16 dividend that is zero or has a magnitude in [2^-60, 2^60] (one step),
 *   - random binary32 dividends of that range (two steps), and (max - min) / 7 on random values.
 * Prints the number of mismatches per check; exit status 0 iff all are zero. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

static float f16_value(uint16_t h) {
    uint32_t e = (h >> 10) & 31, m = h & 1023;
    float v = e == 0 ? ldexpf((float)m, -24) : e == 31 ? (m ? NAN : INFINITY) : ldexpf((float)(m + 1024), (int)e - 25);
    return (h >> 15) ? -v : v;
}
static float from_bits(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static uint32_t to_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static int in_range(float v) { float a = fabsf(v); return a == 0.0f || (a >= 0x1p-60f && a <= 0x1p60f); }
static float quotient(float v, float s, float r, int steps) {
    float q = v * r;
    for (int i = 0; i < steps; ++i) q = fmaf(fmaf(-s, q, v), r, q);
    return q;
}
static int same(float got, float want) { return want == 0.0f ? got == 0.0f : to_bits(got) == to_bits(want); }

int main(int argc, char** argv) {
    const int randoms = argc > 1 ? atoi(argv[1]) : 20000;
    long long bad_r = 0, bad_16 = 0, bad_32 = 0, bad_7 = 0;
#pragma omp parallel for schedule(dynamic, 64) reduction(+ : bad_r, bad_16, bad_32)
    for (int h = 1; h <= 0x7BFF; ++h) {
        const float s = f16_value((uint16_t)h), r = 1.0f / s;
        for (int d = -4; d <= 4; ++d) {
            const float r0 = from_bits(to_bits(r) + (uint32_t)d);
            if (to_bits(fmaf(fmaf(-s, r0, 1.0f), r0, r0)) != to_bits(r)) bad_r++;
        }
        for (uint32_t b = 0; b < 65536; ++b) {
            const float v = from_bits(b << 16), w = f16_value((uint16_t)b);
            if (in_range(v) && !same(quotient(v, s, r, 1), v / s)) bad_16++;
            if (in_range(w) && !same(quotient(w, s, r, 1), w / s)) bad_16++;
        }
        uint64_t x = 0x9E3779B97F4A7C15ull * (uint64_t)h + 1;
        for (int i = 0; i < randoms; ++i) {
            x ^= x << 13; x ^= x >> 7; x ^= x << 17;
            const uint32_t e = 67 + (uint32_t)((x >> 40) % 120);                 /* 2^-60 .. below 2^60 */
            const float v = from_bits(((uint32_t)(x >> 63) << 31) | (e << 23) | ((uint32_t)x & 0x7FFFFFu));
            if (!same(quotient(v, s, r, 2), v / s)) bad_32++;
        }
    }
    uint64_t x = 88172645463325252ull;
    for (long i = 0; i < 2000L * randoms; ++i) {
        x ^= x << 13; x ^= x >> 7; x ^= x << 17;
        const uint32_t e = 87 + (uint32_t)((x >> 40) % 140);                     /* 2^-40 .. below 2^100 */
        const float v = from_bits((e << 23) | ((uint32_t)x & 0x7FFFFFu));
        if (!same(quotient(v, 7.0f, 0x1.24924ap-3f, 2), v / 7.0f)) bad_7++;
    }
    printf("reciprocal %lld quotient16 %lld quotient32 %lld seventh %lld\n", bad_r, bad_16, bad_32, bad_7);
    return (bad_r || bad_16 || bad_32 || bad_7) ? 1 : 0;
}
