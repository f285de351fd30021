/*
 * CPU oracle for the weight-only-quantized linear layer  y = x * Deq(W)^T.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is the plain definition written out, slow on
 * purpose, and shares nothing with the GPU library.  Only tests, the smoke
 * check and the benchmark's CPU-baseline leg may call it.
 *
 * What it follows (RWKVQuant, Sec. 2.2 and Sec. 3.1):
 *   - Scalar quantization, Eq. "SQ":  Q(x) = clamp(round(x/s) + z, 0, 2^b - 1).
 *     The paper names the inverse only as "Deq" (Sec. 3.2); it is the algebraic
 *     inverse  w = (q - z) * s,  taken here as one binary32 subtraction followed
 *     by one binary32 multiplication (round to nearest even, no fused
 *     multiply-add, no re-association).  s and z are stored per group of
 *     `group` consecutive input channels as fp16 and widened exactly.
 *   - Vector quantization, Eq. "VQ": W viewed as (N*K/d, d) row-major, i.e. each
 *     vector is d consecutive input channels of one output row; a k-bit index
 *     selects a row of a (2^k, d) codebook.  Dequantization returns that
 *     codebook row, widened exactly from fp16.  One codebook serves one
 *     block_rows x block_cols block of W.
 *   - Hybrid choice, Eq. "optimization goal": each matrix is wholly SQ or wholly
 *     VQ (phi_m); the caller picks the function.
 *   - The linear maps of App. A.1 (r_t = W_r(...), ...):  y[m][n] = sum_k
 *     w[n][k] * x[m][k], k ascending, multiply then add, in binary32 or (for
 *     checking the binary32 sum itself) in binary64.
 *
 * Bit strings: a row of packed fields is an array of uint32 words read as one
 * little-endian bit string: bit p of the string is bit (p & 31) of word p >> 5.
 * Field i of width b occupies bits [b*i, b*i + b) and may straddle two words.
 *
 * Pins (tests/test_oracle_*.py): hand-packed words and straddling fields,
 * closed-form SQ values, exact rational arithmetic for the rounding order,
 * exact codebook reproduction and block mapping, the SQ-as-VQ identity,
 * numpy's fp16 conversions, brute-force dot products, one-hot/ones inputs.
 *
 * Build: gcc -O2 -fopenmp -ffp-contract=off -fno-fast-math -shared -fPIC.
 * Threads only split output rows, so results never depend on the thread count.
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---------- scalar format conversions (exact widening, nearest-even narrowing) ---------- */

static float bits_to_float(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static uint32_t float_to_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }

/* fp16 bit pattern -> binary32, exact for every input. */
float rwkvq_oracle_half_to_float(uint16_t h) {
    uint32_t sign = (uint32_t)(h >> 15) << 31;
    uint32_t e = (h >> 10) & 0x1F;
    uint32_t m = h & 0x3FF;
    if (e == 0x1F) return bits_to_float(sign | 0x7F800000u | (m << 13));   /* inf / nan */
    if (e == 0) {                                                            /* zero / subnormal */
        float v = (float)m * (1.0f / 16777216.0f);                           /* m * 2^-24, exact */
        return sign ? -v : v;
    }
    return bits_to_float(sign | ((e + 112) << 23) | (m << 13));
}

/* binary32 -> bf16 bit pattern, round to nearest even. */
uint16_t rwkvq_oracle_float_to_bf16(float f) {
    uint32_t u = float_to_bits(f);
    if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu))               /* nan stays nan */
        return (uint16_t)((u >> 16) | 0x0040);
    uint32_t lsb = (u >> 16) & 1;
    return (uint16_t)((u + 0x7FFFu + lsb) >> 16);
}

float rwkvq_oracle_bf16_to_float(uint16_t b) { return bits_to_float((uint32_t)b << 16); }

/* binary32 -> fp16 bit pattern, round to nearest even (overflow -> inf, gradual underflow). */
uint16_t rwkvq_oracle_float_to_half(float f) {
    uint32_t u = float_to_bits(f);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000);
    uint32_t a = u & 0x7FFFFFFFu;
    if (a >= 0x7F800000u) return (uint16_t)(sign | 0x7C00 | (a > 0x7F800000u ? 0x0200 : 0));
    int e = (int)(a >> 23) - 127;                      /* unbiased exponent */
    uint32_t m = (a & 0x007FFFFFu) | 0x00800000u;      /* 24-bit significand (normal input) */
    if ((a >> 23) == 0) return sign;                   /* binary32 subnormal: far below fp16 range */
    int shift;                                         /* bits dropped from the 24-bit significand */
    if (e >= -14) shift = 13;                          /* fp16 normal: keep 11 bits */
    else shift = 13 + (-14 - e);                       /* fp16 subnormal: keep fewer */
    if (shift > 25) return sign;                       /* below half of the smallest subnormal */
    uint32_t kept = m >> shift;
    uint32_t rem = m & ((1u << shift) - 1);
    uint32_t half = 1u << (shift - 1);
    if (rem > half || (rem == half && (kept & 1))) kept++;
    uint32_t out;
    if (e >= -14) out = ((uint32_t)(e + 15 - 1) << 10) + kept;   /* kept carries the hidden 1 */
    else out = kept;                                             /* may round up into the normal range */
    if (out >= 0x7C00) out = 0x7C00;
    return (uint16_t)(sign | out);
}

/* ---------- bit-string fields ---------- */

uint32_t rwkvq_oracle_field(const uint32_t* words, int width, int64_t index) {
    int64_t p = (int64_t)width * index;
    int64_t w = p >> 5;
    int off = (int)(p & 31);
    uint64_t two = words[w];
    if (off + width > 32) two |= (uint64_t)words[w + 1] << 32;
    return (uint32_t)((two >> off) & ((1u << width) - 1u));
}

void rwkvq_oracle_unpack(const uint32_t* words, int64_t rows, int64_t words_per_row,
                         int width, int64_t fields_per_row, uint16_t* out) {
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t i = 0; i < fields_per_row; ++i)
            out[r * fields_per_row + i] =
                (uint16_t)rwkvq_oracle_field(words + r * words_per_row, width, i);
}

/* ---------- dequantization of one output row ---------- */

static void sq_row(const uint32_t* row_words, const uint16_t* row_scales, const uint16_t* row_zeros,
                   int64_t K, int bits, int group, float* w) {
    for (int64_t k = 0; k < K; ++k) {
        float q = (float)rwkvq_oracle_field(row_words, bits, k);
        float z = rwkvq_oracle_half_to_float(row_zeros[k / group]);
        float s = rwkvq_oracle_half_to_float(row_scales[k / group]);
        float d = q - z;          /* first rounding  */
        w[k] = d * s;             /* second rounding */
    }
}

static void vq_row(const uint32_t* row_words, const uint16_t* codebooks, int64_t n, int64_t K,
                   int vdim, int kbits, int block_rows, int block_cols, float* w) {
    int64_t entries = (int64_t)1 << kbits;
    int64_t col_blocks = K / block_cols;
    for (int64_t j = 0; j < K / vdim; ++j) {
        uint32_t idx = rwkvq_oracle_field(row_words, kbits, j);
        int64_t cb = (n / block_rows) * col_blocks + (j * vdim) / block_cols;
        const uint16_t* entry = codebooks + (cb * entries + idx) * vdim;
        for (int e = 0; e < vdim; ++e) w[j * vdim + e] = rwkvq_oracle_half_to_float(entry[e]);
    }
}

/* weight_round: 0 = keep binary32, 1 = nearest fp16, 2 = nearest bf16 (value kept in a float). */
static void round_row(float* w, int64_t K, int weight_round) {
    if (weight_round == 1)
        for (int64_t k = 0; k < K; ++k) w[k] = rwkvq_oracle_half_to_float(rwkvq_oracle_float_to_half(w[k]));
    else if (weight_round == 2)
        for (int64_t k = 0; k < K; ++k) w[k] = rwkvq_oracle_bf16_to_float(rwkvq_oracle_float_to_bf16(w[k]));
}

void rwkvq_oracle_round(float* a, int64_t n, int weight_round) { round_row(a, n, weight_round); }

/* ---------- full-matrix dequantization: w is [N][K] binary32 ---------- */

void rwkvq_oracle_sq_dequant(const uint32_t* codes, const uint16_t* scales, const uint16_t* zeros,
                             int64_t N, int64_t K, int bits, int group, float* w) {
    int64_t wpr = K * bits / 32, G = K / group;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        sq_row(codes + n * wpr, scales + n * G, zeros + n * G, K, bits, group, w + n * K);
}

void rwkvq_oracle_vq_dequant(const uint32_t* indices, const uint16_t* codebooks, int64_t N, int64_t K,
                             int vdim, int kbits, int block_rows, int block_cols, float* w) {
    int64_t wpr = (K / vdim) * kbits / 32;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        vq_row(indices + n * wpr, codebooks, n, K, vdim, kbits, block_rows, block_cols, w + n * K);
}

/* ---------- contraction ---------- */

static double dot_row(const float* w, const float* x, int64_t K, int acc64) {
    if (acc64) {
        double a = 0.0;
        for (int64_t k = 0; k < K; ++k) a += (double)w[k] * (double)x[k];
        return a;
    }
    float a = 0.0f;
    for (int64_t k = 0; k < K; ++k) { float p = w[k] * x[k]; a = a + p; }
    return (double)a;
}

/* y[m][n] = sum_k w[n][k] x[m][k];  w [N][K], x [M][K], y [M][N] (binary64 holds either result). */
void rwkvq_oracle_gemm(const float* w, const float* x, int64_t M, int64_t N, int64_t K,
                       int acc64, double* y) {
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t m = 0; m < M; ++m) y[m * N + n] = dot_row(w + n * K, x + m * K, K, acc64);
}

/* Dequantize row by row and contract: same arithmetic as dequant + gemm, without holding W. */
void rwkvq_oracle_sq_linear(const uint32_t* codes, const uint16_t* scales, const uint16_t* zeros,
                            int64_t N, int64_t K, int bits, int group, const float* x, int64_t M,
                            int weight_round, int acc64, double* y) {
    int64_t wpr = K * bits / 32, G = K / group;
#pragma omp parallel
    {
        float* w = (float*)malloc((size_t)K * sizeof(float));
#pragma omp for schedule(static)
        for (int64_t n = 0; n < N; ++n) {
            sq_row(codes + n * wpr, scales + n * G, zeros + n * G, K, bits, group, w);
            round_row(w, K, weight_round);
            for (int64_t m = 0; m < M; ++m) y[m * N + n] = dot_row(w, x + m * K, K, acc64);
        }
        free(w);
    }
}

void rwkvq_oracle_vq_linear(const uint32_t* indices, const uint16_t* codebooks, int64_t N, int64_t K,
                            int vdim, int kbits, int block_rows, int block_cols, const float* x,
                            int64_t M, int weight_round, int acc64, double* y) {
    int64_t wpr = (K / vdim) * kbits / 32;
#pragma omp parallel
    {
        float* w = (float*)malloc((size_t)K * sizeof(float));
#pragma omp for schedule(static)
        for (int64_t n = 0; n < N; ++n) {
            vq_row(indices + n * wpr, codebooks, n, K, vdim, kbits, block_rows, block_cols, w);
            round_row(w, K, weight_round);
            for (int64_t m = 0; m < M; ++m) y[m * N + n] = dot_row(w, x + m * K, K, acc64);
        }
        free(w);
    }
}

int rwkvq_oracle_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
