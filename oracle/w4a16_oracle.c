/*
 * CPU oracle for the W4A16 mixed-precision matrix multiplication.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It defines what the GPU library must
 * compute and is used only by the tests, by the smoke check and by the
 * benchmark's host-baseline leg.  It shares no code, header, table or helper
 * with the HIP path and the product never calls it.
 *
 * What it computes is the plain definition of the operation (Section 3,
 * Eq. 2):   C = A * Dequant(W),   Dequant(W) = s (W - z)
 * with A in FP16 [M,K], W in INT4 [K,N] and C produced from wider partial
 * sums (Section 3: partial results are FP32 and cast to FP16 at the very end;
 * Algorithm 1 lists the inputs and the FP16 output).  The method only
 * re-associates this one sum (Split-K, tiling), so the oracle is the
 * definition itself, written as scalar loops, summed in binary64.
 *
 * Readings where the paper is silent (storage, Section 2.2 only says that
 * 4-bit values are packed into wider integers such as INT32):
 *   - codes are unsigned 0..15; eight codes of consecutive k share one 32-bit
 *     word of Wp[K/8, N] (row-major, n contiguous); code of k = 8r+i sits in
 *     bits 4i .. 4i+3 of Wp[r, n];
 *   - s and z are per (group, n) with group = `group` consecutive k;
 *     scales are FP16 [K/group, N]; zero points are unsigned 0..15, eight of
 *     consecutive n per 32-bit word of Zp[K/group, N/8], the one of n = 8c+j
 *     in bits 4j .. 4j+3, stored as the value itself;
 *   - w[k,n] = float(s) * float(q - z): an 11-bit significand times an
 *     integer of magnitude <= 15 has at most 15 significant bits, so the
 *     binary32 product is exact and needs no rounding rule;
 *   - the dequantized weight is NOT rounded to FP16 before the product.
 *
 * Plain C, no intrinsics.  OpenMP only spreads independent output columns
 * over the host cores; it does not change any sum.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* IEEE-754 binary16 bit pattern -> binary32 value (exact; every binary16
 * value, subnormals, infinities and NaNs included, is a binary32 value). */
float w4a16_oracle_half_to_float(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) & 1u;
    uint32_t expo = (uint32_t)(h >> 10) & 0x1Fu;
    uint32_t frac = (uint32_t)h & 0x3FFu;
    float mag;
    if (expo == 0) {
        /* zero or subnormal: frac * 2^-24 */
        mag = (float)frac * (1.0f / 16777216.0f);
    } else if (expo == 31) {
        uint32_t bits = 0x7F800000u | (frac << 13);
        memcpy(&mag, &bits, sizeof mag);
    } else {
        /* (1024 + frac) * 2^(expo - 25) */
        mag = ldexpf((float)(1024u + frac), (int)expo - 25);
    }
    return sign ? -mag : mag;
}

/* Code q[k,n] in 0..15 (Section 2.2: 4-bit values packed in INT32). */
static inline int code_at(const uint32_t *Wp, int N, int k, int n)
{
    uint32_t word = Wp[(size_t)(k / 8) * (size_t)N + (size_t)n];
    return (int)((word >> (4 * (k % 8))) & 0xFu);
}

/* Zero point z[g,n] in 0..15. */
static inline int zero_at(const uint32_t *Zp, int N, int g, int n)
{
    uint32_t word = Zp[(size_t)g * (size_t)(N / 8) + (size_t)(n / 8)];
    return (int)((word >> (4 * (n % 8))) & 0xFu);
}

/* Dequant(W)[k,n] = s (W - z)  (Eq. 2), in binary32 (exact, see header). */
static inline float weight_at(const uint32_t *Wp, const uint16_t *scales,
                              const uint32_t *Zp, int group, int N, int k, int n)
{
    int g = k / group;
    int q = code_at(Wp, N, k, n);
    int z = zero_at(Zp, N, g, n);
    float s = w4a16_oracle_half_to_float(scales[(size_t)g * (size_t)N + (size_t)n]);
    return s * (float)(q - z);
}

static int shape_ok(int group, int M, int N, int K)
{
    if (M < 0 || N < 1 || K < 1 || group < 1) return 0;
    if (K % 8 != 0 || N % 8 != 0 || K % group != 0) return 0;
    return 1;
}

/* q[K,N] (uint8) <- Wp[K/8,N]. */
int w4a16_oracle_unpack_codes(const uint32_t *Wp, int K, int N, uint8_t *q)
{
    if (!shape_ok(8, 0, N, K)) return 1;
    for (int k = 0; k < K; ++k)
        for (int n = 0; n < N; ++n)
            q[(size_t)k * N + n] = (uint8_t)code_at(Wp, N, k, n);
    return 0;
}

/* z[G,N] (uint8) <- Zp[G,N/8]. */
int w4a16_oracle_unpack_zeros(const uint32_t *Zp, int G, int N, uint8_t *z)
{
    if (G < 1 || N < 1 || N % 8 != 0) return 1;
    for (int g = 0; g < G; ++g)
        for (int n = 0; n < N; ++n)
            z[(size_t)g * N + n] = (uint8_t)zero_at(Zp, N, g, n);
    return 0;
}

/* w[K,N] (binary32) <- Dequant(W) of Eq. 2. */
int w4a16_oracle_dequant(const uint32_t *Wp, const uint16_t *scales,
                         const uint32_t *Zp, int group, int K, int N, float *w)
{
    if (!shape_ok(group, 0, N, K)) return 1;
    for (int k = 0; k < K; ++k)
        for (int n = 0; n < N; ++n)
            w[(size_t)k * N + n] = weight_at(Wp, scales, Zp, group, N, k, n);
    return 0;
}

/* One output element of Eq. 2: sum_k X[m,k] * Dequant(W)[k,n], every product
 * and sum in binary64 (a binary16 times a 15-bit binary32 value is exact in
 * binary64; only the additions round).  k runs 0..K-1 in order. */
static double element_at(const uint16_t *X, const uint32_t *Wp,
                         const uint16_t *scales, const uint32_t *Zp,
                         int group, int N, int K, int m, int n)
{
    double acc = 0.0;
    for (int k = 0; k < K; ++k) {
        double x = (double)w4a16_oracle_half_to_float(X[(size_t)m * K + k]);
        double w = (double)weight_at(Wp, scales, Zp, group, N, k, n);
        acc += x * w;
    }
    return acc;
}

/* ref[M,N] (binary64) <- A * Dequant(W)  (Eq. 2). */
int w4a16_oracle_gemm(const uint16_t *X, const uint32_t *Wp,
                      const uint16_t *scales, const uint32_t *Zp,
                      int group, int M, int N, int K, double *ref)
{
    if (!shape_ok(group, M, N, K)) return 1;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int m = 0; m < M; ++m)
            ref[(size_t)m * N + n] = element_at(X, Wp, scales, Zp, group, N, K, m, n);
    return 0;
}

/* The same element-by-element definition on chosen columns only:
 * ref[M,ncols], ref[m,j] = (A * Dequant(W))[m, cols[j]].  For spot checks of
 * shapes whose full result takes the host too long. */
int w4a16_oracle_gemm_columns(const uint16_t *X, const uint32_t *Wp,
                              const uint16_t *scales, const uint32_t *Zp,
                              int group, int M, int N, int K,
                              const int32_t *cols, int ncols, double *ref)
{
    if (!shape_ok(group, M, N, K) || ncols < 0) return 1;
    for (int j = 0; j < ncols; ++j)
        if (cols[j] < 0 || cols[j] >= N) return 1;
#pragma omp parallel for schedule(static)
    for (int j = 0; j < ncols; ++j)
        for (int m = 0; m < M; ++m)
            ref[(size_t)m * ncols + j] = element_at(X, Wp, scales, Zp, group, N, K, m, cols[j]);
    return 0;
}

/* ---- variants the paper names without evaluating them ---------------------- */

/* Symmetric quantization (Section 2.1: "symmetric" means z = 0 in Eq. 1, on
 * signed codes).  Reading for this library's unsigned storage: the stored
 * code is the signed code plus 8, so Dequant(W)[k,n] = s (q - 8) and there is
 * no zero-point tensor.  Binary32, exact for the same reason as weight_at. */
static inline float symmetric_weight_at(const uint32_t *Wp, const uint16_t *scales,
                                        int group, int N, int k, int n)
{
    int grp = k / group;
    int signed_code = code_at(Wp, N, k, n) - 8;   /* -8 .. 7 */
    float s = w4a16_oracle_half_to_float(scales[(size_t)grp * (size_t)N + (size_t)n]);
    return s * (float)signed_code;
}

/* w[K,N] (binary32) <- s (W - 8). */
int w4a16_oracle_dequant_symmetric(const uint32_t *Wp, const uint16_t *scales,
                                   int group, int K, int N, float *w)
{
    if (!shape_ok(group, 0, N, K)) return 1;
    for (int k = 0; k < K; ++k)
        for (int n = 0; n < N; ++n)
            w[(size_t)k * N + n] = symmetric_weight_at(Wp, scales, group, N, k, n);
    return 0;
}

/* ref[M,N] (binary64) <- A * s (W - 8): Eq. 2 with the symmetric reading,
 * every product and sum in binary64, k ascending. */
int w4a16_oracle_gemm_symmetric(const uint16_t *X, const uint32_t *Wp,
                                const uint16_t *scales, int group,
                                int M, int N, int K, double *ref)
{
    if (!shape_ok(group, M, N, K)) return 1;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int m = 0; m < M; ++m) {
            double sum = 0.0;
            for (int k = 0; k < K; ++k) {
                double x = (double)w4a16_oracle_half_to_float(X[(size_t)m * K + k]);
                sum += x * (double)symmetric_weight_at(Wp, scales, group, N, k, n);
            }
            ref[(size_t)m * N + n] = sum;
        }
    return 0;
}

/* BF16 activations.  The paper's A is "16-bit floating point"; its own runs use
 * FP16, BF16 is the other 16-bit format models ship in.  A bfloat16 is the
 * upper half of a binary32: sign, the same 8 exponent bits, the top 7
 * fraction bits.  Decoded here field by field (not by a bit cast), so that a
 * mistake in either would show. */
float w4a16_oracle_bfloat_to_float(uint16_t b)
{
    uint32_t negative = (uint32_t)(b >> 15) & 1u;
    uint32_t biased = (uint32_t)(b >> 7) & 0xFFu;
    uint32_t mant = (uint32_t)b & 0x7Fu;
    float val;
    if (biased == 0) {
        /* zero or subnormal: mant * 2^-133 */
        val = ldexpf((float)mant, -133);
    } else if (biased == 255) {
        val = mant ? nanf("") : INFINITY;
    } else {
        /* (128 + mant) * 2^(biased - 134) */
        val = ldexpf((float)(128u + mant), (int)biased - 134);
    }
    return negative ? -val : val;
}

/* ref[M,N] (binary64) <- A * Dequant(W) (Eq. 2) with A given as bfloat16 bit
 * patterns; W, s, z exactly as in the FP16 form (the scales stay FP16: they
 * belong to the quantized weights).  A bfloat16 (8 significant bits) times a
 * 15-bit binary32 weight is exact in binary64; only the additions round. */
int w4a16_oracle_gemm_bf16(const uint16_t *Xb, const uint32_t *Wp,
                           const uint16_t *scales, const uint32_t *Zp,
                           int group, int M, int N, int K, double *ref)
{
    if (!shape_ok(group, M, N, K)) return 1;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int m = 0; m < M; ++m) {
            double total = 0.0;
            for (int kk = 0; kk < K; ++kk) {
                double xb = (double)w4a16_oracle_bfloat_to_float(Xb[(size_t)m * K + kk]);
                total += xb * (double)weight_at(Wp, scales, Zp, group, N, kk, n);
            }
            ref[(size_t)m * N + n] = total;
        }
    return 0;
}

/* Threads the gemm above spreads its columns over. */
int w4a16_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
