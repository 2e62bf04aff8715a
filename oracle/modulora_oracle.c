/*
 * CPU oracle for the ModuLoRA linear layer (forward and backward).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, obviously-correct
 * statement of what the layer computes, used only to check the GPU library.
 * It shares no code with the GPU path and the product never calls it.
 *
 * What it follows (ModuLoRA, arXiv 2309.16119):
 *   - Section 2.2, eq. (2): a b-bit quantizer stores integer codes plus zero
 *     and scale parameters, and dequantization is an affine map of the codes.
 *     Here the affine map is written in the integer-zero-point form
 *     W[n][k] = (q[n][k] - zero[g][n]) * scale[g][n], g = k / group_size,
 *     which is the same family as the paper's s*q + z with z = -s*zero.
 *   - Section 3.1, eq. (3) and Figure 1: forward  y = x W^T + (x A) B  (LoRA
 *     term scaled by lora_scale; the paper's B, A^T are called A, B here).
 *   - Figure 1 (LPLinear.backward) and Section 3.1.1: grad_input = grad_out W
 *     plus the adapter path  d y~/d y = W^T + B A^T; adapter gradients do not
 *     involve the quantized weights.
 *   - Section 3.2: the dequantized weight is materialized in a 16-bit float
 *     format; here that format is bfloat16 with one round-to-nearest-even.
 *
 * Conventions
 *   K = d_in, N = d_out, M = tokens, r = LoRA rank, G = K / group_size.
 *   qweight : uint32 [K*bits/32][N], N contiguous.  Column n's codes form one
 *             bitstream: code k occupies stream bits [k*bits, k*bits+bits),
 *             stream bit j is bit (j mod 32) of word qweight[j / 32][n].
 *   scales  : IEEE binary16 bit patterns [G][N];  zeros : uint8 [G][N].
 *   X, dY   : bfloat16 bit patterns, row-major [M][K] and [M][N].
 *   A [K][r], B [r][N] : float32.   All results are float64 unless stated.
 *
 * Every sum is accumulated in float64 in the order of the written definition.
 * The steps follow Figure 1: dequantize the whole weight, then multiply; the
 * rank-r intermediates U = X A and T = dY B^T are formed first, as defined.
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- number formats -------------------------------------------------- */

/* bfloat16 is the upper half of a binary32. */
static double bf16_bits_to_double(uint16_t h) {
    uint32_t u = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* IEEE binary16 -> double, decoded field by field (normal, subnormal, zero;
 * infinities and NaNs are mapped to the matching binary32 value). */
static float fp16_bits_to_float(uint16_t h) {
    uint32_t sign = (h >> 15) & 1u;
    uint32_t expo = (h >> 10) & 0x1Fu;
    uint32_t mant = h & 0x3FFu;
    double v;
    if (expo == 0) {
        v = (double)mant / 1024.0 / 16384.0;            /* mant * 2^-24 */
    } else if (expo == 31) {
        uint32_t u = (sign << 31) | 0x7F800000u | (mant << 13);
        float f;
        memcpy(&f, &u, sizeof f);
        return f;
    } else {
        v = 1.0 + (double)mant / 1024.0;
        int e = (int)expo - 15;
        while (e > 0) { v *= 2.0; --e; }
        while (e < 0) { v *= 0.5; ++e; }
    }
    return (float)(sign ? -v : v);                       /* exact: 11 bits */
}

/* float32 -> bfloat16 bit pattern, round to nearest, ties to even. */
static uint16_t float_to_bf16_rne(float f) {
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu)) {
        return (uint16_t)((u >> 16) | 0x0040u);          /* quiet NaN */
    }
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    return (uint16_t)(u >> 16);
}

/* ---- O1: unpack ------------------------------------------------------- */

/* Code k of column n, read from the bitstream definition. */
static uint32_t code_at(const uint32_t *qweight, int64_t N, int bits,
                        int64_t n, int64_t k) {
    int64_t j = k * bits;                 /* first stream bit of the code */
    int64_t w = j / 32;
    int o = (int)(j % 32);
    uint32_t v = qweight[w * N + n] >> o;
    if (o + bits > 32) {
        v |= qweight[(w + 1) * N + n] << (32 - o);
    }
    return v & ((1u << bits) - 1u);
}

/* q_out[n][k] (uint8, row-major [N][K]) = code k of column n. */
int oracle_unpack(const uint32_t *qweight, int64_t K, int64_t N, int bits,
                  uint8_t *q_out) {
    if (bits < 1 || bits > 8 || (K * bits) % 32 != 0) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k)
            q_out[n * K + k] = (uint8_t)code_at(qweight, N, bits, n, k);
    return 0;
}

/* ---- O2: dequantize --------------------------------------------------- */

/* Exact binary32 value (q - zero) * scale.  |q - zero| <= 255 needs 8 bits,
 * a binary16 significand has 11, so the product fits the 24-bit significand
 * of binary32 and the multiplication below does not round. */
static float dequant_value_f32(const uint32_t *qweight, const uint16_t *scales,
                               const uint8_t *zeros, int64_t N, int bits,
                               int64_t group, int64_t n, int64_t k) {
    int64_t g = k / group;
    int q = (int)code_at(qweight, N, bits, n, k);
    int z = (int)zeros[g * N + n];
    float s = fp16_bits_to_float(scales[g * N + n]);
    return (float)(q - z) * s;
}

/* W32[n][k] float32 [N][K]: the exact affine dequantization. */
int oracle_dequant_f32(const uint32_t *qweight, const uint16_t *scales,
                       const uint8_t *zeros, int64_t K, int64_t N, int bits,
                       int64_t group, float *W32) {
    if (bits < 1 || bits > 8 || group <= 0 || K % group != 0) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k)
            W32[n * K + k] = dequant_value_f32(qweight, scales, zeros, N, bits,
                                               group, n, k);
    return 0;
}

/* What[n][k] bfloat16 bit patterns [N][K]: the materialized weight. */
int oracle_dequant_bf16(const uint32_t *qweight, const uint16_t *scales,
                        const uint8_t *zeros, int64_t K, int64_t N, int bits,
                        int64_t group, uint16_t *What) {
    if (bits < 1 || bits > 8 || group <= 0 || K % group != 0) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k)
            What[n * K + k] = float_to_bf16_rne(dequant_value_f32(
                qweight, scales, zeros, N, bits, group, n, k));
    return 0;
}

/* The materialized weight What[n][k], held as float32 [N][K] (every
 * bfloat16 value is a float32 value, so nothing is lost).  Figure 1 of the
 * paper (LPLinear.forward): the weight is materialized first, then multiplied.
 * k_major only chooses the storage order of the copy (so that the loop that
 * consumes it walks memory forwards); the values are the same.
 * Returns NULL when out of memory; the caller frees it. */
static float *materialize(const uint32_t *qweight, const uint16_t *scales,
                          const uint8_t *zeros, int64_t K, int64_t N, int bits,
                          int64_t group, int k_major) {
    float *W = (float *)malloc((size_t)N * (size_t)K * sizeof(float));
    if (!W) return NULL;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            float v = (float)bf16_bits_to_double(float_to_bf16_rne(
                dequant_value_f32(qweight, scales, zeros, N, bits, group, n, k)));
            if (k_major) W[k * N + n] = v;   /* stored [K][N] */
            else         W[n * K + k] = v;   /* stored [N][K] */
        }
    return W;
}

/* P[m][j] = sum_c Act[m][c] * F(c, j), Act bfloat16 [M][C]; F(c, j) is
 * Fm[c*sc + j*sj].  Used for U = X A (sc = r, sj = 1) and T = dY B^T
 * (sc = 1, sj = N). */
static void project(const uint16_t *Act, int64_t M, int64_t C, const float *Fm,
                    int64_t sc, int64_t sj, int64_t r, double *P) {
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t j = 0; j < r; ++j) {
            double acc = 0.0;
            for (int64_t c = 0; c < C; ++c)
                acc += bf16_bits_to_double(Act[m * C + c]) *
                       (double)Fm[c * sc + j * sj];
            P[m * r + j] = acc;
        }
}

/* ---- O3: forward ------------------------------------------------------ */

/* U[m][j] = sum_k X[m][k] A[k][j]
 * Y[m][n] = sum_k X[m][k] What[n][k] + lora_scale * sum_j U[m][j] B[j][n]
 * U_out may be NULL.  r == 0 gives the plain low-precision linear map. */
int oracle_fwd(const uint32_t *qweight, const uint16_t *scales,
               const uint8_t *zeros, int64_t K, int64_t N, int bits,
               int64_t group, const uint16_t *X, int64_t M, const float *A,
               const float *B, int64_t r, double lora_scale, double *Y,
               double *U_out) {
    if (bits < 1 || bits > 8 || group <= 0 || K % group != 0) return 1;
    float *W = materialize(qweight, scales, zeros, K, N, bits, group, 0);
    double *U = (double *)malloc((size_t)(M * r + 1) * sizeof(double));
    if (!W || !U) { free(W); free(U); return 2; }
    project(X, M, K, A, r, 1, r, U);
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            double base = 0.0;
            for (int64_t k = 0; k < K; ++k)
                base += bf16_bits_to_double(X[m * K + k]) * (double)W[n * K + k];
            double lora = 0.0;
            for (int64_t j = 0; j < r; ++j)
                lora += U[m * r + j] * (double)B[j * N + n];
            Y[m * N + n] = base + lora_scale * lora;
        }
    if (U_out) memcpy(U_out, U, (size_t)(M * r) * sizeof(double));
    free(W);
    free(U);
    return 0;
}

/* ---- O4: backward with respect to the input --------------------------- */

/* T[m][j]  = sum_n dY[m][n] B[j][n]
 * dX[m][k] = sum_n dY[m][n] What[n][k] + lora_scale * sum_j T[m][j] A[k][j]
 * T_out may be NULL. */
int oracle_bwd_input(const uint32_t *qweight, const uint16_t *scales,
                     const uint8_t *zeros, int64_t K, int64_t N, int bits,
                     int64_t group, const uint16_t *dY, int64_t M,
                     const float *A, const float *B, int64_t r,
                     double lora_scale, double *dX, double *T_out) {
    if (bits < 1 || bits > 8 || group <= 0 || K % group != 0) return 1;
    float *W = materialize(qweight, scales, zeros, K, N, bits, group, 1);
    double *T = (double *)malloc((size_t)(M * r + 1) * sizeof(double));
    if (!W || !T) { free(W); free(T); return 2; }
    project(dY, M, N, B, 1, N, r, T);
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k) {
            double base = 0.0;
            for (int64_t n = 0; n < N; ++n)
                base += bf16_bits_to_double(dY[m * N + n]) * (double)W[k * N + n];
            double lora = 0.0;
            for (int64_t j = 0; j < r; ++j)
                lora += T[m * r + j] * (double)A[k * r + j];
            dX[m * K + k] = base + lora_scale * lora;
        }
    if (T_out) memcpy(T_out, T, (size_t)(M * r) * sizeof(double));
    free(W);
    free(T);
    return 0;
}

/* ---- O5: adapter gradients -------------------------------------------- */

/* dA[k][j] = lora_scale * sum_m X[m][k] * T[m][j],  T = dY B^T
 * dB[j][n] = lora_scale * sum_m U[m][j] * dY[m][n], U = X A
 * The quantized weights do not appear. */
int oracle_bwd_lora(int64_t K, int64_t N, int64_t M, int64_t r,
                    double lora_scale, const uint16_t *X, const uint16_t *dY,
                    const float *A, const float *B, double *dA, double *dB) {
    double *U = (double *)malloc((size_t)(M * r + 1) * sizeof(double));
    double *T = (double *)malloc((size_t)(M * r + 1) * sizeof(double));
    if (!U || !T) { free(U); free(T); return 2; }
    project(X, M, K, A, r, 1, r, U);
    project(dY, M, N, B, 1, N, r, T);
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < K; ++k)
        for (int64_t j = 0; j < r; ++j) {
            double acc = 0.0;
            for (int64_t m = 0; m < M; ++m)
                acc += bf16_bits_to_double(X[m * K + k]) * T[m * r + j];
            dA[k * r + j] = lora_scale * acc;
        }
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t j = 0; j < r; ++j) {
            double acc = 0.0;
            for (int64_t m = 0; m < M; ++m)
                acc += U[m * r + j] * bf16_bits_to_double(dY[m * N + n]);
            dB[j * N + n] = lora_scale * acc;
        }
    free(U);
    free(T);
    return 0;
}

/* Number of OpenMP threads the products above run on. */
int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
