/*
 * Plain C oracle of the LiquidQuant W4A8 GEMM (TEST INFRASTRUCTURE ONLY).
 *
 * Only tests/, the smoke check and the cpu_baseline leg of the benchmark may
 * build or call this file.  It shares no code, header, table or helper with the
 * HIP library.  No intrinsics, no BLAS, no blocking: each step is the paper's
 * definition written as nested loops, parallelised over output rows with OpenMP.
 *
 * Steps (paper notation; W is [N,K], X is [M,K], Y is [M,N], G = K/g):
 *   1. unpack canonical nibbles   byte[n][k/2] = code[n][k] | code[n][k+1] << 4
 *   2. dequantise, Eq. 8          Wd = code * s_u8 + min(Q_i8),  min = a - 128
 *      cross-checked per element against Eq. 12  (code * s_u8 + a) XOR 0x80
 *   3. main loop (Sec. 2)         ACC[m][n] = sum_k X[m][k] * Wd[n][k]  in int64,
 *                                 checked to fit INT32
 *   4. epilogue (Sec. 4, 5.3)     Y[m][n] = ACC * s_x[m] * s_w[n]  in double
 *      (the caller rounds Y once to FP16).
 *
 * Pinned by tests/test_oracle_pins.py against the numpy oracle, pure-Python brute
 * force and the exact float64 product.
 *
 * Return: 0 ok; -1 Eq. 8 left the INT8 range; -2 Eq. 8 and Eq. 12 disagree or
 * Eq. 11 violated; -3 an accumulator left INT32; -4 bad arguments / out of memory.
 */
#include <stdint.h>
#include <stdlib.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int lqq_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Steps 1-2: canonical packed codes -> dequantised INT8 matrix Wd[N][K]. */
int lqq_oracle_dequant(int N, int K, int g, const uint8_t *packed, const uint8_t *s_u8,
                       const uint8_t *a, int8_t *Wd)
{
    if (N < 1 || K < 2 || g < 1 || K % g != 0 || K % 2 != 0) return -4;
    const int G = K / g;
    int err = 0;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int k = 0; k < K; ++k) {
            const uint8_t byte = packed[(size_t)n * (K / 2) + k / 2];
            const int code = (k % 2 == 0) ? (byte & 0x0F) : (byte >> 4);
            const int s = s_u8[(size_t)n * G + k / g];
            const int off = a[(size_t)n * G + k / g];
            const int mn = off - 128;
            const int plain = code * s + mn;              /* Eq. 8 */
            if (plain < -128 || plain > 127) {
#pragma omp atomic write
                err = -1;
                continue;
            }
            const int t = code * s + off;                 /* Eq. 11: must stay in UINT8 */
            const uint8_t bits = (uint8_t)((uint8_t)t ^ 0x80u); /* Eq. 12 */
            if (t > 255 || (int8_t)bits != (int8_t)plain) {
#pragma omp atomic write
                err = -2;
                continue;
            }
            Wd[(size_t)n * K + k] = (int8_t)plain;
        }
    }
    return err;
}

/* Steps 3-4 on an already dequantised Wd. */
int lqq_oracle_matmul_scale(int M, int N, int K, const int8_t *X, const float *s_x,
                            const int8_t *Wd, const float *s_w, int32_t *ACC, double *Y)
{
    if (M < 1 || N < 1 || K < 1) return -4;
    int err = 0;
#pragma omp parallel for collapse(2) schedule(static)
    for (int m = 0; m < M; ++m) {
        for (int n = 0; n < N; ++n) {
            const int8_t *x = X + (size_t)m * K;
            const int8_t *w = Wd + (size_t)n * K;
            int64_t acc = 0;
            for (int k = 0; k < K; ++k) acc += (int64_t)x[k] * (int64_t)w[k];
            if (acc > INT32_MAX || acc < INT32_MIN) {
#pragma omp atomic write
                err = -3;
            }
            if (ACC) ACC[(size_t)m * N + n] = (int32_t)acc;
            if (Y) Y[(size_t)m * N + n] = (double)acc * (double)s_x[m] * (double)s_w[n];
        }
    }
    return err;
}

/* Whole path, steps 1-4. */
int lqq_oracle_w4a8_gemm(int M, int N, int K, int g, const int8_t *X, const float *s_x,
                         const uint8_t *packed, const uint8_t *s_u8, const uint8_t *a,
                         const float *s_w, int32_t *ACC, double *Y)
{
    if (M < 1 || N < 1 || K < 2) return -4;
    int8_t *Wd = (int8_t *)malloc((size_t)N * K);
    if (!Wd) return -4;
    int rc = lqq_oracle_dequant(N, K, g, packed, s_u8, a, Wd);
    if (rc == 0) rc = lqq_oracle_matmul_scale(M, N, K, X, s_x, Wd, s_w, ACC, Y);
    free(Wd);
    return rc;
}
