/* Oracle GEMM in plain C: C[i][j] = sum_k A[i][k] * B[j][k], fp64 accumulation in k order
 * (Sec. 3.2, tiled-GEMM paragraph: the plain definition the tiled kernel must reproduce).
 * Operands are storage-encoded (bf16 bits, or OCP e4m3 bytes with per-tensor scales) and are
 * decoded to double here.  Rows of C are independent and are spread over OpenMP threads;
 * there is no blocking or reordering of the k sum.
 *
 * TEST INFRASTRUCTURE: linked only by the oracle's Python wrapper.
 * Build: gcc -O2 -fopenmp -shared -fPIC -o libgemm_ref.so gemm_ref.c -lm
 */
#include <math.h>
#include <omp.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static double bf16_to_double(uint16_t h) {
    uint32_t w = ((uint32_t)h) << 16; /* bf16 = upper half of binary32 */
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

static double e4m3_to_double(uint8_t b) {
    int e = (b >> 3) & 0xF, m = b & 0x7;
    double v;
    if (e == 15 && m == 7) return NAN;
    if (e == 0) v = ldexp((double)m / 8.0, -6);
    else v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return (b & 0x80) ? -v : v;
}

int oracle_threads(void) { return omp_get_max_threads(); }

static int gemm_rows(int64_t M, int64_t N, int64_t K, const double *a, const double *b,
                     double *c, int threads) {
    if (threads <= 0) threads = omp_get_max_threads();
#pragma omp parallel for schedule(static) num_threads(threads)
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < N; ++j) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k) acc += a[i * K + k] * b[j * K + k];
            c[i * N + j] = acc;
        }
    }
    return 0;
}

int oracle_gemm_bf16(int64_t M, int64_t N, int64_t K, const uint16_t *A, const uint16_t *B,
                     double *C, int threads) {
    if (M < 0 || N < 0 || K < 0) return -1;
    double *a = (double *)malloc(sizeof(double) * (size_t)(M * K + 1));
    double *b = (double *)malloc(sizeof(double) * (size_t)(N * K + 1));
    if (!a || !b) { free(a); free(b); return -2; }
    for (int64_t t = 0; t < M * K; ++t) a[t] = bf16_to_double(A[t]);
    for (int64_t t = 0; t < N * K; ++t) b[t] = bf16_to_double(B[t]);
    int rc = gemm_rows(M, N, K, a, b, C, threads);
    free(a); free(b);
    return rc;
}

int oracle_gemm_e4m3(int64_t M, int64_t N, int64_t K, const uint8_t *A, const uint8_t *B,
                     double scale_a, double scale_b, double *C, int threads) {
    if (M < 0 || N < 0 || K < 0) return -1;
    double *a = (double *)malloc(sizeof(double) * (size_t)(M * K + 1));
    double *b = (double *)malloc(sizeof(double) * (size_t)(N * K + 1));
    if (!a || !b) { free(a); free(b); return -2; }
    for (int64_t t = 0; t < M * K; ++t) a[t] = scale_a * e4m3_to_double(A[t]);
    for (int64_t t = 0; t < N * K; ++t) b[t] = scale_b * e4m3_to_double(B[t]);
    int rc = gemm_rows(M, N, K, a, b, C, threads);
    free(a); free(b);
    return rc;
}
