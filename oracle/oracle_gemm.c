/*
 * CPU ORACLE -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, obviously-correct definition of what the tiled GEMM path
 * computes.  Only tests, the smoke check and the benchmark's cpu_baseline leg
 * may call this file; the GPU library never links or loads it and shares no
 * source with it.
 *
 * What is computed (paper section 3.1: operations on matrices are reduced to
 * operations on tiles, C_ij accumulates A_ik * B_kj over every k; section 2:
 * forward and backward passes are such products):
 *
 *     C_out[m,n] = C_in[m,n] + sum_{k=0}^{K-1} opA[m,k] * opB[k,n]
 *
 * Every input element is widened exactly to fp64 (fp32 and bf16 both embed
 * exactly), products and sums are fp64, k ascends.  Tiling does not change
 * the value, so the untiled definition is the oracle; oracle_gemm_tiled()
 * walks T x T tiles with clamped edge extents and exists to check exactly
 * that invariant.
 *
 * Element access is by explicit strides so NN / TN / NT are index arithmetic
 * only:  opA[m,k] = A[m*sam + k*sak],  opB[k,n] = B[k*sbk + n*sbn].
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

static inline double load_elem(const void *base, int64_t idx, int dtype)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)base)[idx];
    /* bf16: the 16 stored bits are the top half of an IEEE fp32 */
    uint32_t bits = ((uint32_t)((const uint16_t *)base)[idx]) << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Untiled definition.  c_in may be NULL (meaning zero).  c_out is M x N
 * row-major fp64, leading dimension N. */
int oracle_gemm(const void *A, const void *B, const float *c_in, double *c_out,
                int64_t M, int64_t N, int64_t K,
                int64_t sam, int64_t sak, int64_t sbk, int64_t sbn,
                int64_t ldc_in, int dtype)
{
    if (M < 0 || N < 0 || K < 0) return -1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        double *row = c_out + m * N;
        for (int64_t n = 0; n < N; ++n)
            row[n] = c_in ? (double)c_in[m * ldc_in + n] : 0.0;
        for (int64_t k = 0; k < K; ++k) {
            const double a = load_elem(A, m * sam + k * sak, dtype);
            for (int64_t n = 0; n < N; ++n)
                row[n] += a * load_elem(B, k * sbk + n * sbn, dtype);
        }
    }
    return 0;
}

static inline int64_t min64(int64_t a, int64_t b) { return a < b ? a : b; }

/* Same value through the tile algorithm of section 3.1: C tile (i,j) receives
 * one contribution per k-step, tiles at the right/bottom edge are clamped to
 * the matrix.  Written separately from oracle_gemm on purpose. */
int oracle_gemm_tiled(const void *A, const void *B, const float *c_in, double *c_out,
                      int64_t M, int64_t N, int64_t K, int64_t T,
                      int64_t sam, int64_t sak, int64_t sbk, int64_t sbn,
                      int64_t ldc_in, int dtype)
{
    if (M < 0 || N < 0 || K < 0 || T <= 0) return -1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return -1;
    const int64_t nI = (M + T - 1) / T, nJ = (N + T - 1) / T, nK = (K + T - 1) / T;
#pragma omp parallel for schedule(dynamic)
    for (int64_t task = 0; task < nI * nJ; ++task) {
        const int64_t ti = task / nJ, tj = task % nJ;
        const int64_t r0 = ti * T, r1 = min64(M, r0 + T);
        const int64_t c0 = tj * T, c1 = min64(N, c0 + T);
        for (int64_t m = r0; m < r1; ++m)
            for (int64_t n = c0; n < c1; ++n)
                c_out[m * N + n] = c_in ? (double)c_in[m * ldc_in + n] : 0.0;
        for (int64_t tk = 0; tk < nK; ++tk) {
            const int64_t k0 = tk * T, k1 = min64(K, k0 + T);
            for (int64_t m = r0; m < r1; ++m)
                for (int64_t n = c0; n < c1; ++n) {
                    double s = 0.0;
                    for (int64_t k = k0; k < k1; ++k)
                        s += load_elem(A, m * sam + k * sak, dtype) *
                             load_elem(B, k * sbk + n * sbn, dtype);
                    c_out[m * N + n] += s;
                }
        }
    }
    return 0;
}

/* Sampled entries: out[s] = c_in[rows[s], cols[s]] + dot over all k.  Used
 * where the full product is out of reach for the CPU. */
int oracle_gemm_samples(const void *A, const void *B, const float *c_in, double *out,
                        const int64_t *rows, const int64_t *cols, int64_t n_samples,
                        int64_t K,
                        int64_t sam, int64_t sak, int64_t sbk, int64_t sbn,
                        int64_t ldc_in, int dtype)
{
    if (n_samples < 0 || K < 0) return -1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t s = 0; s < n_samples; ++s) {
        const int64_t m = rows[s], n = cols[s];
        double acc = c_in ? (double)c_in[m * ldc_in + n] : 0.0;
        for (int64_t k = 0; k < K; ++k)
            acc += load_elem(A, m * sam + k * sak, dtype) *
                   load_elem(B, k * sbk + n * sbn, dtype);
        out[s] = acc;
    }
    return 0;
}
