/*
 * CPU fp64 oracle for the BCR (Block-based Column-Row) sparse product.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing on the product path may call this file:
 * it exists so that the GPU library can be checked against a plain, slow,
 * obviously correct statement of what the method computes.  It shares no code
 * with the library and never sees the library's compact format: it masks a
 * dense matrix and multiplies it with a naive triple loop.
 *
 * What it follows:
 *  - BCR sparsity (Section 3.2, "Motivation of Fine-Grained BCR Pruning"; the
 *    constraint set of Section 5.2): the weight matrix is cut into equal
 *    blocks; each block independently drops whole rows and whole columns, and
 *    the survivors of a block form a full (kept rows) x (kept columns) matrix.
 *  - Unified GEMM view (Section 3.1): a CONV layer becomes weight matrix x
 *    im2col input matrix, FC / RNN gates become matrix x vector; both are
 *    Y = W_bcr * X with the pruned weight matrix as the left operand.
 *
 * Precision: everything in fp64.  Callers widen fp16 / bf16 / fp32 storage
 * values exactly before calling.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* W_bcr[i][k] = W[i][k] if row (i mod BR) and column (k mod BC) are both kept
 * by block (i / BR, k / BC), else +0.0.  Blocks are numbered row-major.
 * Returns 0, or -1 on a malformed argument. */
int bcr_oracle_mask(const double *W, int64_t M, int64_t K, int32_t BR, int32_t BC,
                    const int32_t *row_ptr, const uint16_t *row_idx,
                    const int32_t *col_ptr, const uint16_t *col_idx,
                    double *Wm)
{
    if (!W || !Wm || !row_ptr || !col_ptr || BR <= 0 || BC <= 0 || M % BR || K % BC)
        return -1;
    int64_t nbr = M / BR, nbc = K / BC;
    unsigned char *rk = (unsigned char *)malloc((size_t)BR);
    unsigned char *ck = (unsigned char *)malloc((size_t)BC);
    if (!rk || !ck) { free(rk); free(ck); return -1; }
    for (int64_t s = 0; s < nbr; ++s) {
        for (int64_t c = 0; c < nbc; ++c) {
            int64_t b = s * nbc + c;
            memset(rk, 0, (size_t)BR);
            memset(ck, 0, (size_t)BC);
            for (int32_t t = row_ptr[b]; t < row_ptr[b + 1]; ++t) rk[row_idx[t]] = 1;
            for (int32_t t = col_ptr[b]; t < col_ptr[b + 1]; ++t) ck[col_idx[t]] = 1;
            for (int32_t i = 0; i < BR; ++i) {
                for (int32_t j = 0; j < BC; ++j) {
                    int64_t at = (s * BR + i) * K + (c * BC + j);
                    Wm[at] = (rk[i] && ck[j]) ? W[at] : 0.0;
                }
            }
        }
    }
    free(rk);
    free(ck);
    return 0;
}

/* Y[i][n] = sum_k Wm[i][k] * X[k][n]        (M x K times K x N, row-major)
 * S[i][n] = sum_k |Wm[i][k] * X[k][n]|      (scale for the error metric; may be NULL)
 * skip_zero != 0 skips k with Wm[i][k] == 0, which changes nothing but time
 * (and the sign of a zero result). */
int bcr_oracle_matmul(const double *Wm, const double *X, int64_t M, int64_t K, int64_t N,
                      double *Y, double *S, int32_t skip_zero)
{
    if (!Wm || !X || !Y || M < 0 || K < 0 || N < 0)
        return -1;
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t i = 0; i < M; ++i) {
        double *y = Y + i * N;
        double *s = S ? S + i * N : NULL;
        for (int64_t n = 0; n < N; ++n) y[n] = 0.0;
        if (s) for (int64_t n = 0; n < N; ++n) s[n] = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            double w = Wm[i * K + k];
            if (skip_zero && w == 0.0) continue;
            const double *x = X + k * N;
            for (int64_t n = 0; n < N; ++n) y[n] += w * x[n];
            if (s) for (int64_t n = 0; n < N; ++n) s[n] += fabs(w * x[n]);
        }
    }
    return 0;
}

int32_t bcr_oracle_threads(void)
{
#ifdef _OPENMP
    return (int32_t)omp_get_max_threads();
#else
    return 1;
#endif
}
