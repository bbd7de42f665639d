/*
 * CPU oracle for CSR SPMM, SDDMM and FusedMM.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, FP64-accumulating implementation of the three operations,
 * written out from their definitions (paper eq. (1)-(3)) with the loop
 * structure of the paper's row algorithms (Algorithms 1-3: one thread per row,
 * a loop over the row's stored entries, an inner loop over the dense width).
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call
 * it; the product path never does.  It shares no code with the HIP kernels.
 *
 * Storage (paper, "Matrix Storage Layout"): dense matrices row-major; the
 * sparse matrix in CSR with 0-based int32 rowptr (M+1 entries, rowptr[M] =
 * nnz), int32 colidx and FP32 vals in row-major order of the stored entries.
 *
 * Readings taken where the paper is silent or inconsistent:
 *  - SDDMM masks with an all-ones pattern in eq. (1); here every stored entry
 *    is additionally scaled by vals[j] (vals == NULL gives the paper's form).
 *    The scale is applied to the finished dot product.
 *  - Algorithm 3's second loop reads B[k,l]; eq. (3) and the text make clear
 *    it must be the second dense matrix (here C, K x N).
 *  - The "Initialize C[i,:] <- 0" first lines of Algorithms 1 and 3 touch an
 *    input and are ignored.
 *  - The dot length D (columns of A and B) and the output width N (columns of
 *    C and O) of FusedMM may differ; the paper has D == N.
 *  - Stored entries need not be sorted or unique: SPMM/FusedMM sum duplicates,
 *    SDDMM produces one value per stored entry.
 *
 * Every function also returns, per output entry, the sum of the absolute
 * values of the terms that were added up ("abs" arrays).  Parity tests accept
 * |gpu - oracle| <= 1e-5 * abs.
 *
 * `rows`/`nrows`: if rows != NULL only the listed rows are computed.  For SPMM
 * and FusedMM the outputs are then packed (nrows x N, in list order); for
 * SDDMM the outputs stay at their CSR positions and other positions are left
 * untouched.
 *
 * Parity pins (tests/test_oracle_*.py): dense brute force of eq. (1)-(3) in
 * numpy FP64, the worked CSR example of Fig. 1, identity / permutation /
 * all-ones special cases, scipy.sparse as a library cross-check, linearity and
 * reordering invariants, and planted-mistake checks.  The paper prints no
 * numerical outputs of its own kernels, so parity against the paper's runs
 * themselves is unpinned.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>

/* SPMM, eq. (2) / Algorithm 2:  O[i,:] = sum_j vals[j] * B[colidx[j],:]  over the entries j of row i. */
void oracle_spmm(int32_t M, int32_t K, int32_t N,
                 const int32_t *rowptr, const int32_t *colidx, const float *vals,
                 const float *B, double *O, double *absO,
                 const int32_t *rows, int32_t nrows) {
    (void)K;
    const int32_t R = rows ? nrows : M;
#pragma omp parallel for schedule(dynamic, 4)
    for (int32_t t = 0; t < R; ++t) {
        const int32_t i = rows ? rows[t] : t;
        double *acc = O + (size_t)t * N;
        double *aac = absO + (size_t)t * N;
        for (int32_t l = 0; l < N; ++l) { acc[l] = 0.0; aac[l] = 0.0; }
        for (int32_t j = rowptr[i]; j < rowptr[i + 1]; ++j) {
            const double s = (double)vals[j];
            const int32_t k = colidx[j];
            const float *Bk = B + (size_t)k * N;
            for (int32_t l = 0; l < N; ++l) {
                const double term = s * (double)Bk[l];
                acc[l] += term;
                aac[l] += fabs(term);
            }
        }
    }
}

/* SDDMM, eq. (1) / Algorithm 1:  P[j] = vals[j] * <A[i,:], B[colidx[j],:]>  for every entry j of row i. */
void oracle_sddmm(int32_t M, int32_t K, int32_t D,
                  const int32_t *rowptr, const int32_t *colidx, const float *vals,
                  const float *A, const float *B, double *P, double *absP,
                  const int32_t *rows, int32_t nrows) {
    (void)K;
    const int32_t R = rows ? nrows : M;
#pragma omp parallel for schedule(dynamic, 4)
    for (int32_t t = 0; t < R; ++t) {
        const int32_t i = rows ? rows[t] : t;
        const float *Ai = A + (size_t)i * D;
        for (int32_t j = rowptr[i]; j < rowptr[i + 1]; ++j) {
            const int32_t k = colidx[j];
            const float *Bk = B + (size_t)k * D;
            double dp = 0.0, adp = 0.0;
            for (int32_t l = 0; l < D; ++l) {
                const double term = (double)Ai[l] * (double)Bk[l];
                dp += term;
                adp += fabs(term);
            }
            const double s = vals ? (double)vals[j] : 1.0;
            P[j] = s * dp;
            absP[j] = fabs(s) * adp;
        }
    }
}

/*
 * FusedMM, eq. (3) / Algorithm 3:  O[i,:] = sum_j score_j * C[colidx[j],:],
 * score_j = vals[j] * <A[i,:], B[colidx[j],:]>, the scores of a row kept in a
 * per-row scratch array (FP64, never rounded to FP32) exactly as the
 * algorithm's `arow`.
 */
void oracle_fusedmm(int32_t M, int32_t K, int32_t D, int32_t N,
                    const int32_t *rowptr, const int32_t *colidx, const float *vals,
                    const float *A, const float *B, const float *C,
                    double *O, double *absO,
                    const int32_t *rows, int32_t nrows) {
    (void)K;
    const int32_t R = rows ? nrows : M;
#pragma omp parallel for schedule(dynamic, 4)
    for (int32_t t = 0; t < R; ++t) {
        const int32_t i = rows ? rows[t] : t;
        const int32_t nnzr = rowptr[i + 1] - rowptr[i];
        double *arow = (double *)malloc(sizeof(double) * (size_t)(nnzr > 0 ? nnzr : 1));
        double *aabs = (double *)malloc(sizeof(double) * (size_t)(nnzr > 0 ? nnzr : 1));
        const float *Ai = A + (size_t)i * D;
        /* first loop of Algorithm 3: the row's sampled scores */
        for (int32_t j = 0; j < nnzr; ++j) {
            const int32_t k = colidx[rowptr[i] + j];
            const float *Bk = B + (size_t)k * D;
            double dp = 0.0, adp = 0.0;
            for (int32_t l = 0; l < D; ++l) {
                const double term = (double)Ai[l] * (double)Bk[l];
                dp += term;
                adp += fabs(term);
            }
            const double s = vals ? (double)vals[rowptr[i] + j] : 1.0;
            arow[j] = s * dp;
            aabs[j] = fabs(s) * adp;
        }
        /* second loop: SAXPY of the rows of the second dense matrix */
        double *acc = O + (size_t)t * N;
        double *aac = absO + (size_t)t * N;
        for (int32_t l = 0; l < N; ++l) { acc[l] = 0.0; aac[l] = 0.0; }
        for (int32_t j = 0; j < nnzr; ++j) {
            const int32_t k = colidx[rowptr[i] + j];
            const float *Ck = C + (size_t)k * N;
            for (int32_t l = 0; l < N; ++l) {
                acc[l] += arow[j] * (double)Ck[l];
                aac[l] += aabs[j] * fabs((double)Ck[l]);
            }
        }
        free(arow);
        free(aabs);
    }
}

int oracle_num_threads(void) {
    int n = 1;
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    n = omp_get_max_threads();
#endif
    return n;
}
