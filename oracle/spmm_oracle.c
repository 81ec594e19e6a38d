/*
 * CPU oracle for CSR SpMM.  TEST INFRASTRUCTURE ONLY: nothing in the product
 * path may call this; only the test-suite, the smoke check and the CPU-baseline
 * leg of the benchmark do.  It shares no code with the HIP kernels.
 *
 * What it computes is the plain definition of SpMM from the paper's
 * Section 2.1 (the fourth of the sparse-dense hybrid forms listed under
 * Eq. 1):   Y[i,k] = sum_j A[i,j] * X[j,k]
 * with A sparse in CSR (dense row level, compressed column level, Section 6)
 * and X, Y dense row-major.  Every point of the paper's design space
 * (Section 3.3) produces this same result; the points differ only in who
 * adds what, so the oracle is the definition written out row by row, in
 * double precision: products of two fp32 numbers are exact in fp64, and the
 * fp64 running sum is far more accurate than any fp32 order of summation.
 *
 * Next to the result it returns BND[i,k] = sum_j |A[i,j]| * |X[j,k]|, the
 * scale against which fp32 results are judged
 * (|C - C_ref| <= 1e-5 * BND elementwise).
 *
 * Parity pins (tests, CPU only): brute-force dense triple loop on tiny
 * matrices, exact integer-valued inputs, empty A => 0, identity A => B,
 * diagonal scaling, linearity in A, scipy.sparse csr @ dense in float64.
 */
#include <stdint.h>
#include <stddef.h>
#include <math.h>

/* One output row.  Stored entries are taken as they come: no assumption that
 * column indices inside a row are sorted or distinct (duplicates just add),
 * explicit zeros are ordinary entries. */
static void oracle_row(int64_t i, int64_t N,
                       const int32_t *rowptr, const int32_t *colidx,
                       const float *vals, const float *B,
                       double *c_row, double *bnd_row)
{
    for (int64_t k = 0; k < N; ++k) {
        c_row[k] = 0.0;
        if (bnd_row) bnd_row[k] = 0.0;
    }
    for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
        const double a = (double)vals[p];
        const float *b_row = B + (int64_t)colidx[p] * N;
        for (int64_t k = 0; k < N; ++k) {
            const double b = (double)b_row[k];
            c_row[k] += a * b;
            if (bnd_row) bnd_row[k] += fabs(a) * fabs(b);
        }
    }
}

/*
 * Full result.  C_ref and BND are M x N row-major double (BND may be NULL).
 * nthreads > 1 splits the rows statically and evenly over that many OpenMP
 * threads (rows are independent); the per-row arithmetic is unchanged.
 * Returns 0, or 1 on an argument that makes no sense.
 */
int oracle_spmm_csr(int64_t M, int64_t K, int64_t N,
                    const int32_t *rowptr, const int32_t *colidx,
                    const float *vals, const float *B,
                    double *C_ref, double *BND, int nthreads)
{
    if (M < 0 || K < 0 || N < 0) return 1;
    if (M > 0 && !rowptr) return 1;
    if (nthreads < 1) nthreads = 1;
    (void)K;
#pragma omp parallel for schedule(static) num_threads(nthreads)
    for (int64_t i = 0; i < M; ++i)
        oracle_row(i, N, rowptr, colidx, vals, B,
                   C_ref + i * N, BND ? BND + i * N : NULL);
    return 0;
}

/*
 * Selected rows only: output row t holds row rows[t] of the full result.
 * Used to check full-size GPU results on sampled outputs.
 */
int oracle_spmm_csr_rows(int64_t M, int64_t K, int64_t N,
                         const int32_t *rowptr, const int32_t *colidx,
                         const float *vals, const float *B,
                         const int64_t *rows, int64_t nrows,
                         double *C_ref, double *BND)
{
    if (M < 0 || K < 0 || N < 0 || nrows < 0) return 1;
    (void)K;
    for (int64_t t = 0; t < nrows; ++t) {
        if (rows[t] < 0 || rows[t] >= M) return 1;
        oracle_row(rows[t], N, rowptr, colidx, vals, B,
                   C_ref + t * N, BND ? BND + t * N : NULL);
    }
    return 0;
}
