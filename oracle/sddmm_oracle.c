/*
 * CPU oracle for CSR SDDMM.  TEST INFRASTRUCTURE ONLY: nothing in the product
 * path may call this; only the test-suite, the smoke check and the CPU-baseline
 * leg of the benchmark do.  It shares no code with the HIP kernels.
 *
 * What it computes is the plain definition of the sampled dense-dense matrix
 * product from the paper's Section 2.1 (the third of the sparse-dense hybrid
 * forms listed under Eq. 1):
 *     Y[i,k] = A[i,k] * sum_j X1[i,j] * X2[j,k]      for the stored (i,k) of A
 * with A sparse in CSR and the result stored on A's pattern, entry by entry:
 *     out[p] = vals[p] * sum_{j<J} X1[row(p), j] * X2T[colidx[p], j].
 * X1 is M x J row-major; the second dense operand is taken transposed,
 * X2T[k,j] = X2[j,k], K x J row-major, so that both factors of an entry are
 * contiguous rows (a layout choice of the interface, not of the paper).
 * The reduction runs along the dense dimension j (Section 2.1: "along two
 * dense dimensions" for this operator).  Double precision throughout:
 * products of two fp32 numbers are exact in fp64.
 *
 * Next to the result it returns BND[p] = |vals[p]| * sum_j |X1| * |X2T|, the
 * scale against which fp32 results are judged (|out - ref| <= 1e-5 * BND).
 *
 * Parity pins (tests, CPU only): sampling the dense product X1 * X2 computed
 * by a brute-force triple loop, exact integer-valued inputs, J = 1 (a plain
 * product of three numbers), all-ones operands (out = vals * J), X2T =
 * identity (out picks X1[i, k]), scaling of a row of X1, and
 * scipy.sparse A.multiply(X1 @ X2) in float64.
 */
#include <stdint.h>
#include <stddef.h>
#include <math.h>

/*
 * out and BND (may be NULL) have rowptr[M] entries, in the order of colidx.
 * nthreads > 1 splits the rows statically over OpenMP threads (entries are
 * independent).  Returns 0, or 1 on an argument that makes no sense.
 */
int oracle_sddmm_csr(int64_t M, int64_t K, int64_t J,
                     const int32_t *rowptr, const int32_t *colidx,
                     const float *vals, const float *X1, const float *X2T,
                     double *out, double *BND, int nthreads)
{
    if (M < 0 || K < 0 || J < 0) return 1;
    if (M > 0 && !rowptr) return 1;
    if (nthreads < 1) nthreads = 1;
    (void)K;
#pragma omp parallel for schedule(static) num_threads(nthreads)
    for (int64_t i = 0; i < M; ++i) {
        const float *x1 = X1 + i * J;
        for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
            const float *x2 = X2T + (int64_t)colidx[p] * J;
            double dot = 0.0, absdot = 0.0;
            for (int64_t j = 0; j < J; ++j) {
                const double u = (double)x1[j], v = (double)x2[j];
                dot += u * v;
                absdot += fabs(u) * fabs(v);
            }
            out[p] = (double)vals[p] * dot;
            if (BND) BND[p] = fabs((double)vals[p]) * absdot;
        }
    }
    return 0;
}
