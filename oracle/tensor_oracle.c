/*
 * CPU oracles for the two third-order members of the paper's sparse-dense
 * hybrid algebra, MTTKRP and TTM.  TEST INFRASTRUCTURE ONLY: nothing in the
 * product path may call this; only the test-suite, the smoke check and the
 * CPU-baseline leg of the benchmark do.  It shares no code with the HIP
 * kernels.
 *
 * Both are the plain definitions of the paper's Section 2.1 (the first and
 * the second form listed under Eq. 1), written out over the stored entries of
 * a third-order sparse tensor A:
 *     MTTKRP   Y[i,j]   = sum_{k,l} A[i,k,l] * X1[k,j] * X2[l,j]
 *     TTM      Y[i,j,l] = sum_k     A[i,j,k] * X1[k,l]
 * A is stored as compressed sparse fibers, in the index order of the formula:
 * the first index is dense (slice i owns fibers fptr[i] .. fptr[i+1]-1), a
 * fiber f carries its second index fidx[f] and owns entries eptr[f] ..
 * eptr[f+1]-1, an entry p carries its third index eidx[p] and its value
 * vals[p].  Dense operands are row-major.  TTM's result is kept on A's stored
 * fibers, one dense row of L numbers per fiber (Yf[f,:] = Y[i, fidx[f], :];
 * rows of Y without a stored fiber are zero and are not materialised).
 * Double precision throughout: every term is the exact product of fp32
 * numbers rounded once (three factors) or not at all (two factors).
 *
 * Next to the result each function returns BND, the same sum over absolute
 * values, the scale against which fp32 results are judged
 * (|Y - ref| <= 1e-5 * BND).
 *
 * Parity pins (tests, CPU only): numpy einsum over the densified tensor,
 * a brute-force loop over coordinate triples, exact integer-valued inputs, a
 * hand-worked example, one-fiber-per-slice tensors (MTTKRP turns into an
 * SDDMM-like row product, TTM into SpMM), all-ones factor matrices (MTTKRP
 * = the SpMM of the tensor flattened over its second index), linearity in
 * the values, and permutation of the slices.
 */
#include <stdint.h>
#include <stddef.h>
#include <math.h>

/*
 * Y and BND (may be NULL) are I x J row-major.  X1 is K x J, X2 is L x J.
 * nthreads > 1 splits the slices statically over OpenMP threads.
 * Returns 0, or 1 on an argument that makes no sense.
 */
int oracle_mttkrp_csf(int64_t I, int64_t K, int64_t L, int64_t J,
                      const int32_t *fptr, const int32_t *fidx,
                      const int32_t *eptr, const int32_t *eidx, const float *vals,
                      const float *X1, const float *X2,
                      double *Y, double *BND, int nthreads)
{
    if (I < 0 || K < 0 || L < 0 || J < 0) return 1;
    if (I > 0 && (!fptr || !Y)) return 1;
    if (nthreads < 1) nthreads = 1;
    (void)K;
    (void)L;
#pragma omp parallel for schedule(static) num_threads(nthreads)
    for (int64_t i = 0; i < I; ++i) {
        double *y = Y + i * J;
        double *b = BND ? BND + i * J : NULL;
        for (int64_t j = 0; j < J; ++j) {
            y[j] = 0.0;
            if (b) b[j] = 0.0;
        }
        for (int64_t f = fptr[i]; f < fptr[i + 1]; ++f) {
            const float *x1 = X1 + (int64_t)fidx[f] * J;
            for (int64_t p = eptr[f]; p < eptr[f + 1]; ++p) {
                const float *x2 = X2 + (int64_t)eidx[p] * J;
                const double a = (double)vals[p];
                for (int64_t j = 0; j < J; ++j) {
                    const double u = (double)x1[j], v = (double)x2[j];
                    y[j] += a * u * v;
                    if (b) b[j] += fabs(a) * fabs(u) * fabs(v);
                }
            }
        }
    }
    return 0;
}

/*
 * Yf and BND (may be NULL) are F x L row-major, F = number of stored fibers;
 * X1 is K x L.  The slice a fiber belongs to does not enter the sum, so the
 * fiber-level arrays are all this needs.
 */
int oracle_ttm_csf(int64_t F, int64_t K, int64_t L,
                   const int32_t *eptr, const int32_t *eidx, const float *vals,
                   const float *X1, double *Yf, double *BND, int nthreads)
{
    if (F < 0 || K < 0 || L < 0) return 1;
    if (F > 0 && (!eptr || !Yf)) return 1;
    if (nthreads < 1) nthreads = 1;
    (void)K;
#pragma omp parallel for schedule(static) num_threads(nthreads)
    for (int64_t f = 0; f < F; ++f) {
        double *y = Yf + f * L;
        double *b = BND ? BND + f * L : NULL;
        for (int64_t l = 0; l < L; ++l) {
            y[l] = 0.0;
            if (b) b[l] = 0.0;
        }
        for (int64_t p = eptr[f]; p < eptr[f + 1]; ++p) {
            const float *x1 = X1 + (int64_t)eidx[p] * L;
            const double a = (double)vals[p];
            for (int64_t l = 0; l < L; ++l) {
                y[l] += a * (double)x1[l];
                if (b) b[l] += fabs(a) * fabs((double)x1[l]);
            }
        }
    }
    return 0;
}
