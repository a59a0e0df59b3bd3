/*
 * CPU oracle for the matrix chain D = A (B C)  --  TEST INFRASTRUCTURE, not part of the product.
 *
 * Only the test-suite, the smoke check and the bench's cpu_baseline leg may call this file.
 * It shares no code with the GPU path or with the inspector.
 *
 * What it computes is the plain, unfused definition (paper Section 1, Eq. 1, and the
 * two-operation decomposition D1 = B C, D = A D1 stated right after it; the loop nests are the
 * un-tiled bodies of the GeMM-SpMM and SpMM-SpMM listings of Section 3.2):
 *
 *   dense B :  D1[i][c] = sum_{k = 0 .. bCol-1, ascending}      B[i][k]   * C[k][c]
 *   CSR   B :  D1[i][c] = sum_{q = Bp[i] .. Bp[i+1]-1, storage} Bx[q]     * C[Bi[q]][c]
 *   second  :  D [j][c] = sum_{q = Ap[j] .. Ap[j+1]-1, storage} Ax[q]     * D1[Ai[q]][c]
 *
 * and, for the variant with the transpose of C that Section 3.2 mentions (Ct is cCol x bCol),
 *
 *   dense B :  D1[i][c] = sum_{k = 0 .. bCol-1, ascending}      B[i][k]   * Ct[c][k]
 *
 * Everything is scalar fp64 with a separate multiply and add (compile with -ffp-contract=off),
 * each output element accumulated in one fixed order.  Single-precision problems are promoted
 * to fp64 by the caller (exactly) and D1 is kept in fp64.  Outputs are overwritten (the
 * listings' "+=" assumes zeroed outputs).  Explicit zeros, duplicate and unsorted column
 * indices are legal: entries are summed in storage order.
 *
 * The "_par" entry points run the same loops with the output rows divided among OpenMP
 * threads; every output element keeps its own summation order, so results are bit-identical
 * to the serial ones.
 *
 * All matrices are row-major and contiguous.  `rows` (may be NULL) restricts the computation to
 * a list of output rows; other rows of the output are left untouched.
 */
#include <stddef.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* D1[i][:] = B[i][:] * C for one row i.  B is n x bcol, C is bcol x ccol, D1 is n x ccol. */
static void gemm_row(int64_t i, int64_t bcol, int64_t ccol,
                     const double *B, const double *C, double *D1)
{
    for (int64_t c = 0; c < ccol; ++c) {
        double acc = 0.0;
        for (int64_t k = 0; k < bcol; ++k) {
            double prod = B[i * bcol + k] * C[k * ccol + c];
            acc = acc + prod;
        }
        D1[i * ccol + c] = acc;
    }
}

/* D1[i][:] = B[i][:] * Ct^T for one row i.  B is n x bcol, Ct is ccol x bcol, D1 is n x ccol. */
static void gemm_ct_row(int64_t i, int64_t bcol, int64_t ccol,
                        const double *B, const double *Ct, double *D1)
{
    for (int64_t c = 0; c < ccol; ++c) {
        double acc = 0.0;
        for (int64_t k = 0; k < bcol; ++k) {
            double prod = B[i * bcol + k] * Ct[c * bcol + k];
            acc = acc + prod;
        }
        D1[i * ccol + c] = acc;
    }
}

/* Y[j][:] = sum over stored entries of row j of  vals * X[col][:].  X and Y have ccol columns. */
static void spmm_row(int64_t j, const int32_t *rowptr, const int32_t *colidx,
                     const double *vals, int64_t ccol, const double *X, double *Y)
{
    for (int64_t c = 0; c < ccol; ++c) {
        double acc = 0.0;
        for (int64_t q = rowptr[j]; q < rowptr[j + 1]; ++q) {
            double prod = vals[q] * X[(int64_t)colidx[q] * ccol + c];
            acc = acc + prod;
        }
        Y[j * ccol + c] = acc;
    }
}

void orc_gemm(int64_t n, int64_t bcol, int64_t ccol, const double *B, const double *C,
              double *D1, const int64_t *rows, int64_t n_rows_listed)
{
    if (rows) {
        for (int64_t r = 0; r < n_rows_listed; ++r) gemm_row(rows[r], bcol, ccol, B, C, D1);
    } else {
        for (int64_t i = 0; i < n; ++i) gemm_row(i, bcol, ccol, B, C, D1);
    }
}

void orc_gemm_ct(int64_t n, int64_t bcol, int64_t ccol, const double *B, const double *Ct,
                 double *D1, const int64_t *rows, int64_t n_rows_listed)
{
    if (rows) {
        for (int64_t r = 0; r < n_rows_listed; ++r) gemm_ct_row(rows[r], bcol, ccol, B, Ct, D1);
    } else {
        for (int64_t i = 0; i < n; ++i) gemm_ct_row(i, bcol, ccol, B, Ct, D1);
    }
}

void orc_spmm(int64_t n, const int32_t *rowptr, const int32_t *colidx, const double *vals,
              int64_t ccol, const double *X, double *Y, const int64_t *rows,
              int64_t n_rows_listed)
{
    if (rows) {
        for (int64_t r = 0; r < n_rows_listed; ++r)
            spmm_row(rows[r], rowptr, colidx, vals, ccol, X, Y);
    } else {
        for (int64_t j = 0; j < n; ++j) spmm_row(j, rowptr, colidx, vals, ccol, X, Y);
    }
}

void orc_gemm_par(int64_t n, int64_t bcol, int64_t ccol, const double *B, const double *C,
                  double *D1)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) gemm_row(i, bcol, ccol, B, C, D1);
}

void orc_spmm_par(int64_t n, const int32_t *rowptr, const int32_t *colidx, const double *vals,
                  int64_t ccol, const double *X, double *Y)
{
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t j = 0; j < n; ++j) spmm_row(j, rowptr, colidx, vals, ccol, X, Y);
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
