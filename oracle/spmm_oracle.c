/*
 * CPU ORACLE -- TEST INFRASTRUCTURE ONLY.  Not part of the product path: nothing under the
 * product package may include, link, load or call this file.  Only the tests, the smoke check
 * and the benchmark's cpu_baseline leg use it.  It shares no code, header, table or helper with
 * the HIP implementation.
 *
 * What it computes: the plain definition of sparse-times-dense matrix multiply,
 *     Y = A * X,  A is M x K sparse, X is K x N dense, Y is M x N dense
 * (paper Sec. 3.1, Fig. 2(a)/(b): three nested loops over M, N and the non-zeros of row m; Sec. 3.2:
 * row m with K_(m) stored entries costs K_(m)*N multiply-adds; Sec. 3.4: each output is the inner
 * product of a sparse row with a dense column).  All eight algorithms of the paper's space (Table 1)
 * reach exactly this result up to rounding order, so the oracle is the definition itself, written
 * as those three loops, accumulated in double precision:
 *
 *     C_ref[i][n] = sum_{p = rowptr[i]}^{rowptr[i+1]-1}  (double)vals[p] * (double)B[colind[p]*N + n]
 *     S_abs[i][n] = sum_p |vals[p]| * |B[colind[p]*N + n]|          (scale for the error bound)
 *
 * A is CSR (rowptr int32[m+1], colind int32[nnz], vals fp32[nnz]); B and the outputs are row-major
 * with leading dimension N.  Stored entries are taken in ascending p; columns need not be sorted and
 * repeated (i,j) entries add.  The product of two fp32 numbers is exact in fp64, and the fp64 sum of
 * len terms is off by at most about len * 2^-53 * S_abs.
 *
 * Rows are independent, so the OpenMP loop over rows does not change any result bit.
 */
#include <stdint.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static void one_row(int64_t i, int64_t N, const int32_t *rowptr, const int32_t *colind,
                    const float *vals, const float *B, double *c_row, double *s_row)
{
    for (int64_t n = 0; n < N; ++n) {                       /* N-loop */
        double acc = 0.0, sabs = 0.0;
        for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {   /* K-loop over stored entries */
            double a = (double)vals[p];
            double b = (double)B[(int64_t)colind[p] * N + n];
            acc += a * b;
            sabs += fabs(a) * fabs(b);
        }
        c_row[n] = acc;
        if (s_row) s_row[n] = sabs;
    }
}

/* Full product.  c_ref, s_abs: m x N doubles (s_abs may be NULL). */
void oracle_spmm(int64_t m, int64_t N, const int32_t *rowptr, const int32_t *colind,
                 const float *vals, const float *B, double *c_ref, double *s_abs)
{
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < m; ++i)                          /* M-loop */
        one_row(i, N, rowptr, colind, vals, B, c_ref + i * N, s_abs ? s_abs + i * N : 0);
}

/* Same arithmetic for a chosen subset of rows: output row t holds row rows[t] of the product. */
void oracle_spmm_rows(int64_t nrows, const int64_t *rows, int64_t N, const int32_t *rowptr,
                      const int32_t *colind, const float *vals, const float *B,
                      double *c_ref, double *s_abs)
{
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t t = 0; t < nrows; ++t)
        one_row(rows[t], N, rowptr, colind, vals, B, c_ref + t * N, s_abs ? s_abs + t * N : 0);
}

/*
 * Product with the transposed matrix, straight from the definition (A^T)[j][i] = A[i][j]:
 *     D[j][n] = sum over stored entries (i, j) of A   (double)vals[p] * (double)G[i*N + n]
 * This is the gradient of  <G, A*X>  with respect to X (the backward pass of the aggregation step of
 * a graph-convolution layer, the application of Sec. 6's GCN experiment).  The loops walk A in its
 * own CSR order and scatter into row colind[p] of the output, so no transposed structure is built;
 * serial, because different rows of A add into the same output row.  d_ref, s_abs: k x N doubles,
 * overwritten (s_abs may be NULL).
 */
void oracle_spmm_transposed(int64_t m, int64_t k, int64_t N, const int32_t *rowptr,
                            const int32_t *colind, const float *vals, const float *G,
                            double *d_ref, double *s_abs)
{
    for (int64_t t = 0; t < k * N; ++t) {
        d_ref[t] = 0.0;
        if (s_abs) s_abs[t] = 0.0;
    }
    for (int64_t i = 0; i < m; ++i)
        for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
            double a = (double)vals[p];
            int64_t j = colind[p];
            for (int64_t n = 0; n < N; ++n) {
                double g = (double)G[i * N + n];
                d_ref[j * N + n] += a * g;
                if (s_abs) s_abs[j * N + n] += fabs(a) * fabs(g);
            }
        }
}
