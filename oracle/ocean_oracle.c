/*
 * CPU oracle for C = A*B on CSR inputs.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the checker the GPU library is compared against.  It is never
 * linked into, loaded by or called from the product path; it shares no code,
 * header, table or helper with the HIP sources.
 *
 * What it computes is the plain definition of the sparse product (paper,
 * Section 2.1): for every row i of A the set of output columns is
 *     J_i = union over stored A_ik of { j : B_kj stored },
 * and C_ij = sum_k A_ik * B_kj over stored pairs.  An output entry exists for
 * every structurally reachable (i, j): numerical cancellation and explicitly
 * stored zeros do not remove entries.  Rows come out with ascending column
 * ids (Section 2.3: CSR-compliant output).  The estimator, the binning and the
 * choice of accumulator in the paper are performance devices that must not
 * change this result (Section 3.2, overflow handling), so none of them
 * appears here.
 *
 * Method: Gustavson's row-by-row algorithm (Section 2.1) with a dense
 * accumulator of length n per thread (Section 2.2, "dense accumulator"):
 * acc[j] += a*b, absacc[j] += |a*b|, a flag marks first touches, the touched
 * column list is sorted, the row is emitted and only touched slots are
 * cleared.  All arithmetic is IEEE double.  absacc is the per-entry scale
 * sum_k |A_ik*B_kj| against which value tolerances are stated.
 *
 * Rows are independent, so a row range [r0, r1) can be produced on its own;
 * OpenMP spreads rows over threads and nothing else is reordered.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int g_threads = 0; /* 0 = OpenMP default */

void oracle_set_threads(int t) { g_threads = t; }

int oracle_get_threads(void)
{
#ifdef _OPENMP
    return g_threads > 0 ? g_threads : omp_get_max_threads();
#else
    return 1;
#endif
}

static int nthreads(void) { return oracle_get_threads(); }

/* Intermediate products per row of A: prod[i] = sum over stored A_ik of the
 * number of stored entries in row k of B (Section 3.2: an upper bound of the
 * row's output size).  Returns the total P. */
int64_t oracle_row_products(int64_t m, const int64_t *a_rp, const int32_t *a_col,
                            const int64_t *b_rp, int64_t *prod)
{
    int64_t total = 0;
    for (int64_t i = 0; i < m; ++i) {
        int64_t p = 0;
        for (int64_t e = a_rp[i]; e < a_rp[i + 1]; ++e) {
            int64_t k = a_col[e];
            p += b_rp[k + 1] - b_rp[k];
        }
        prod[i] = p;
        total += p;
    }
    return total;
}

static int cmp_i32(const void *x, const void *y)
{
    int32_t a = *(const int32_t *)x, b = *(const int32_t *)y;
    return (a > b) - (a < b);
}

/* Exact number of distinct output columns of rows [r0, r1): what a symbolic
 * pass returns (Section 2.3).  nnz has r1-r0 entries. */
void oracle_count_rows(int64_t r0, int64_t r1, const int64_t *a_rp, const int32_t *a_col,
                       const int64_t *b_rp, const int32_t *b_col, int64_t n, int64_t *nnz)
{
#pragma omp parallel num_threads(nthreads())
    {
        uint8_t *flag = (uint8_t *)calloc((size_t)(n > 0 ? n : 1), 1);
        int32_t *list = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
#pragma omp for schedule(dynamic, 64)
        for (int64_t i = r0; i < r1; ++i) {
            int64_t cnt = 0;
            for (int64_t e = a_rp[i]; e < a_rp[i + 1]; ++e) {
                int64_t k = a_col[e];
                for (int64_t p = b_rp[k]; p < b_rp[k + 1]; ++p) {
                    int32_t j = b_col[p];
                    if (!flag[j]) { flag[j] = 1; list[cnt++] = j; }
                }
            }
            for (int64_t t = 0; t < cnt; ++t) flag[list[t]] = 0;
            nnz[i - r0] = cnt;
        }
        free(flag);
        free(list);
    }
}

/* Rows [r0, r1) of C.  out_ptr has r1-r0+1 entries: offsets of each row
 * inside c_col / c_val / c_abs (relative to the start of the block), i.e. the
 * exclusive prefix sum of oracle_count_rows' result.  a_val and b_val are
 * double (float inputs are widened by the caller, which is exact). */
void oracle_multiply_rows(int64_t r0, int64_t r1, const int64_t *a_rp, const int32_t *a_col,
                          const double *a_val, const int64_t *b_rp, const int32_t *b_col,
                          const double *b_val, int64_t n, const int64_t *out_ptr,
                          int32_t *c_col, double *c_val, double *c_abs)
{
#pragma omp parallel num_threads(nthreads())
    {
        size_t nn = (size_t)(n > 0 ? n : 1);
        double *acc = (double *)calloc(nn, sizeof(double));
        double *absacc = (double *)calloc(nn, sizeof(double));
        uint8_t *flag = (uint8_t *)calloc(nn, 1);
        int32_t *list = (int32_t *)malloc(sizeof(int32_t) * nn);
#pragma omp for schedule(dynamic, 64)
        for (int64_t i = r0; i < r1; ++i) {
            int64_t cnt = 0;
            for (int64_t e = a_rp[i]; e < a_rp[i + 1]; ++e) {
                int64_t k = a_col[e];
                double a = a_val[e];
                for (int64_t p = b_rp[k]; p < b_rp[k + 1]; ++p) {
                    int32_t j = b_col[p];
                    double t = a * b_val[p];
                    if (!flag[j]) { flag[j] = 1; list[cnt++] = j; }
                    acc[j] += t;
                    absacc[j] += fabs(t);
                }
            }
            int64_t o = out_ptr[i - r0];
            if (cnt > n / 32) {
                /* dense-ish row: walking the flags in order yields ascending columns */
                int64_t w = 0;
                for (int64_t j = 0; j < n && w < cnt; ++j)
                    if (flag[j]) list[w++] = (int32_t)j;
            } else {
                qsort(list, (size_t)cnt, sizeof(int32_t), cmp_i32);
            }
            for (int64_t t = 0; t < cnt; ++t) {
                int32_t j = list[t];
                c_col[o + t] = j;
                c_val[o + t] = acc[j];
                c_abs[o + t] = absacc[j];
                acc[j] = 0.0;
                absacc[j] = 0.0;
                flag[j] = 0;
            }
        }
        free(acc);
        free(absacc);
        free(flag);
        free(list);
    }
}
