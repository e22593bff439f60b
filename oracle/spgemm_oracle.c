/*
 * CPU oracle for C = A*B on CSR matrices with fp16 inputs.  TEST INFRASTRUCTURE ONLY:
 * tests, the smoke check and the benchmark's cpu_baseline leg call it; the product
 * (the HIP library) neither links nor calls anything in this directory.
 *
 * What it computes is the plain definition of the sparse product (paper Section 2.2):
 * an output position (i,j) exists when some k has both a_ik and b_kj stored, and its
 * value is the sum over those k of a_ik*b_kj.  Inputs are fp16 numbers, handed over
 * widened (exactly) to fp64 by the caller; the mixed-precision unit the paper targets
 * multiplies them exactly and accumulates in fp32 (Section 2.6), so the reference value
 * is the exact products (22 significant bits at most) summed in fp64.
 * Beside each value the oracle returns s_ij = sum_k |a_ik||b_kj|, the scale of the
 * acceptance bound |c - c_ref| <= 1e-5*s + 1e-7.
 *
 * The pattern is structural, like the paper's counting kernel (Section 4.2): a stored
 * entry counts even when its value is 0.0, and an entry whose terms cancel stays.
 *
 * Algorithm: row-wise Gustavson with a dense accumulator and a marker array.  No
 * blocking, no tiling, nothing shared with the GPU code.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

static int compare_int32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/*
 * Structural size of rows [row_begin,row_end) of C, and the number of intermediate
 * products (inner-loop trips) those rows need; 2*products is the FLOP count of the
 * benchmark metric.  c_row_nnz has row_end-row_begin entries.  Returns products, or -1
 * when memory runs out.
 */
int64_t oracle_spgemm_row_nnz(int64_t n_cols_b,
                              const int64_t *a_row_ptr, const int32_t *a_col,
                              const int64_t *b_row_ptr, const int32_t *b_col,
                              int64_t row_begin, int64_t row_end, int64_t *c_row_nnz)
{
    int64_t *mark = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n_cols_b > 0 ? n_cols_b : 1));
    if (!mark) return -1;
    for (int64_t j = 0; j < n_cols_b; ++j) mark[j] = -1;
    int64_t products = 0;
    for (int64_t i = row_begin; i < row_end; ++i) {
        int64_t count = 0;
        for (int64_t p = a_row_ptr[i]; p < a_row_ptr[i + 1]; ++p) {
            int64_t k = a_col[p];
            for (int64_t q = b_row_ptr[k]; q < b_row_ptr[k + 1]; ++q) {
                int64_t j = b_col[q];
                if (mark[j] != i) { mark[j] = i; ++count; }
                ++products;
            }
        }
        c_row_nnz[i - row_begin] = count;
    }
    free(mark);
    return products;
}

/*
 * Rows [row_begin,row_end) of C.  c_col / c_val / c_abs receive the rows back to back
 * (the caller sized them with oracle_spgemm_row_nnz), columns ascending inside a row.
 * Returns the number of entries written, or -1 when memory runs out.
 */
int64_t oracle_spgemm_rows(int64_t n_cols_b,
                           const int64_t *a_row_ptr, const int32_t *a_col, const double *a_val,
                           const int64_t *b_row_ptr, const int32_t *b_col, const double *b_val,
                           int64_t row_begin, int64_t row_end,
                           int32_t *c_col, double *c_val, double *c_abs)
{
    size_t n = (size_t)(n_cols_b > 0 ? n_cols_b : 1);
    int64_t *mark = (int64_t *)malloc(sizeof(int64_t) * n);
    double *acc = (double *)malloc(sizeof(double) * n);
    double *mag = (double *)malloc(sizeof(double) * n);
    int32_t *list = (int32_t *)malloc(sizeof(int32_t) * n);
    if (!mark || !acc || !mag || !list) { free(mark); free(acc); free(mag); free(list); return -1; }
    for (int64_t j = 0; j < n_cols_b; ++j) mark[j] = -1;
    int64_t out = 0;
    for (int64_t i = row_begin; i < row_end; ++i) {
        int64_t count = 0;
        for (int64_t p = a_row_ptr[i]; p < a_row_ptr[i + 1]; ++p) {
            int64_t k = a_col[p];
            double a = a_val[p];
            for (int64_t q = b_row_ptr[k]; q < b_row_ptr[k + 1]; ++q) {
                int64_t j = b_col[q];
                double prod = a * b_val[q];
                if (mark[j] != i) {
                    mark[j] = i;
                    list[count++] = (int32_t)j;
                    acc[j] = 0.0;
                    mag[j] = 0.0;
                }
                acc[j] += prod;
                mag[j] += fabs(prod);
            }
        }
        qsort(list, (size_t)count, sizeof(int32_t), compare_int32);
        for (int64_t t = 0; t < count; ++t) {
            int32_t j = list[t];
            c_col[out] = j;
            c_val[out] = acc[j];
            c_abs[out] = mag[j];
            ++out;
        }
    }
    free(mark); free(acc); free(mag); free(list);
    return out;
}
