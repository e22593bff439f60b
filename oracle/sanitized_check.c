/*
 * Driver for a sanitizer build of the CPU oracle.  TEST INFRASTRUCTURE ONLY (like everything in this
 * directory): tests/test_oracle_sanitized.py compiles it together with spgemm_oracle.c under
 * -fsanitize=address,undefined and runs it on CSR matrices it has written to a file.
 *
 * File layout (little endian): int64 rows_a, cols_a, nnz_a, rows_b, cols_b, nnz_b; then a_row_ptr
 * int64[rows_a+1], a_col int32[nnz_a], a_val double[nnz_a], b_row_ptr int64[rows_b+1], b_col int32[nnz_b],
 * b_val double[nnz_b].  Prints: products, nnz(C), sum of column indices, sum of values, sum of magnitudes.
 * The checks themselves are the sanitizers' (out-of-bounds and use-after-free accesses, signed overflow,
 * misaligned or null pointers); the test compares the printed figures with the ordinary build's.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int64_t oracle_spgemm_row_nnz(int64_t n_cols_b, const int64_t *a_row_ptr, const int32_t *a_col,
                              const int64_t *b_row_ptr, const int32_t *b_col, int64_t row_begin, int64_t row_end,
                              int64_t *c_row_nnz);
int64_t oracle_spgemm_rows(int64_t n_cols_b, const int64_t *a_row_ptr, const int32_t *a_col, const double *a_val,
                           const int64_t *b_row_ptr, const int32_t *b_col, const double *b_val, int64_t row_begin,
                           int64_t row_end, int32_t *c_col, double *c_val, double *c_abs);

static void *read_array(FILE *f, size_t count, size_t size)
{
    void *p = malloc(count * size + 1);          /* exact size (+1 so that an empty array is not NULL) */
    if (!p || fread(p, size, count, f) != count) { fprintf(stderr, "short read\n"); exit(2); }
    return p;
}

int main(int argc, char **argv)
{
    if (argc != 2) { fprintf(stderr, "usage: %s file\n", argv[0]); return 2; }
    FILE *f = fopen(argv[1], "rb");
    if (!f) { perror("open"); return 2; }
    int64_t h[6];
    if (fread(h, sizeof(int64_t), 6, f) != 6) { fprintf(stderr, "short header\n"); return 2; }
    int64_t *a_rp = read_array(f, (size_t)h[0] + 1, sizeof(int64_t));
    int32_t *a_col = read_array(f, (size_t)h[2], sizeof(int32_t));
    double *a_val = read_array(f, (size_t)h[2], sizeof(double));
    int64_t *b_rp = read_array(f, (size_t)h[3] + 1, sizeof(int64_t));
    int32_t *b_col = read_array(f, (size_t)h[5], sizeof(int32_t));
    double *b_val = read_array(f, (size_t)h[5], sizeof(double));
    fclose(f);
    int64_t *counts = malloc(sizeof(int64_t) * (size_t)(h[0] + 1));
    /* in two halves, as the streamed comparisons call it: row ranges that do not start at zero */
    int64_t half = h[0] / 2, products = 0, total = 0;
    products += oracle_spgemm_row_nnz(h[4], a_rp, a_col, b_rp, b_col, 0, half, counts);
    products += oracle_spgemm_row_nnz(h[4], a_rp, a_col, b_rp, b_col, half, h[0], counts + half);
    for (int64_t i = 0; i < h[0]; ++i) total += counts[i];
    int32_t *c_col = malloc(sizeof(int32_t) * (size_t)total + 1);
    double *c_val = malloc(sizeof(double) * (size_t)total + 1), *c_abs = malloc(sizeof(double) * (size_t)total + 1);
    int64_t first = 0;
    for (int64_t i = 0; i < half; ++i) first += counts[i];
    int64_t wrote = oracle_spgemm_rows(h[4], a_rp, a_col, a_val, b_rp, b_col, b_val, 0, half, c_col, c_val, c_abs);
    wrote += oracle_spgemm_rows(h[4], a_rp, a_col, a_val, b_rp, b_col, b_val, half, h[0], c_col + first, c_val + first,
                                c_abs + first);
    int64_t col_sum = 0;
    double val_sum = 0.0, abs_sum = 0.0;
    for (int64_t e = 0; e < total; ++e) { col_sum += c_col[e]; val_sum += c_val[e]; abs_sum += c_abs[e]; }
    printf("%lld %lld %lld %.17g %.17g\n", (long long)products, (long long)wrote, (long long)col_sum, val_sum, abs_sum);
    free(a_rp); free(a_col); free(a_val); free(b_rp); free(b_col); free(b_val);
    free(counts); free(c_col); free(c_val); free(c_abs);
    return wrote == total ? 0 : 1;
}
