/* Driver of the host-sanitizer test (tests/test_oracle_sanitized.py): linked with oracle/ftc_oracle.c under
 * -fsanitize=address,undefined, it runs every routine of the oracle once on the case stored in argv[1] and
 * writes the results to argv[2].  Any out-of-bounds access, use of a freed block, leak, signed overflow or
 * misaligned access inside the oracle ends the process with a report and a non-zero status.
 *
 * Case file (little endian): int32 n, nnz, D, d_out, blk_h, blk_w; int32 row_ptr[n + 1]; int32 col_idx[nnz];
 * double X[n * D]; double W[D * d_out]; double beta.  Every array is copied into a heap block of exactly its
 * size, so that the sanitizer's red zones sit directly behind the last element. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_set_threads(int t);
void oracle_gcn_norm(int32_t n, const int32_t *row_ptr, const int32_t *col_idx, double *vals, double *dinv);
void oracle_build_windows(int32_t n, const int32_t *row_ptr, const int32_t *col_idx, int32_t blk_h, int32_t blk_w,
                          int32_t *edge_to_row, int32_t *edge_to_col, int32_t *block_partition,
                          int32_t *win_col_ptr, int32_t *win_cols, int64_t *summary);
void oracle_spmm(int32_t n, const int32_t *row_ptr, const int32_t *col_idx, const double *vals, const double *X,
                 int64_t ldx, int32_t D, double *out, double *abs_out, int64_t ldo);
void oracle_sddmm(int32_t n, const int32_t *row_ptr, const int32_t *col_idx, const double *X, const double *Y,
                  int64_t ld, int32_t D, const double *rs, const double *cs, double alpha, double *s_out,
                  double *abs_out);
void oracle_row_rnorm(int32_t n, const double *H, int64_t ld, int32_t D, double *rinv);
void oracle_edge_softmax(int32_t n, const int32_t *row_ptr, const double *s, double *p);
void oracle_gemm(int32_t n, int32_t d_in, int32_t d_out, const double *X, int64_t ldx, const double *W, int64_t ldw,
                 double *Z, double *abs_out, int64_t ldz);
void oracle_gcn_layer(int32_t n, const int32_t *row_ptr, const int32_t *col_idx, const double *vals, const double *X,
                      int64_t ldx, int32_t d_in, const double *W, int32_t d_out, int32_t relu, double *Z,
                      double *Zabs, double *out, double *abs_out);
void oracle_agnn_layer(int32_t n, const int32_t *row_ptr, const int32_t *col_idx, const double *H, int64_t ld,
                       int32_t D, double beta, double *rinv, double *p_out, double *out, double *abs_out);
int64_t oracle_tile_capacity(int64_t block_counter, int32_t blk_h, int32_t blk_w);

static void *take(FILE *f, size_t count, size_t size)
{
    /* a block of exactly count * size bytes (one byte for an empty array, never read) */
    void *p = malloc(count * size ? count * size : 1);
    if (!p || fread(p, size, count, f) != count) {
        fprintf(stderr, "short case file\n");
        exit(3);
    }
    return p;
}

static void *blank(size_t count, size_t size)
{
    void *p = malloc(count * size ? count * size : 1);
    if (!p) exit(3);
    memset(p, 0, count * size);
    return p;
}

static void put(FILE *f, const void *p, size_t count, size_t size)
{
    if (fwrite(p, size, count, f) != count) exit(4);
}

int main(int argc, char **argv)
{
    if (argc != 3) return 2;
    FILE *in = fopen(argv[1], "rb"), *out = fopen(argv[2], "wb");
    if (!in || !out) return 2;
    int32_t h[6];
    if (fread(h, sizeof(int32_t), 6, in) != 6) return 3;
    const int32_t n = h[0], nnz = h[1], D = h[2], d_out = h[3], blk_h = h[4], blk_w = h[5];
    int32_t *row_ptr = take(in, (size_t)n + 1, 4), *col_idx = take(in, (size_t)nnz, 4);
    double *X = take(in, (size_t)n * D, 8), *W = take(in, (size_t)D * d_out, 8), *beta = take(in, 1, 8);
    fclose(in);
    oracle_set_threads(2);

    /* normalisation */
    double *vals = blank(nnz, 8), *dinv = blank(n, 8);
    oracle_gcn_norm(n, row_ptr, col_idx, vals, dinv);
    put(out, vals, nnz, 8);
    put(out, dinv, n, 8);

    /* window index */
    const int32_t n_win = (n + blk_h - 1) / blk_h;
    int32_t *e2r = blank(nnz, 4), *e2c = blank(nnz, 4), *bp = blank(n_win, 4), *wcp = blank((size_t)n_win + 1, 4);
    int32_t *wc = blank(nnz, 4);
    int64_t summary[2] = {0, 0};
    oracle_build_windows(n, row_ptr, col_idx, blk_h, blk_w, e2r, e2c, bp, wcp, wc, summary);
    put(out, e2r, nnz, 4);
    put(out, e2c, nnz, 4);
    put(out, bp, n_win, 4);
    put(out, wcp, (size_t)n_win + 1, 4);
    put(out, wc, nnz, 4);
    put(out, summary, 2, 8);
    const int64_t cap = oracle_tile_capacity(summary[1], blk_h, blk_w);
    put(out, &cap, 1, 8);

    /* kernels */
    double *y = blank((size_t)n * D, 8), *ya = blank((size_t)n * D, 8);
    oracle_spmm(n, row_ptr, col_idx, vals, X, D, D, y, ya, D);
    put(out, y, (size_t)n * D, 8);
    put(out, ya, (size_t)n * D, 8);
    double *rinv = blank(n, 8);
    oracle_row_rnorm(n, X, D, D, rinv);
    put(out, rinv, n, 8);
    double *s = blank(nnz, 8), *sa = blank(nnz, 8);
    oracle_sddmm(n, row_ptr, col_idx, X, X, D, D, rinv, rinv, *beta, s, sa);
    put(out, s, nnz, 8);
    put(out, sa, nnz, 8);
    double *p = blank(nnz, 8);
    oracle_edge_softmax(n, row_ptr, s, p);
    put(out, p, nnz, 8);
    double *Z = blank((size_t)n * d_out, 8), *Za = blank((size_t)n * d_out, 8);
    oracle_gemm(n, D, d_out, X, D, W, d_out, Z, Za, d_out);
    put(out, Z, (size_t)n * d_out, 8);
    put(out, Za, (size_t)n * d_out, 8);

    /* layers */
    double *g = blank((size_t)n * d_out, 8), *ga = blank((size_t)n * d_out, 8);
    oracle_gcn_layer(n, row_ptr, col_idx, vals, X, D, D, W, d_out, 1, Z, Za, g, ga);
    put(out, g, (size_t)n * d_out, 8);
    put(out, ga, (size_t)n * d_out, 8);
    oracle_agnn_layer(n, row_ptr, col_idx, X, D, D, *beta, rinv, p, y, ya);
    put(out, y, (size_t)n * D, 8);
    put(out, ya, (size_t)n * D, 8);
    put(out, p, nnz, 8);
    fclose(out);

    void *all[] = {row_ptr, col_idx, X, W, beta, vals, dinv, e2r, e2c, bp, wcp, wc, y, ya, rinv, s, sa, p, Z, Za, g, ga};
    for (size_t i = 0; i < sizeof(all) / sizeof(all[0]); ++i) free(all[i]);
    return 0;
}
