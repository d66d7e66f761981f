/*
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, fp64 CPU oracle for the sparse neighbour
 * aggregation path of FTC-GNN (arXiv 2412.12218).  Nothing in the product library
 * includes, links or calls this file; it shares no code with the HIP kernels.
 *
 * Each function is the mathematical definition written as serial loops over the CSR
 * arrays (`nodePointer` = row_ptr, `edgeList` = col_idx; Section V.A, sparse graph
 * transformation).  There is no blocking, fusion or reordering.  The only library
 * primitives used are qsort/bsearch (window sort), sqrt and exp.
 *
 * Rows are independent in every routine, so an optional OpenMP `parallel for` over
 * rows (or windows) is the only concession to speed; it does not change any result
 * because no two iterations write the same location and each row's sum keeps its
 * serial order.
 *
 * All dense matrices are row-major fp64 with an explicit leading dimension.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int g_threads = 1;

/* Number of host threads used by the row loops (1 = serial). Returns the value in use. */
int oracle_set_threads(int t)
{
#ifdef _OPENMP
    if (t < 1) t = omp_get_num_procs();
    g_threads = t;
#else
    (void)t;
    g_threads = 1;
#endif
    return g_threads;
}

/*
 * GCN normalisation: the stored pattern is A+I (the caller has inserted the
 * self-loops), d~_i = number of stored entries of row i, and the edge value is
 * A^_ij = 1 / sqrt(d~_i * d~_j).  The paper only names the GCN model (Section VI,
 * benchmark models); this is the standard symmetric normalisation.
 * dinv may be NULL; otherwise dinv[i] = d~_i^(-1/2).
 */
void oracle_gcn_norm(int32_t n, const int32_t *row_ptr, const int32_t *col_idx,
                     double *vals, double *dinv)
{
    for (int32_t i = 0; i < n; ++i) {
        double di = (double)(row_ptr[i + 1] - row_ptr[i]);
        if (dinv) dinv[i] = di > 0.0 ? 1.0 / sqrt(di) : 0.0;
        for (int32_t e = row_ptr[i]; e < row_ptr[i + 1]; ++e) {
            int32_t j = col_idx[e];
            double dj = (double)(row_ptr[j + 1] - row_ptr[j]);
            vals[e] = 1.0 / sqrt(di * dj);
        }
    }
}

static int cmp_i32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/*
 * Sparse graph transformation (Section V.A): the rows are cut into windows of blk_h
 * consecutive rows.  For window w the neighbour ids of all its edges are sorted
 * ascending and duplicates removed, giving the window's condensed column list S_w.
 *   edge_to_row[e]     = global row of edge e                      (`edgeToRow`)
 *   edge_to_col[e]     = position of col_idx[e] inside S_w         (`edgeToColumn`)
 *   block_partition[w] = ceil(|S_w| / blk_w)                       (`blockPartition`)
 *   win_col_ptr / win_cols = the lists S_w back to back (condensed column -> row of X,
 *                            the kernel-side `sparse_AToX_index` precomputed)
 *   summary[0] = sum |S_w|,  summary[1] = sum of block_partition   (`block_counter`)
 * win_cols must have room for nnz entries.
 */
void oracle_build_windows(int32_t n, const int32_t *row_ptr, const int32_t *col_idx,
                          int32_t blk_h, int32_t blk_w,
                          int32_t *edge_to_row, int32_t *edge_to_col,
                          int32_t *block_partition, int32_t *win_col_ptr,
                          int32_t *win_cols, int64_t *summary)
{
    int32_t n_win = (n + blk_h - 1) / blk_h;
    int64_t total_unique = 0, total_blocks = 0;
    win_col_ptr[0] = 0;
    for (int32_t w = 0; w < n_win; ++w) {
        int32_t r0 = w * blk_h;
        int32_t r1 = r0 + blk_h < n ? r0 + blk_h : n;
        int32_t e0 = row_ptr[r0], e1 = row_ptr[r1];
        int32_t cnt = e1 - e0;
        int32_t *sorted = win_cols + win_col_ptr[w];
        int32_t uniq = 0;
        if (cnt > 0) {
            int32_t *tmp = (int32_t *)malloc(sizeof(int32_t) * (size_t)cnt);
            memcpy(tmp, col_idx + e0, sizeof(int32_t) * (size_t)cnt);
            qsort(tmp, (size_t)cnt, sizeof(int32_t), cmp_i32);
            for (int32_t k = 0; k < cnt; ++k)
                if (k == 0 || tmp[k] != tmp[k - 1]) sorted[uniq++] = tmp[k];
            free(tmp);
        }
        for (int32_t r = r0; r < r1; ++r)
            for (int32_t e = row_ptr[r]; e < row_ptr[r + 1]; ++e) {
                edge_to_row[e] = r;
                int32_t *hit = (int32_t *)bsearch(col_idx + e, sorted, (size_t)uniq,
                                                  sizeof(int32_t), cmp_i32);
                edge_to_col[e] = (int32_t)(hit - sorted);
            }
        block_partition[w] = (uniq + blk_w - 1) / blk_w;
        win_col_ptr[w + 1] = win_col_ptr[w] + uniq;
        total_unique += uniq;
        total_blocks += block_partition[w];
    }
    summary[0] = total_unique;
    summary[1] = total_blocks;
}

/*
 * SpMM (Section I.A.2: C = A x B with A sparse): out[i,k] = sum_e vals[e] * X[col[e],k]
 * over the stored entries e of row i, in storage order.  vals == NULL means all ones.
 * abs_out (may be NULL) receives sum_e |vals[e] * X[col[e],k]|, the scale against
 * which rounding error is judged.
 */
void oracle_spmm(int32_t n, const int32_t *row_ptr, const int32_t *col_idx,
                 const double *vals, const double *X, int64_t ldx, int32_t D,
                 double *out, double *abs_out, int64_t ldo)
{
#pragma omp parallel for schedule(dynamic, 256) num_threads(g_threads)
    for (int32_t i = 0; i < n; ++i) {
        for (int32_t k = 0; k < D; ++k) {
            double s = 0.0, a = 0.0;
            for (int32_t e = row_ptr[i]; e < row_ptr[i + 1]; ++e) {
                double t = (vals ? vals[e] : 1.0) * X[(int64_t)col_idx[e] * ldx + k];
                s += t;
                a += fabs(t);
            }
            out[(int64_t)i * ldo + k] = s;
            if (abs_out) abs_out[(int64_t)i * ldo + k] = a;
        }
    }
}

/*
 * SDDMM (Section I.A.2: D = A o (B x C) with A the 0/1 pattern): for every stored
 * entry e = (i, j):  s[e] = alpha * rs[i] * cs[j] * sum_k X[i,k] * Y[j,k].
 * rs / cs may be NULL (taken as 1).  abs_out (may be NULL) gets the same expression
 * with |X[i,k] * Y[j,k]| summed.
 */
void oracle_sddmm(int32_t n, const int32_t *row_ptr, const int32_t *col_idx,
                  const double *X, const double *Y, int64_t ld, int32_t D,
                  const double *rs, const double *cs, double alpha,
                  double *s_out, double *abs_out)
{
#pragma omp parallel for schedule(dynamic, 256) num_threads(g_threads)
    for (int32_t i = 0; i < n; ++i) {
        for (int32_t e = row_ptr[i]; e < row_ptr[i + 1]; ++e) {
            int32_t j = col_idx[e];
            double dot = 0.0, a = 0.0;
            for (int32_t k = 0; k < D; ++k) {
                double t = X[(int64_t)i * ld + k] * Y[(int64_t)j * ld + k];
                dot += t;
                a += fabs(t);
            }
            double scale = alpha * (rs ? rs[i] : 1.0) * (cs ? cs[j] : 1.0);
            s_out[e] = scale * dot;
            if (abs_out) abs_out[e] = fabs(scale) * a;
        }
    }
}

/* Inverse Euclidean row norms for the AGNN cosine: rinv[i] = 1 / max(||h_i||, 1e-12). */
void oracle_row_rnorm(int32_t n, const double *H, int64_t ld, int32_t D, double *rinv)
{
    for (int32_t i = 0; i < n; ++i) {
        double q = 0.0;
        for (int32_t k = 0; k < D; ++k) q += H[(int64_t)i * ld + k] * H[(int64_t)i * ld + k];
        double nrm = sqrt(q);
        rinv[i] = 1.0 / (nrm > 1e-12 ? nrm : 1e-12);
    }
}

/*
 * Edge softmax over the stored entries of each row:
 *   p[e] = exp(s[e] - m_i) / sum_{e' in row i} exp(s[e'] - m_i),  m_i = max of the row.
 * Empty rows write nothing.  p may alias s.
 */
void oracle_edge_softmax(int32_t n, const int32_t *row_ptr, const double *s, double *p)
{
#pragma omp parallel for schedule(dynamic, 256) num_threads(g_threads)
    for (int32_t i = 0; i < n; ++i) {
        int32_t e0 = row_ptr[i], e1 = row_ptr[i + 1];
        if (e0 == e1) continue;
        double m = s[e0];
        for (int32_t e = e0 + 1; e < e1; ++e)
            if (s[e] > m) m = s[e];
        double z = 0.0;
        for (int32_t e = e0; e < e1; ++e) z += exp(s[e] - m);
        for (int32_t e = e0; e < e1; ++e) p[e] = exp(s[e] - m) / z;
    }
}

/* Update phase (Section I.A.2): Z = X * W, X n x d_in, W d_in x d_out, plain triple loop.
 * abs_out (may be NULL) = |X| * |W|. */
void oracle_gemm(int32_t n, int32_t d_in, int32_t d_out, const double *X, int64_t ldx,
                 const double *W, int64_t ldw, double *Z, double *abs_out, int64_t ldz)
{
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (int32_t i = 0; i < n; ++i)
        for (int32_t k = 0; k < d_out; ++k) {
            double s = 0.0, a = 0.0;
            for (int32_t j = 0; j < d_in; ++j) {
                double t = X[(int64_t)i * ldx + j] * W[(int64_t)j * ldw + k];
                s += t;
                a += fabs(t);
            }
            Z[(int64_t)i * ldz + k] = s;
            if (abs_out) abs_out[(int64_t)i * ldz + k] = a;
        }
}

/*
 * GCN layer forward: out = act(A^ * (X * W)), act = ReLU when relu != 0, identity
 * otherwise.  No intermediate rounding.  abs_out (may be NULL) = |A^| * (|X| * |W|).
 * Z and Zabs are caller-provided n x d_out scratch.
 */
void oracle_gcn_layer(int32_t n, const int32_t *row_ptr, const int32_t *col_idx,
                      const double *vals, const double *X, int64_t ldx, int32_t d_in,
                      const double *W, int32_t d_out, int32_t relu,
                      double *Z, double *Zabs, double *out, double *abs_out)
{
    oracle_gemm(n, d_in, d_out, X, ldx, W, d_out, Z, Zabs, d_out);
    oracle_spmm(n, row_ptr, col_idx, vals, Z, d_out, d_out, out, NULL, d_out);
    if (abs_out) {
        /* |vals| * Zabs, written out term by term */
        for (int32_t i = 0; i < n; ++i)
            for (int32_t k = 0; k < d_out; ++k) {
                double a = 0.0;
                for (int32_t e = row_ptr[i]; e < row_ptr[i + 1]; ++e)
                    a += fabs(vals ? vals[e] : 1.0) * Zabs[(int64_t)col_idx[e] * d_out + k];
                abs_out[(int64_t)i * d_out + k] = a;
            }
    }
    if (relu)
        for (int64_t t = 0; t < (int64_t)n * d_out; ++t)
            if (out[t] < 0.0) out[t] = 0.0;
}

/*
 * AGNN propagation layer forward: scores s_ij = beta * cos(h_i, h_j) on the stored
 * entries, P = row-wise edge softmax of s, out = P * H with the un-normalised H.
 * p_out has nnz entries; rinv is caller-provided scratch of n entries.
 */
void oracle_agnn_layer(int32_t n, const int32_t *row_ptr, const int32_t *col_idx,
                       const double *H, int64_t ld, int32_t D, double beta,
                       double *rinv, double *p_out, double *out, double *abs_out)
{
    oracle_row_rnorm(n, H, ld, D, rinv);
    oracle_sddmm(n, row_ptr, col_idx, H, H, ld, D, rinv, rinv, beta, p_out, NULL);
    oracle_edge_softmax(n, row_ptr, p_out, p_out);
    oracle_spmm(n, row_ptr, col_idx, p_out, H, ld, D, out, abs_out, D);
}

/* Padded tile capacity of a transformed graph: every TC block holds blk_h x blk_w cells
 * (dataset table, Section VI: the "edges" column equals blocks x 16 x 8). */
int64_t oracle_tile_capacity(int64_t block_counter, int32_t blk_h, int32_t blk_w)
{
    return block_counter * (int64_t)blk_h * (int64_t)blk_w;
}
