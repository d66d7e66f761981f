/*
 * ftc.h -- C ABI of libftc: sparse neighbour aggregation for GCN / AGNN on AMD gfx950,
 * after FTC-GNN (arXiv 2412.12218).
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  - Every array pointer inside the structs and in the argument lists is a DEVICE
 *    pointer owned by the caller; the structs themselves and all scalars live on the
 *    host.  The library never allocates or frees device memory, never synchronises and
 *    never prints: a call validates its arguments on the host and enqueues kernels on
 *    `stream` (a hipStream_t passed as void*, NULL = the default stream).  Scratch
 *    memory comes from a caller-provided workspace whose size is returned by the
 *    matching *_workspace_bytes query (a pure host function).  The library keeps no state
 *    between calls apart from the thread-local error text (and the built-in scratch buffer of
 *    ftc_spmm_noalloc); a call may be recorded into a HIP graph, the first one included.
 *  - Return value: FTC_OK or a negative ftc_status; ftc_last_error() returns a
 *    thread-local description of the last failure.
 *  - The graph is a CSR adjacency with int32 indices (`nodePointer` / `edgeList` in the
 *    paper, Section V.A).  Column indices within a row may be unsorted and may repeat;
 *    repeated entries are separate edges whose contributions add.  Index validity
 *    (monotone row_ptr, 0 <= col < n) is the caller's responsibility and can be checked
 *    with ftc_validate_csr.
 *  - Dense matrices are row-major with a leading dimension in ELEMENTS.  The vector
 *    kernels need the base pointer 16-byte aligned and ld * sizeof(element) a multiple of
 *    16 with D a multiple of 8 (16-bit types) or 4 (fp32); other shapes take a slower
 *    generic kernel.  Outputs never alias inputs unless stated.
 *  - n == 0 or nnz == 0 is legal.  A row without stored entries produces a zero output row
 *    (SpMM / layers) and no softmax output.
 */
#ifndef FTC_H
#define FTC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FTC_OK = 0,
    FTC_EINVAL = -1,       /* null pointer, negative size, inconsistent sizes          */
    FTC_EUNSUPPORTED = -2, /* dtype / dimension / tile combination not implemented      */
    FTC_EALIGN = -3,       /* pointer or leading dimension violates a stated alignment  */
    FTC_EWORKSPACE = -4,   /* workspace missing or smaller than *_workspace_bytes says  */
    FTC_EHIP = -5          /* the HIP runtime reported an error at launch               */
} ftc_status;

typedef enum { FTC_F32 = 0, FTC_F16 = 1, FTC_BF16 = 2 } ftc_dtype;

/* Kernel family used by ftc_spmm / ftc_sddmm and the layers built on them. */
typedef enum {
    FTC_PATH_AUTO = 0, /* per row window: matrix-core tiles where the condensed window is
                          dense enough, vector gather elsewhere                          */
    FTC_PATH_VALU = 1, /* vector gather path for every window                           */
    FTC_PATH_MFMA = 2  /* matrix-core condensed-tile path for every window (16-bit only) */
} ftc_path;

/* CSR adjacency: row_ptr[n+1], col_idx[nnz]; row_ptr[0] == 0, row_ptr[n] == nnz. */
typedef struct {
    int32_t n;
    int32_t nnz;
    const int32_t *row_ptr;
    const int32_t *col_idx;
} ftc_csr;

/*
 * Output of the sparse graph transformation (Section V.A).  Rows are cut into windows
 * of blk_h consecutive rows (the last one may be short); S_w is the ascending list of
 * distinct column ids used by window w.
 *   edge_to_row[e]      global row of edge e                              [nnz]
 *   edge_to_col[e]      position of col_idx[e] in S_w of the edge's window [nnz]
 *   block_partition[w]  ceil(|S_w| / blk_w): TC blocks of window w        [n_windows]
 *   win_col_ptr[w]      start of S_w inside win_cols                      [n_windows+1]
 *   win_cols            S_0, S_1, ... back to back; capacity nnz entries  [nnz]
 *   summary[0]          sum of |S_w|;  summary[1] = sum of block_partition
 *                       (`block_counter`)                                 [2]
 * All arrays are allocated by the caller before ftc_build_windows fills them.
 */
typedef struct {
    int32_t blk_h;
    int32_t blk_w;
    int32_t n_windows; /* ceil(n / blk_h) */
    int32_t *edge_to_row;
    int32_t *edge_to_col;
    int32_t *block_partition;
    int32_t *win_col_ptr;
    int32_t *win_cols;
    int64_t *summary;
} ftc_windows;

/* Library version: major * 10000 + minor * 100 + patch. */
int32_t ftc_version(void);

/* Description of the last error on this host thread ("" if none). Never NULL. */
const char *ftc_last_error(void);

/*
 * Checks on the device that row_ptr is non-decreasing with row_ptr[0] == 0 and
 * row_ptr[n] == nnz, and that every column index lies in [0, n).  *flag (device int32)
 * is set to 0 when the graph is valid, otherwise to a bit mask: 1 = row_ptr, 2 = col_idx.
 */
int32_t ftc_validate_csr(const ftc_csr *g, int32_t *flag, void *stream);

/*
 * Sparse graph transformation (Section V.A, `edgeToRow`, `edgeToColumn`,
 * `blockPartition`, `block_counter`; TC_BLK_H = 16 and TC_BLK_W = 8 in the paper, both
 * free here with 1 <= blk_h <= 64 and blk_w >= 1).  Fills every array of `out`;
 * out->blk_h, blk_w and n_windows are inputs and must be consistent with g->n.  The
 * result is uniquely determined (ascending order, strict de-duplication).
 */
size_t ftc_build_windows_workspace_bytes(int32_t n, int32_t nnz, int32_t blk_h, int32_t blk_w);
int32_t ftc_build_windows(const ftc_csr *g, ftc_windows *out, void *ws, size_t ws_bytes,
                          void *stream);

/*
 * The same transformation with its independent kernels side by side.  Windows of different sizes
 * are condensed by different kernels (Section V.A: the windows do not depend on each other), each of
 * which fills only part of the GPU; given three more streams they overlap (0.39 instead of 0.54 ms
 * on the R-MAT benchmark graph).  `side` holds three hipStream_t and four hipEvent_t (timing may be
 * disabled) created by the caller on the device of `stream`, all at the default priority: `stream`
 * forks into the side streams through `fork` after the classification and waits for `join[i]` of
 * each before the final scan, so for the caller everything still happens in stream order and nothing
 * waits on the host.  The handles are used only during the call; two calls that overlap in time need
 * two sets.  side == NULL is ftc_build_windows.
 */
typedef struct {
    void *stream[3]; /* hipStream_t */
    void *fork;      /* hipEvent_t  */
    void *join[3];   /* hipEvent_t  */
} ftc_side_streams;
int32_t ftc_build_windows_concurrent(const ftc_csr *g, ftc_windows *out, void *ws, size_t ws_bytes,
                                     const ftc_side_streams *side, void *stream);

/*
 * Symmetric GCN normalisation for a pattern that already contains the self-loops
 * (the paper names the GCN model in Section VI; the formula is the standard
 * A^ = D~^-1/2 (A+I) D~^-1/2).  d~_i = number of stored entries of row i,
 * dinv[i] = d~_i^-1/2 (0 for an empty row), vals[e] = dinv[row(e)] * dinv[col_idx[e]].
 * Either output may be NULL.  w may be NULL; when given, its edge_to_row is used to
 * find the row of an edge.
 */
int32_t ftc_gcn_norm(const ftc_csr *g, const ftc_windows *w, float *vals, float *dinv,
                     void *stream);

/*
 * Sparse neighbour aggregation (Section V.A; SpMM C = A x B of Section I.A.2):
 *   out[i, 0:D] = sum over stored entries e of row i of vals[e] * X[col_idx[e], 0:D]
 * accumulated in fp32.  vals == NULL means all ones.  X has g->n rows of dtype x_dtype;
 * out has g->n rows of dtype out_dtype.  out_scale (n floats, may be NULL) multiplies output
 * row i by out_scale[i]; relu != 0 then applies max(0, .) before the store.
 * w may be NULL (vector path on the CSR only).  `path` is an ftc_path.
 */
size_t ftc_spmm_workspace_bytes(int32_t n, int32_t nnz, int32_t D);
int32_t ftc_spmm(const ftc_csr *g, const ftc_windows *w, const float *vals, const void *X,
                 int32_t ldx, int32_t x_dtype, int32_t D, void *out, int32_t ldo,
                 int32_t out_dtype, const float *out_scale, int32_t relu, int32_t path, void *ws,
                 size_t ws_bytes, void *stream);

/*
 * ftc_spmm for callers that cannot allocate device memory and have no workspace to pass: code under
 * HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments, same
 * kernels and bit-identical results; the scratch memory is a buffer of FTC_NOALLOC_SCRATCH_MIB MiB
 * built into the library (one copy per GPU, held until the process ends).  The call allocates and
 * frees nothing.  FTC_EWORKSPACE when ftc_spmm_workspace_bytes(n, nnz, D) exceeds the buffer (about
 * nnz * D > 4e9 with 16-bit features).  The device that `stream` belongs to must be current.  All
 * calls on one GPU share the buffer: calls that overlap in time on one GPU (different streams, or
 * several host threads) race; calls in one stream are safe.  Nothing in the buffer has to be zero and
 * nothing is kept between calls.  The first call on a device looks up the buffer's address.
 */
#define FTC_NOALLOC_SCRATCH_MIB 64
int32_t ftc_spmm_noalloc(const ftc_csr *g, const ftc_windows *w, const float *vals, const void *X,
                         int32_t ldx, int32_t x_dtype, int32_t D, void *out, int32_t ldo,
                         int32_t out_dtype, const float *out_scale, int32_t relu, int32_t path,
                         void *stream);

/*
 * Sparse edge feature computation (Section V.A; SDDMM D = A o (B x C) of Section I.A.2,
 * A taken as the 0/1 pattern), result laid out like col_idx (`EdgeValList`):
 *   edge_out[e] = alpha * row_scale[i] * col_scale[j] * sum_k X[i,k] * Y[j,k],
 *   i = row of e, j = col_idx[e].
 * X and Y have g->n rows, the same dtype and leading dimension, and may be the same
 * matrix.  row_scale / col_scale may be NULL (1.0).
 * cosine != 0 selects the AGNN edge score instead: the scales are the inverse Euclidean norms of
 * the rows themselves,
 *   edge_out[e] = alpha * sum_k X[i,k] * Y[j,k] / (max(||X[i,:]||, 1e-12) * max(||Y[j,:]||, 1e-12)),
 * row_scale and col_scale must then be NULL; no array of norms has to exist, the vector
 * kernel recomputes them from the rows it has loaded.
 */
size_t ftc_sddmm_workspace_bytes(int32_t n, int32_t nnz, int32_t D);
int32_t ftc_sddmm(const ftc_csr *g, const ftc_windows *w, const void *X, const void *Y,
                  int32_t ld, int32_t dtype, int32_t D, const float *row_scale,
                  const float *col_scale, float alpha, int32_t cosine, float *edge_out,
                  int32_t path, void *ws, size_t ws_bytes, void *stream);

/*
 * Inverse Euclidean row norms used by the AGNN cosine: rinv[i] = 1 / max(||H[i,:]||, 1e-12).
 */
int32_t ftc_row_rnorm(int32_t n, const void *H, int32_t ld, int32_t dtype, int32_t D,
                      float *rinv, void *stream);

/*
 * Edge softmax over the stored entries of every row (the attention weights of AGNN,
 * which the paper names in Section VI):
 *   p[e] = exp(s[e] - m_i) / sum_{e' in row i} exp(s[e'] - m_i),  m_i = max over row i.
 * p_out may alias e_in.  Rows without entries write nothing.  w may be NULL; with a window
 * index the work is split by edges (edge_to_row), which keeps hub rows from serialising,
 * and a workspace of ftc_edge_softmax_workspace_bytes is needed (none when w is NULL).
 */
size_t ftc_edge_softmax_workspace_bytes(int32_t n, int32_t nnz);
int32_t ftc_edge_softmax(const ftc_csr *g, const ftc_windows *w, const float *e_in, float *p_out,
                         void *ws, size_t ws_bytes, void *stream);

/*
 * Dense update phase (Section I.A.2): Z = X * W, X n x d_in (dtype), W d_in x d_out
 * row-major of the same dtype, fp32 accumulation, Z n x d_out of z_dtype.
 * Any d_in, d_out >= 1: W stays on chip for d_in <= 256 and d_out <= 64 (the benchmark models);
 * wider inputs are contracted in chunks, wider outputs written in groups of 64 columns (X is read
 * once per group).  row_scale (n floats, may be NULL) multiplies row i of the product by
 * row_scale[i]; relu != 0 then applies max(0, .).
 */
int32_t ftc_update_gemm(int32_t n, const void *X, int32_t ldx, int32_t dtype, int32_t d_in,
                        const void *W, int32_t d_out, void *Z, int32_t ldz, int32_t z_dtype,
                        const float *row_scale, int32_t relu, void *stream);

/*
 * GCN layer forward: out = act(A^ * (X * W)) with A^ given by (g, vals); update first,
 * then aggregation (Eq. 1-2 of Section I).  W is d_in x d_out row-major, same dtype as X.
 * The intermediate X * W lives in the workspace: fp16 for fp16 inputs, fp32 otherwise.
 * dinv (n floats, may be NULL) selects the factored form of the symmetric normalisation:
 * the edge values are dinv[i] * dinv[j], `vals` is ignored (may be NULL), row j of X * W is
 * scaled by dinv[j] when it is written, the aggregation runs without edge values and output
 * row i is scaled by dinv[i].  No per-edge value array is read then.
 */
size_t ftc_gcn_layer_workspace_bytes(int32_t n, int32_t nnz, int32_t d_in, int32_t d_out);
int32_t ftc_gcn_layer(const ftc_csr *g, const ftc_windows *w, const float *vals,
                      const float *dinv, const void *X, int32_t ldx, int32_t dtype, int32_t d_in,
                      const void *W, int32_t d_out, int32_t relu, void *out, int32_t ldo,
                      int32_t out_dtype, int32_t path, void *ws, size_t ws_bytes, void *stream);

/*
 * AGNN propagation layer forward: s_ij = beta * cos(h_i, h_j) on the stored entries,
 * P = edge softmax of s, out = P * H (H not normalised).  edge_p, when not NULL,
 * receives P (nnz floats).  Without edge_p (and with a window index) scores, softmax and
 * aggregation run fused in one pass over the edges; the softmax is then shifted by |beta|,
 * an upper bound of every score, instead of by the row maximum (same result); for |beta| >= 43 the
 * unfused chain with the row-wise softmax is used.
 * row_z, when not NULL, receives the softmax denominators of that pass,
 * z_i = sum over row i of exp(beta * cos - |beta|) (n floats, 0 for a row without entries): what
 * ftc_agnn_layer_backward_fused needs instead of P.  out_f32, when not NULL, receives the result
 * once more, unrounded (n x D fp32, leading dimension ld_f32, a multiple of 4; rows 16-byte
 * aligned): the backward pass takes <dY_i, out_i> from it when `out` itself is 16-bit.  Only the
 * fused pass produces these two (FTC_EUNSUPPORTED together with edge_p, without a window index or
 * for shapes it does not cover).
 */
size_t ftc_agnn_layer_workspace_bytes(int32_t n, int32_t nnz, int32_t D);
int32_t ftc_agnn_layer(const ftc_csr *g, const ftc_windows *w, const void *H, int32_t ld,
                       int32_t dtype, int32_t D, float beta, void *out, int32_t ldo,
                       int32_t out_dtype, float *edge_p, float *row_z, float *out_f32,
                       int32_t ld_f32, int32_t path, void *ws, size_t ws_bytes, void *stream);

/*
 * ---- Backward pass ----------------------------------------------------------------------------
 * The paper speaks of GNN training as well as inference (Sections II and V) and gives no gradient
 * formulas; the entry points below compute the derivatives of the forward definitions above.
 * Gradient arrays are fp32.  The sparse products of the backward pass run on the forward SpMM /
 * SDDMM kernels.
 */

/*
 * Transposed index of a symmetric pattern: T[e] = position of the stored entry (j, i) for the
 * stored entry e = (i, j), -1 where the pattern does not hold it; *flag (device int32) becomes 1
 * if any entry has no partner, else 0.  Needs ascending, duplicate-free columns inside every row.
 * w may be NULL (its edge_to_row only saves a search).
 */
int32_t ftc_transpose_index(const ftc_csr *g, const ftc_windows *w, int32_t *T, int32_t *flag,
                            void *stream);

/*
 * Derivative of ftc_edge_softmax: ds[e] = p[e] * (dp[e] - sum over the row of p * dp).
 * ds may alias dp.  w and the workspace (ftc_edge_softmax_workspace_bytes) as in ftc_edge_softmax:
 * with the window index the work is split by entries, not rows (no long-row imbalance).
 */
int32_t ftc_edge_softmax_backward(const ftc_csr *g, const ftc_windows *w, const float *p,
                                  const float *dp, float *ds, void *ws, size_t ws_bytes,
                                  void *stream);

/*
 * Weight gradient of the update phase: dW = X^T * G, X n x d_in (x_dtype), G n x d_out (fp32),
 * dW d_in x d_out row-major (fp32).  One pass covers ceil(d_in / 4) * ceil(d_out / 4) <= 1024 and
 * d_in + d_out <= 506; a wider X is taken in groups of up to 256 input columns (every pass reads G
 * again), d_out <= 504 (FTC_EUNSUPPORTED beyond).  Partial sums of row blocks are added in a fixed
 * order (reproducible).
 */
size_t ftc_weight_grad_workspace_bytes(int32_t n, int32_t d_in, int32_t d_out);
int32_t ftc_weight_grad(int32_t n, const void *X, int32_t ldx, int32_t x_dtype, int32_t d_in,
                        const float *G, int32_t ldg, int32_t d_out, float *dW, void *ws,
                        size_t ws_bytes, void *stream);

/*
 * Backward of ftc_update_gemm (Z = act(X * W), no row scale) for a loss with dL/dZ = dZ (n x d_out,
 * fp32): dP = dZ where the layer's output Z was positive (Z == NULL: no ReLU, dP = dZ),
 * dW = X^T * dP (d_in x d_out, fp32), dX = dP * W^T (n x d_in, of type dx_dtype; dX == NULL:
 * skipped).  Any d_in; d_out <= 504 (beyond 64 output columns dX is computed by the kernels of
 * ftc_update_gemm on the transposed weights).
 */
size_t ftc_update_gemm_backward_workspace_bytes(int32_t n, int32_t d_in, int32_t d_out);
int32_t ftc_update_gemm_backward(int32_t n, const void *X, int32_t ldx, int32_t dtype, int32_t d_in,
                                 const void *W, int32_t d_out, const void *Z, int32_t ldz,
                                 int32_t z_dtype, const float *dZ, int32_t lddz, void *dX,
                                 int32_t lddx, int32_t dx_dtype, float *dW, void *ws,
                                 size_t ws_bytes, void *stream);

/*
 * Backward of ftc_gcn_layer for a loss with dL/d(out) = dY (n x d_out, fp32):
 *   dP = dY where the layer's output Y was positive (Y == NULL: no ReLU, dP = dY),
 *   dZ = A^^T * dP,  dW = X^T * dZ (d_in x d_out),  dX = dZ * W^T (n x d_in; dX == NULL: skipped).
 * (gT, wT, valsT) describe A^^T: the transposed graph, its window index and its edge values; for
 * the symmetric GCN normalisation they are the forward graph itself.  dinv != NULL selects the
 * factored normalisation as in ftc_gcn_layer (valsT ignored).  X, W as in the forward call;
 * d_out <= 504.
 */
size_t ftc_gcn_layer_backward_workspace_bytes(int32_t n, int32_t nnz, int32_t d_in, int32_t d_out);
int32_t ftc_gcn_layer_backward(const ftc_csr *gT, const ftc_windows *wT, const float *valsT,
                               const float *dinv, const void *X, int32_t ldx, int32_t dtype,
                               int32_t d_in, const void *W, int32_t d_out, const void *Y,
                               int32_t ldy, int32_t y_dtype, const float *dY, int32_t lddy,
                               float *dX, int32_t lddx, float *dW, int32_t path, void *ws,
                               size_t ws_bytes, void *stream);

/*
 * Backward of ftc_agnn_layer for a loss with dL/d(out) = dY (n x D, same dtype and leading
 * dimension as H): dH (n x D, of type dh_dtype: fp32, or a 16-bit type when the layer below takes
 * its incoming gradient in that type) and *dbeta (device fp32).  p are the probabilities of the
 * forward pass (edge_p of ftc_agnn_layer), T the transposed index of the pattern, which must be
 * symmetric (ftc_transpose_index with flag 0).  With hn_i = h_i / max(|h_i|, 1e-12),
 * c_e = <hn_i, hn_j>:
 *   dp_e = <dY_i, h_j>,  ds = softmax backward of (p, dp),  dbeta = sum_e ds_e c_e,
 *   q_i = beta * sum_e (ds_e + ds_T(e)) hn_j,
 *   dH_i = sum_e p_T(e) dY_j  +  (q_i - hn_i <hn_i, q_i>) / |h_i|.
 */
size_t ftc_agnn_layer_backward_workspace_bytes(int32_t n, int32_t nnz, int32_t D);
int32_t ftc_agnn_layer_backward(const ftc_csr *g, const ftc_windows *w, const int32_t *T,
                                const void *H, int32_t ld, int32_t dtype, int32_t D, float beta,
                                const float *p, const void *dY, int32_t lddy, void *dH,
                                int32_t lddh, int32_t dh_dtype, float *dbeta, int32_t path,
                                void *ws, size_t ws_bytes, void *stream);

/*
 * The same gradients in one pass over the entries, for a symmetric pattern: every entry gathers
 * h_j and dY_j once and the per-node pair (1 / z_j, <dY_j, Y_j>); no edge array (probabilities,
 * transposed index) is read or written.  row_z are the denominators of the forward pass (row_z of
 * ftc_agnn_layer with the same H and beta), Y its output (n x D, any dtype; it enters through
 * <dY_i, Y_i> = sum over row i of p * dp, so a 16-bit Y costs accuracy -- a few 1e-3 of a row's
 * largest gradient entry with bf16 -- and out_f32 of the forward call is the better choice).
 * H and dY share dtype and leading dimension, rows 16-byte aligned; the window index is required;
 * (dtype, D) must be a width the single-pass forward covers, with at most 128 elements once
 * padded to its lane layout (ftc_plan_graph reports it), and |beta| < 43.  FTC_EUNSUPPORTED otherwise: use
 * ftc_agnn_layer_backward.  The formulas hold on a symmetric pattern only.  pattern_flag (device
 * int32, may be NULL) is the flag ftc_transpose_index wrote for this graph: when it is not zero
 * (some entry has no transposed partner) every element of dH and *dbeta is set to NaN instead of a
 * gradient of nothing.  NULL: the caller vouches for the symmetry.
 */
size_t ftc_agnn_layer_backward_fused_workspace_bytes(int32_t n, int32_t nnz, int32_t D);
int32_t ftc_agnn_layer_backward_fused(const ftc_csr *g, const ftc_windows *w, const void *H,
                                      int32_t ld, int32_t dtype, int32_t D, float beta,
                                      const float *row_z, const void *Y, int32_t ldy,
                                      int32_t y_dtype, const void *dY, int32_t lddy, void *dH,
                                      int32_t lddh, int32_t dh_dtype, float *dbeta,
                                      const int32_t *pattern_flag, void *ws, size_t ws_bytes,
                                      void *stream);

/*
 * ---- Locality reordering (preprocessing) ------------------------------------------------------
 * The sparse graph transformation (Section IV.A) condenses the columns that the rows of a window
 * share; how many they share, and how often a gathered feature row is still in cache, depends on
 * the numbering of the nodes, which the paper takes as given.  These calls relabel the nodes before
 * the transformation and keep a permutation-in / permutation-out contract:
 *   perm[new] = old id, inv[old] = new id (device, int32, n entries each);
 *   features enter the new numbering with ftc_permute_rows(map = perm), results leave it with
 *   ftc_permute_rows(map = inv); the layers themselves run on the relabelled graph unchanged.
 * All results are unique (stable sorts) and reproducible.
 */
enum {
    FTC_ORDER_NONE = -1,          /* keep the numbering (a value of ftc_plan.reorder only) */
    FTC_ORDER_DEGREE = 0,         /* descending number of stored entries of the row, ties: ascending id */
    FTC_ORDER_DEGREE_CLASSES = 1, /* descending bit length of that number (power-of-two classes), ties:
                                     ascending id -- keeps the given order inside a class */
    FTC_ORDER_COMMUNITIES = 2     /* a value of ftc_plan.reorder only: ftc_label_propagation +
                                     ftc_order_by_key are worth a trial (keep the result if the window
                                     build's sum_uniq drops) */
};

/* Workspace of ftc_degree_order, ftc_order_by_key, ftc_label_propagation and ftc_permute_graph. */
size_t ftc_reorder_workspace_bytes(int32_t n, int32_t nnz);

/* perm and inv of the ordering `mode` of g's nodes. */
int32_t ftc_degree_order(const ftc_csr *g, int32_t mode, int32_t *perm, int32_t *inv, void *ws,
                         size_t ws_bytes, void *stream);

/*
 * perm and inv of the ascending order of keys[0 .. n) (device, int32, >= 0), ties by ascending id:
 * nodes with equal keys -- the same community label, say -- become neighbours in the new numbering.
 * *flag (device int32) becomes 1 if a key is negative (it is then ordered as 0), else 0.
 */
int32_t ftc_order_by_key(int32_t n, const int32_t *keys, int32_t *perm, int32_t *inv,
                         int32_t *flag, void *ws, size_t ws_bytes, void *stream);

/*
 * Community labels by synchronous label propagation, for a community ordering with
 * ftc_order_by_key: every node starts with its own id; in each of `rounds` rounds every node takes
 * the label that occurs most often among the stored entries of its row (duplicates count, a
 * self-loop counts the node's own label; the smallest label on a tie), all nodes at once from the
 * labels of the round before; a row without entries keeps its label.  labels: device int32[n].
 * Ten rounds recover the blocks of the stochastic-block-model benchmark graph.  Unique result.
 */
int32_t ftc_label_propagation(const ftc_csr *g, int32_t rounds, int32_t *labels, void *ws,
                              size_t ws_bytes, void *stream);

/*
 * Relabelled graph: row `new` of the output holds the entries of row perm[new] of g with every
 * column c replaced by inv[c], ascending inside the row, duplicates kept.  row_ptr_out has n + 1
 * entries, col_idx_out nnz.  (perm, inv) may come from ftc_degree_order or from the caller (e.g. a
 * community ordering); *flag (device int32) becomes 1 if they are not a permutation and its
 * inverse -- no index is followed unchecked, the output is then unspecified -- else 0.
 */
int32_t ftc_permute_graph(const ftc_csr *g, const int32_t *perm, const int32_t *inv,
                          int32_t *row_ptr_out, int32_t *col_idx_out, int32_t *flag, void *ws,
                          size_t ws_bytes, void *stream);

/*
 * out[r, :] = X[map[r], :] for r in [0, n): X and out are n x D matrices of the same dtype; a map
 * entry outside [0, n) gives a row of zeros.  out must not alias X.
 */
int32_t ftc_permute_rows(int32_t n, const void *X, int32_t ldx, int32_t dtype, int32_t D,
                         const int32_t *map, void *out, int32_t ldo, void *stream);

/*
 * ---- Per-graph plan ---------------------------------------------------------------------------
 * The paper's outlook (Section VII) names a framework that adapts its use of the hardware to the
 * input graph.  Here the adaptation has two levels.  Per window: FTC_PATH_AUTO sends a window to the
 * matrix cores or to the vector kernels by its density, with measured crossovers (ftc_spmm,
 * ftc_sddmm).  Per graph: ftc_plan_graph turns a few statistics, gathered once at build time, into
 * the choices that hold for the whole graph.  The statistics live on the device (ftc_degree_stats,
 * and summary[0] of ftc_build_windows); the caller copies them to the host once per graph.
 */

/* stats[0] = sum over the rows of (stored entries)^2, stats[1] = longest row (device, int64[2]). */
int32_t ftc_degree_stats(const ftc_csr *g, int64_t *stats, void *stream);

typedef struct {
    double skew;          /* n * sum_deg_sq / nnz^2: mean popularity of the node an entry points to, relative to
                             the mean row length (1 for a regular graph; row lengths stand in for column counts,
                             exact on symmetric patterns) */
    double reuse;         /* nnz / sum_uniq: stored entries per condensed column, averaged over the windows */
    int32_t reorder;      /* the ordering to apply, for a feature matrix (n * D elements) larger than one L2
                             (4 MiB): FTC_ORDER_DEGREE_CLASSES when skew >= 2, FTC_ORDER_COMMUNITIES (a trial
                             of the community ordering) for flatter degrees with at least 8 entries per row on
                             average; else FTC_ORDER_NONE */
    int32_t agnn_single_pass;           /* ftc_agnn_layer without edge_p runs as one pass for this (dtype, D) */
    int32_t agnn_backward_single_pass;  /* ftc_agnn_layer_backward_fused covers this (dtype, D) */
    int32_t spmm_mfma_windows;   /* FTC_PATH_AUTO may send windows of this (dtype, D) to the matrix cores ... */
    int32_t sddmm_mfma_windows;  /* ... for SpMM / for SDDMM */
    float mfma_min_reuse;        /* entries per condensed column from which a window goes there (< 0: never) */
} ftc_plan;

/* Host-only, pure.  sum_deg_sq from ftc_degree_stats, sum_uniq = summary[0] of ftc_build_windows. */
int32_t ftc_plan_graph(int32_t n, int32_t nnz, int64_t sum_deg_sq, int64_t sum_uniq, int32_t D,
                       int32_t dtype, ftc_plan *plan);

#ifdef __cplusplus
}
#endif
#endif /* FTC_H */
