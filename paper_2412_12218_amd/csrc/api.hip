// C ABI of libftc: host-side argument validation and dispatch.  See include/ftc.h for the
// contract of every entry point.
#include <cstdarg>
#include <cstdio>
#include <mutex>

#include "ftc_common.hpp"

namespace ftc {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

int32_t launch_status(const char *what)
{
    const hipError_t e = hipGetLastError();
    if (e == hipSuccess) return FTC_OK;
    set_error("%s: HIP error %d (%s)", what, static_cast<int>(e), hipGetErrorString(e));
    return FTC_EHIP;
}

static int32_t fail(int32_t code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

static int32_t check_csr(const ftc_csr *g, const char *who)
{
    if (!g) return fail(FTC_EINVAL, "%s: graph is NULL", who);
    if (g->n < 0 || g->nnz < 0) return fail(FTC_EINVAL, "%s: negative n or nnz", who);
    if (!g->row_ptr) return fail(FTC_EINVAL, "%s: row_ptr is NULL", who);
    if (g->nnz > 0 && !g->col_idx) return fail(FTC_EINVAL, "%s: col_idx is NULL", who);
    if (g->n == 0 && g->nnz != 0) return fail(FTC_EINVAL, "%s: nnz > 0 with n == 0", who);
    return FTC_OK;
}

static int32_t check_windows(const ftc_csr *g, const ftc_windows *w, const char *who, bool need_arrays)
{
    if (!w) return fail(FTC_EINVAL, "%s: window index is NULL", who);
    if (w->blk_h < 1 || w->blk_h > 64 || w->blk_w < 1)
        return fail(FTC_EUNSUPPORTED, "%s: need 1 <= blk_h <= 64 and blk_w >= 1", who);
    if (w->n_windows != (g->n + w->blk_h - 1) / w->blk_h)
        return fail(FTC_EINVAL, "%s: n_windows != ceil(n / blk_h)", who);
    if (need_arrays) {
        if (!w->win_col_ptr || !w->summary || (w->n_windows > 0 && !w->block_partition))
            return fail(FTC_EINVAL, "%s: window arrays are NULL", who);
        if (g->nnz > 0 && (!w->edge_to_row || !w->edge_to_col || !w->win_cols))
            return fail(FTC_EINVAL, "%s: window edge arrays are NULL", who);
    }
    return FTC_OK;
}

static int32_t check_dense(const void *p, int ld, int dtype, int D, const char *who, const char *name)
{
    if (!p) return fail(FTC_EINVAL, "%s: %s is NULL", who, name);
    if (!valid_dtype(dtype)) return fail(FTC_EUNSUPPORTED, "%s: unknown dtype for %s", who, name);
    if (D < 1 || ld < D) return fail(FTC_EINVAL, "%s: need D >= 1 and ld >= D for %s", who, name);
    if (reinterpret_cast<uintptr_t>(p) % elem_size(dtype) != 0)
        return fail(FTC_EALIGN, "%s: %s is not aligned to its element size", who, name);
    return FTC_OK;
}

}  // namespace ftc

using namespace ftc;

// FTC_PATH_AUTO sends a window to the matrix cores when it has at least this many edges per
// condensed column (average reuse of a gathered row).  Values are the measured crossovers of the
// density sweep (bench.py --sweep, fp16, 2^18 nodes, 8.4 M edges): the vector path wins at every
// density up to completely full tiles for D <= 128 (both operations) and for SpMM at D = 256;
// SDDMM at D = 256 crosses over between 2.3 and 2.8 edges per condensed column.  A negative
// value means "never".
static float spmm_mfma_reuse(int D) { (void)D; return -1.f; }
static float sddmm_mfma_reuse(int D) { return D >= 256 ? 2.6f : -1.f; }
// Larger windows (hub rows) always stay on the edge-balanced vector kernels.
static constexpr int MFMA_MAX_WINDOW_EDGES = 4096;
// |beta| up to which the single-pass AGNN kernels (forward and backward) are used
static constexpr float AGNN_FUSED_MAX_BETA = 43.f;

static size_t flag_bytes(int32_t n) { return align_up(static_cast<size_t>((n + 15) / 16), 256); }

#define FTC_TRY(expr)                   \
    do {                                \
        const int32_t st__ = (expr);    \
        if (st__ != FTC_OK) return st__; \
    } while (0)

extern "C" {

int32_t ftc_version(void) { return 100; }

const char *ftc_last_error(void) { return g_err; }

int32_t ftc_validate_csr(const ftc_csr *g, int32_t *flag, void *stream)
{
    FTC_TRY(check_csr(g, "ftc_validate_csr"));
    if (!flag) return fail(FTC_EINVAL, "ftc_validate_csr: flag is NULL");
    return launch_validate(*g, flag, static_cast<hipStream_t>(stream));
}

size_t ftc_build_windows_workspace_bytes(int32_t n, int32_t nnz, int32_t blk_h, int32_t blk_w)
{
    if (n < 0 || nnz < 0 || blk_h < 1 || blk_w < 1) return 0;
    return build_windows_ws(n, nnz, blk_h, blk_w);
}

int32_t ftc_build_windows_concurrent(const ftc_csr *g, ftc_windows *out, void *ws, size_t ws_bytes,
                                     const ftc_side_streams *side, void *stream)
{
    FTC_TRY(check_csr(g, "ftc_build_windows"));
    FTC_TRY(check_windows(g, out, "ftc_build_windows", true));
    const size_t need = build_windows_ws(g->n, g->nnz, out->blk_h, out->blk_w);
    if (!ws || ws_bytes < need)
        return fail(FTC_EWORKSPACE, "ftc_build_windows: workspace of %zu bytes needed, %zu given", need,
                    ws ? ws_bytes : static_cast<size_t>(0));
    if (reinterpret_cast<uintptr_t>(ws) % 256 != 0)
        return fail(FTC_EALIGN, "ftc_build_windows: workspace must be 256-byte aligned");
    if (side) {
        bool ok = side->fork != nullptr;
        for (int i = 0; i < 3; ++i) {
            ok = ok && side->stream[i] && side->join[i] && side->stream[i] != stream;
            for (int j = 0; j < i; ++j) ok = ok && side->stream[i] != side->stream[j] && side->join[i] != side->join[j];
            ok = ok && side->join[i] != side->fork;
        }
        if (!ok)
            return fail(FTC_EINVAL, "ftc_build_windows_concurrent: side needs three distinct streams other than `stream` and "
                                    "four distinct events");
    }
    return launch_build_windows(*g, *out, ws, ws_bytes, side, static_cast<hipStream_t>(stream));
}

int32_t ftc_build_windows(const ftc_csr *g, ftc_windows *out, void *ws, size_t ws_bytes, void *stream)
{
    return ftc_build_windows_concurrent(g, out, ws, ws_bytes, nullptr, stream);
}

int32_t ftc_gcn_norm(const ftc_csr *g, const ftc_windows *w, float *vals, float *dinv, void *stream)
{
    FTC_TRY(check_csr(g, "ftc_gcn_norm"));
    if (w) {
        FTC_TRY(check_windows(g, w, "ftc_gcn_norm", false));
        if (g->nnz > 0 && !w->edge_to_row) return fail(FTC_EINVAL, "ftc_gcn_norm: edge_to_row is NULL");
    }
    return launch_gcn_norm(*g, w, vals, dinv, static_cast<hipStream_t>(stream));
}

size_t ftc_spmm_workspace_bytes(int32_t n, int32_t nnz, int32_t D)
{
    if (n < 0 || nnz < 0 || D < 1) return 0;
    return spmm_seg_ws(nnz, D) + flag_bytes(n);
}

int32_t ftc_spmm(const ftc_csr *g, const ftc_windows *w, const float *vals, const void *X, int32_t ldx,
                 int32_t x_dtype, int32_t D, void *out, int32_t ldo, int32_t out_dtype, const float *out_scale,
                 int32_t relu, int32_t path, void *ws, size_t ws_bytes, void *stream)
{
    const Epi epi{relu, out_scale};
    FTC_TRY(check_csr(g, "ftc_spmm"));
    if (g->n == 0) return FTC_OK;
    FTC_TRY(check_dense(X, ldx, x_dtype, D, "ftc_spmm", "X"));
    FTC_TRY(check_dense(out, ldo, out_dtype, D, "ftc_spmm", "out"));
    if (out == X) return fail(FTC_EINVAL, "ftc_spmm: out aliases X");
    if (w) FTC_TRY(check_windows(g, w, "ftc_spmm", true));
    if (path != FTC_PATH_AUTO && path != FTC_PATH_VALU && path != FTC_PATH_MFMA)
        return fail(FTC_EINVAL, "ftc_spmm: unknown path %d", path);
    int vec, lpr;
    const bool rows16 = aligned16(X) && aligned16(out) &&
                        (static_cast<int64_t>(ldx) * elem_size(x_dtype)) % 16 == 0 &&
                        (static_cast<int64_t>(ldo) * elem_size(out_dtype)) % 16 == 0;
    const bool seg_ok = w && rows16 && seg_shape(x_dtype, D, &vec, &lpr);
    const bool mfma_ok = seg_ok && w->blk_h == 16 && mfma_shape_ok(x_dtype, D);
    if (path == FTC_PATH_MFMA && !mfma_ok)
        return fail(FTC_EUNSUPPORTED,
                    "ftc_spmm: the matrix-core path needs a window index with blk_h = 16, fp16/bf16 "
                    "features with D a multiple of 8 (<= 256) and 16-byte aligned rows");
    // a graph without entries only has its output rows cleared, whatever the path
    const bool can_seg = seg_ok && g->nnz > 0, can_mfma = mfma_ok && g->nnz > 0;
    if (can_seg) {
        const size_t need = ftc_spmm_workspace_bytes(g->n, g->nnz, D);
        if (!ws || ws_bytes < need)
            return fail(FTC_EWORKSPACE, "ftc_spmm: workspace of %zu bytes needed, %zu given", need,
                        ws ? ws_bytes : static_cast<size_t>(0));
        if (reinterpret_cast<uintptr_t>(ws) % 256 != 0)
            return fail(FTC_EALIGN, "ftc_spmm: workspace must be 256-byte aligned");
        hipStream_t hs = static_cast<hipStream_t>(stream);
        uint8_t *flags = nullptr;
        const float reuse = path == FTC_PATH_MFMA ? 0.f : spmm_mfma_reuse(D);
        if (can_mfma && path != FTC_PATH_VALU && reuse >= 0.f) {
            flags = reinterpret_cast<uint8_t *>(static_cast<char *>(ws) + spmm_seg_ws(g->nnz, D));
            FTC_TRY(launch_classify(*g, *w, reuse, MFMA_MAX_WINDOW_EDGES, flags, hs));
        }
        FTC_TRY(launch_spmm_seg(*g, *w, vals, X, ldx, x_dtype, D, out, ldo, out_dtype, epi, ws, flags, hs));
        if (flags) return launch_spmm_mfma(*g, *w, vals, X, ldx, x_dtype, D, out, ldo, out_dtype, epi, flags, hs);
        return FTC_OK;
    }
    return launch_spmm_rows(*g, vals, X, ldx, x_dtype, D, out, ldo, out_dtype, epi,
                            static_cast<hipStream_t>(stream));
}

// ftc_spmm for callers that can neither allocate nor hand over a workspace: the scratch memory of the
// aggregation kernels (carry rows of the cut rows, window flags) lives in this file-scope device array,
// one copy per GPU, held until the process ends.  In host code the array's name is only a stand-in; its
// device address is asked for once per device and kept.
}  // extern "C"
namespace {
constexpr size_t NOALLOC_SCRATCH_BYTES = static_cast<size_t>(FTC_NOALLOC_SCRATCH_MIB) << 20;
static __device__ __align__(256) unsigned char scratch[NOALLOC_SCRATCH_BYTES];
constexpr int NOALLOC_MAX_DEVICES = 64;
void *g_scratch_ptr[NOALLOC_MAX_DEVICES];  // device address of `scratch` on every device that has asked
std::mutex g_scratch_mutex;

int32_t scratch_of_current_device(void **ptr)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= NOALLOC_MAX_DEVICES) {
        (void)hipGetLastError();
        return fail(FTC_EHIP, "ftc_spmm_noalloc: no current device (or a device index beyond %d)", NOALLOC_MAX_DEVICES - 1);
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            (void)hipGetLastError();
            return fail(FTC_EHIP, "ftc_spmm_noalloc: hipGetSymbolAddress failed (%d: %s)", static_cast<int>(e),
                        hipGetErrorString(e));
        }
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return FTC_OK;
}
}  // namespace
extern "C" {

int32_t ftc_spmm_noalloc(const ftc_csr *g, const ftc_windows *w, const float *vals, const void *X, int32_t ldx,
                         int32_t x_dtype, int32_t D, void *out, int32_t ldo, int32_t out_dtype, const float *out_scale,
                         int32_t relu, int32_t path, void *stream)
{
    FTC_TRY(check_csr(g, "ftc_spmm_noalloc"));
    if (D < 1) return fail(FTC_EINVAL, "ftc_spmm_noalloc: need D >= 1");
    const size_t need = ftc_spmm_workspace_bytes(g->n, g->nnz, D);
    if (need > NOALLOC_SCRATCH_BYTES)
        return fail(FTC_EWORKSPACE,
                    "ftc_spmm_noalloc: this graph and width need %zu bytes of scratch memory, the built-in buffer holds "
                    "%zu; use ftc_spmm with a workspace",
                    need, NOALLOC_SCRATCH_BYTES);
    void *ptr = nullptr;
    FTC_TRY(scratch_of_current_device(&ptr));
    return ftc_spmm(g, w, vals, X, ldx, x_dtype, D, out, ldo, out_dtype, out_scale, relu, path, ptr, NOALLOC_SCRATCH_BYTES,
                    stream);
}

size_t ftc_sddmm_workspace_bytes(int32_t n, int32_t nnz, int32_t D)
{
    if (n < 0 || nnz < 0 || D < 1) return 0;
    // window flags of the per-window dispatch, then two arrays of inverse row norms (cosine mode on
    // the paths that do not recompute the norms from the rows)
    return align_up(flag_bytes(n), 256) + 2 * align_up(static_cast<size_t>(n) * sizeof(float), 256);
}

int32_t ftc_sddmm(const ftc_csr *g, const ftc_windows *w, const void *X, const void *Y, int32_t ld,
                  int32_t dtype, int32_t D, const float *row_scale, const float *col_scale, float alpha,
                  int32_t cosine, float *edge_out, int32_t path, void *ws, size_t ws_bytes, void *stream)
{
    FTC_TRY(check_csr(g, "ftc_sddmm"));
    if (g->n == 0 || g->nnz == 0) return FTC_OK;
    FTC_TRY(check_dense(X, ld, dtype, D, "ftc_sddmm", "X"));
    FTC_TRY(check_dense(Y, ld, dtype, D, "ftc_sddmm", "Y"));
    if (!edge_out) return fail(FTC_EINVAL, "ftc_sddmm: edge_out is NULL");
    if (cosine && (row_scale || col_scale))
        return fail(FTC_EINVAL, "ftc_sddmm: cosine mode takes no row_scale / col_scale");
    if (w) FTC_TRY(check_windows(g, w, "ftc_sddmm", true));
    if (path != FTC_PATH_AUTO && path != FTC_PATH_VALU && path != FTC_PATH_MFMA)
        return fail(FTC_EINVAL, "ftc_sddmm: unknown path %d", path);
    int vec, lpr;
    const bool can_edges = w && aligned16(X) && aligned16(Y) &&
                           (static_cast<int64_t>(ld) * elem_size(dtype)) % 16 == 0 && seg_shape(dtype, D, &vec, &lpr);
    const bool can_mfma = can_edges && w->blk_h == 16 && mfma_shape_ok(dtype, D);
    if (path == FTC_PATH_MFMA && !can_mfma)
        return fail(FTC_EUNSUPPORTED,
                    "ftc_sddmm: the matrix-core path needs a window index with blk_h = 16, fp16/bf16 "
                    "features with D a multiple of 8 (<= 256) and 16-byte aligned rows");
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const float reuse = path == FTC_PATH_MFMA ? 0.f : sddmm_mfma_reuse(D);
    const bool use_mfma = can_mfma && path != FTC_PATH_VALU && reuse >= 0.f;
    const bool need_ws = use_mfma || (cosine && !can_edges);
    if (need_ws) {
        const size_t need = ftc_sddmm_workspace_bytes(g->n, g->nnz, D);
        if (!ws || ws_bytes < need)
            return fail(FTC_EWORKSPACE, "ftc_sddmm: workspace of %zu bytes needed, %zu given", need,
                        ws ? ws_bytes : static_cast<size_t>(0));
        if (reinterpret_cast<uintptr_t>(ws) % 256 != 0)
            return fail(FTC_EALIGN, "ftc_sddmm: workspace must be 256-byte aligned");
    }
    // Cosine mode: the edge-parallel vector kernel recomputes the norms from the rows it holds; the
    // other kernels take them as scale arrays, which are produced here.
    if (cosine && (use_mfma || !can_edges)) {
        char *p = static_cast<char *>(ws) + align_up(flag_bytes(g->n), 256);
        float *rx = reinterpret_cast<float *>(p);
        float *ry = X == Y ? rx : reinterpret_cast<float *>(p + align_up(static_cast<size_t>(g->n) * sizeof(float), 256));
        FTC_TRY(launch_row_rnorm(g->n, X, ld, dtype, D, rx, hs));
        if (ry != rx) FTC_TRY(launch_row_rnorm(g->n, Y, ld, dtype, D, ry, hs));
        row_scale = rx;
        col_scale = ry;
    }
    if (can_edges) {
        uint8_t *flags = nullptr;
        if (use_mfma) {
            flags = static_cast<uint8_t *>(ws);
            FTC_TRY(launch_classify(*g, *w, reuse, MFMA_MAX_WINDOW_EDGES, flags, hs));
        }
        FTC_TRY(launch_sddmm_edges(*g, *w, X, Y, ld, dtype, D, row_scale, col_scale, alpha, edge_out, flags,
                                   cosine != 0, hs));
        if (flags)
            return launch_sddmm_mfma(*g, *w, X, Y, ld, dtype, D, row_scale, col_scale, alpha, edge_out, flags, hs);
        return FTC_OK;
    }
    return launch_sddmm_rows(*g, X, Y, ld, dtype, D, row_scale, col_scale, alpha, edge_out, hs);
}

int32_t ftc_row_rnorm(int32_t n, const void *H, int32_t ld, int32_t dtype, int32_t D, float *rinv,
                      void *stream)
{
    if (n < 0) return fail(FTC_EINVAL, "ftc_row_rnorm: negative n");
    if (n == 0) return FTC_OK;
    FTC_TRY(check_dense(H, ld, dtype, D, "ftc_row_rnorm", "H"));
    if (!rinv) return fail(FTC_EINVAL, "ftc_row_rnorm: rinv is NULL");
    return launch_row_rnorm(n, H, ld, dtype, D, rinv, static_cast<hipStream_t>(stream));
}

size_t ftc_edge_softmax_workspace_bytes(int32_t n, int32_t nnz)
{
    if (n < 0 || nnz < 0) return 0;
    return softmax_seg_ws(n, nnz);
}

int32_t ftc_edge_softmax(const ftc_csr *g, const ftc_windows *w, const float *e_in, float *p_out, void *ws,
                         size_t ws_bytes, void *stream)
{
    FTC_TRY(check_csr(g, "ftc_edge_softmax"));
    if (g->n == 0 || g->nnz == 0) return FTC_OK;
    if (!e_in || !p_out) return fail(FTC_EINVAL, "ftc_edge_softmax: NULL edge array");
    if (!w) return launch_softmax(*g, e_in, p_out, static_cast<hipStream_t>(stream));
    FTC_TRY(check_windows(g, w, "ftc_edge_softmax", false));
    if (!w->edge_to_row) return fail(FTC_EINVAL, "ftc_edge_softmax: edge_to_row is NULL");
    const size_t need = softmax_seg_ws(g->n, g->nnz);
    if (!ws || ws_bytes < need)
        return fail(FTC_EWORKSPACE, "ftc_edge_softmax: workspace of %zu bytes needed, %zu given", need,
                    ws ? ws_bytes : static_cast<size_t>(0));
    if (reinterpret_cast<uintptr_t>(ws) % 256 != 0)
        return fail(FTC_EALIGN, "ftc_edge_softmax: workspace must be 256-byte aligned");
    return launch_softmax_seg(*g, *w, e_in, p_out, ws, static_cast<hipStream_t>(stream));
}

int32_t ftc_update_gemm(int32_t n, const void *X, int32_t ldx, int32_t dtype, int32_t d_in, const void *W,
                        int32_t d_out, void *Z, int32_t ldz, int32_t z_dtype, const float *row_scale, int32_t relu,
                        void *stream)
{
    if (n < 0) return fail(FTC_EINVAL, "ftc_update_gemm: negative n");
    if (n == 0) return FTC_OK;
    FTC_TRY(check_dense(X, ldx, dtype, d_in, "ftc_update_gemm", "X"));
    FTC_TRY(check_dense(Z, ldz, z_dtype, d_out, "ftc_update_gemm", "Z"));
    if (!W) return fail(FTC_EINVAL, "ftc_update_gemm: W is NULL");
    if (Z == X) return fail(FTC_EINVAL, "ftc_update_gemm: Z aliases X");
    return launch_gemm(n, X, ldx, dtype, d_in, W, d_out, Z, ldz, z_dtype, Epi{relu, row_scale},
                       static_cast<hipStream_t>(stream));
}

// The intermediate Z = X * W: fp16 when the inputs are fp16 (halves the gathered bytes; its rounding,
// 2^-11 relative, stays far below the 16-bit tolerance), fp32 otherwise (a bf16 Z would round at
// 2^-9, the size of the tolerance itself).  Rows padded to 16 bytes.
static int z_dtype_for(int dtype) { return dtype == FTC_F16 ? FTC_F16 : FTC_F32; }
static int z_ld(int d_out, int zdt) { return zdt == FTC_F32 ? (d_out + 3) / 4 * 4 : (d_out + 7) / 8 * 8; }

size_t ftc_gcn_layer_workspace_bytes(int32_t n, int32_t nnz, int32_t d_in, int32_t d_out)
{
    (void)d_in;
    if (n < 0 || nnz < 0 || d_out < 1) return 0;
    // sized for the fp32 intermediate, which covers the fp16 one
    const int ldz = z_ld(d_out, FTC_F32);
    return align_up(static_cast<size_t>(n) * ldz * sizeof(float), 256) + ftc_spmm_workspace_bytes(n, nnz, d_out);
}

int32_t ftc_gcn_layer(const ftc_csr *g, const ftc_windows *w, const float *vals, const float *dinv,
                      const void *X, int32_t ldx, int32_t dtype, int32_t d_in, const void *W, int32_t d_out,
                      int32_t relu, void *out, int32_t ldo, int32_t out_dtype, int32_t path, void *ws,
                      size_t ws_bytes, void *stream)
{
    FTC_TRY(check_csr(g, "ftc_gcn_layer"));
    if (g->n == 0) return FTC_OK;
    const size_t need = ftc_gcn_layer_workspace_bytes(g->n, g->nnz, d_in, d_out);
    if (!ws || ws_bytes < need)
        return fail(FTC_EWORKSPACE, "ftc_gcn_layer: workspace of %zu bytes needed", need);
    if (reinterpret_cast<uintptr_t>(ws) % 256 != 0)
        return fail(FTC_EALIGN, "ftc_gcn_layer: workspace must be 256-byte aligned");
    if (!valid_dtype(dtype)) return fail(FTC_EUNSUPPORTED, "ftc_gcn_layer: unknown dtype");
    const int zdt = z_dtype_for(dtype);
    const int ldz = z_ld(d_out, zdt);
    void *Z = ws;
    const size_t zbytes = align_up(static_cast<size_t>(g->n) * z_ld(d_out, FTC_F32) * sizeof(float), 256);
    // factored normalisation: rows of X*W are scaled by dinv[j] as they are written, the aggregation
    // runs without edge values and scales output row i by dinv[i]
    FTC_TRY(ftc_update_gemm(g->n, X, ldx, dtype, d_in, W, d_out, Z, ldz, zdt, dinv, 0, stream));
    return ftc_spmm(g, w, dinv ? nullptr : vals, Z, ldz, zdt, d_out, out, ldo, out_dtype, dinv, relu, path,
                    static_cast<char *>(ws) + zbytes, ws_bytes - zbytes, stream);
}

static size_t agnn_unfused_bytes(int32_t n, int32_t nnz, int32_t D)
{
    return align_up(static_cast<size_t>(nnz) * sizeof(float), 256) +
           align_up(ftc_sddmm_workspace_bytes(n, nnz, D), 256) +
           align_up(ftc_edge_softmax_workspace_bytes(n, nnz), 256) + ftc_spmm_workspace_bytes(n, nnz, D);
}

size_t ftc_agnn_layer_workspace_bytes(int32_t n, int32_t nnz, int32_t D)
{
    if (n < 0 || nnz < 0 || D < 1) return 0;
    const size_t a = agnn_unfused_bytes(n, nnz, D), b = agnn_fused_ws(nnz, D);
    return a > b ? a : b;
}

int32_t ftc_agnn_layer(const ftc_csr *g, const ftc_windows *w, const void *H, int32_t ld, int32_t dtype,
                       int32_t D, float beta, void *out, int32_t ldo, int32_t out_dtype, float *edge_p, float *row_z,
                       float *out_f32, int32_t ld_f32, int32_t path, void *ws, size_t ws_bytes, void *stream)
{
    FTC_TRY(check_csr(g, "ftc_agnn_layer"));
    if (g->n == 0) return FTC_OK;
    FTC_TRY(check_dense(H, ld, dtype, D, "ftc_agnn_layer", "H"));
    FTC_TRY(check_dense(out, ldo, out_dtype, D, "ftc_agnn_layer", "out"));
    if (out == H) return fail(FTC_EINVAL, "ftc_agnn_layer: out aliases H");
    if (w) FTC_TRY(check_windows(g, w, "ftc_agnn_layer", true));
    const size_t need = ftc_agnn_layer_workspace_bytes(g->n, g->nnz, D);
    if (!ws || ws_bytes < need)
        return fail(FTC_EWORKSPACE, "ftc_agnn_layer: workspace of %zu bytes needed", need);
    if (reinterpret_cast<uintptr_t>(ws) % 256 != 0)
        return fail(FTC_EALIGN, "ftc_agnn_layer: workspace must be 256-byte aligned");
    char *p = static_cast<char *>(ws);

    // One pass over the edges when the probabilities are not asked for and the vector path applies.
    int vec, lpr;
    const bool rows16 = aligned16(H) && aligned16(out) && (static_cast<int64_t>(ld) * elem_size(dtype)) % 16 == 0 &&
                        (static_cast<int64_t>(ldo) * elem_size(out_dtype)) % 16 == 0;
    if (out_f32) {
        FTC_TRY(check_dense(out_f32, ld_f32, FTC_F32, D, "ftc_agnn_layer", "out_f32"));
        if (!aligned16(out_f32) || ld_f32 % 4 != 0)
            return fail(FTC_EALIGN, "ftc_agnn_layer: rows of out_f32 must be 16-byte aligned");
        if (static_cast<void *>(out_f32) == out || static_cast<const void *>(out_f32) == H)
            return fail(FTC_EINVAL, "ftc_agnn_layer: out_f32 aliases out or H");
    }
    const bool keep = row_z || out_f32;
    // the single pass shifts the softmax by |beta| instead of the row maximum: exp(-2 |beta|) must stay a
    // normal fp32 number; beyond that the chain with the row-wise softmax takes over
    const bool beta_ok = fabsf(beta) < AGNN_FUSED_MAX_BETA;
    if (!edge_p && w && beta_ok && (g->nnz > 0 || keep) && path != FTC_PATH_MFMA && rows16 &&
        seg_shape(dtype, D, &vec, &lpr))
        return launch_agnn_fused(*g, *w, H, ld, dtype, D, beta, out, ldo, out_dtype, row_z, out_f32, ld_f32, p,
                                 static_cast<hipStream_t>(stream));
    if (keep)
        return fail(FTC_EUNSUPPORTED,
                    "ftc_agnn_layer: |beta| < 43 is needed, and row_z and out_f32 come from the single-pass route only (window index, no edge_p, not "
                    "FTC_PATH_MFMA, 16-byte aligned rows, a width the edge-balanced kernels cover)");

    float *scores = edge_p ? edge_p : reinterpret_cast<float *>(p);
    p += align_up(static_cast<size_t>(g->nnz) * sizeof(float), 256);
    const size_t sd = align_up(ftc_sddmm_workspace_bytes(g->n, g->nnz, D), 256);
    void *ws_sddmm = p;
    p += sd;
    const size_t sm = align_up(ftc_edge_softmax_workspace_bytes(g->n, g->nnz), 256);
    void *ws_softmax = p;
    p += sm;
    const size_t rest = ws_bytes - static_cast<size_t>(p - static_cast<char *>(ws));
    FTC_TRY(ftc_sddmm(g, w, H, H, ld, dtype, D, nullptr, nullptr, beta, 1, scores, path, ws_sddmm, sd, stream));
    FTC_TRY(ftc_edge_softmax(g, w, scores, scores, ws_softmax, sm, stream));
    return ftc_spmm(g, w, scores, H, ld, dtype, D, out, ldo, out_dtype, nullptr, 0, path, p, rest, stream);
}

// ---------------------------------------------------------------------------------------------------
// Backward pass (gradients are fp32)

int32_t ftc_transpose_index(const ftc_csr *g, const ftc_windows *w, int32_t *T, int32_t *flag, void *stream)
{
    FTC_TRY(check_csr(g, "ftc_transpose_index"));
    if (!flag) return fail(FTC_EINVAL, "ftc_transpose_index: flag is NULL");
    if (g->nnz > 0 && !T) return fail(FTC_EINVAL, "ftc_transpose_index: T is NULL");
    const int32_t *e2r = nullptr;
    if (w) {
        FTC_TRY(check_windows(g, w, "ftc_transpose_index", false));
        e2r = w->edge_to_row;
    }
    return launch_transpose_index(*g, e2r, T, flag, static_cast<hipStream_t>(stream));
}

int32_t ftc_edge_softmax_backward(const ftc_csr *g, const ftc_windows *w, const float *p, const float *dp, float *ds,
                                  void *ws, size_t ws_bytes, void *stream)
{
    FTC_TRY(check_csr(g, "ftc_edge_softmax_backward"));
    if (g->n == 0 || g->nnz == 0) return FTC_OK;
    if (!p || !dp || !ds) return fail(FTC_EINVAL, "ftc_edge_softmax_backward: NULL edge array");
    if (!w) return launch_softmax_backward(*g, p, dp, ds, static_cast<hipStream_t>(stream));
    FTC_TRY(check_windows(g, w, "ftc_edge_softmax_backward", false));
    if (!w->edge_to_row) return fail(FTC_EINVAL, "ftc_edge_softmax_backward: edge_to_row is NULL");
    const size_t need = softmax_seg_ws(g->n, g->nnz);
    if (!ws || ws_bytes < need)
        return fail(FTC_EWORKSPACE, "ftc_edge_softmax_backward: workspace of %zu bytes needed, %zu given", need,
                    ws ? ws_bytes : static_cast<size_t>(0));
    if (reinterpret_cast<uintptr_t>(ws) % 256 != 0)
        return fail(FTC_EALIGN, "ftc_edge_softmax_backward: workspace must be 256-byte aligned");
    return launch_softmax_backward_seg(*g, *w, p, dp, ds, ws, static_cast<hipStream_t>(stream));
}

size_t ftc_weight_grad_workspace_bytes(int32_t n, int32_t d_in, int32_t d_out)
{
    if (n < 0 || d_in < 1 || d_out < 1) return 0;
    return weight_grad_ws(n, d_in, d_out);
}

int32_t ftc_weight_grad(int32_t n, const void *X, int32_t ldx, int32_t x_dtype, int32_t d_in, const float *G,
                        int32_t ldg, int32_t d_out, float *dW, void *ws, size_t ws_bytes, void *stream)
{
    if (n < 0) return fail(FTC_EINVAL, "ftc_weight_grad: negative n");
    FTC_TRY(check_dense(X, ldx, x_dtype, d_in, "ftc_weight_grad", "X"));
    FTC_TRY(check_dense(G, ldg, FTC_F32, d_out, "ftc_weight_grad", "G"));
    if (!dW) return fail(FTC_EINVAL, "ftc_weight_grad: dW is NULL");
    if (d_in < 1 || d_out < 1 || weight_grad_group(d_in, d_out) == 0)
        return fail(FTC_EUNSUPPORTED, "ftc_weight_grad: d_out too wide (8 input columns next to it must fit: d_out <= 504)");
    const size_t need = weight_grad_ws(n, d_in, d_out);
    if (!ws || ws_bytes < need) return fail(FTC_EWORKSPACE, "ftc_weight_grad: workspace of %zu bytes needed", need);
    return launch_weight_grad(n, X, ldx, x_dtype, d_in, G, ldg, d_out, dW, ws, static_cast<hipStream_t>(stream));
}

static int pad4(int d) { return (d + 3) / 4 * 4; }

size_t ftc_update_gemm_backward_workspace_bytes(int32_t n, int32_t d_in, int32_t d_out)
{
    if (n < 0 || d_in < 1 || d_out < 1) return 0;
    return align_up(static_cast<size_t>(n) * pad4(d_out) * sizeof(float), 256) + weight_grad_ws(n, d_in, d_out) +
           input_grad_ws(d_in, d_out);
}

int32_t ftc_update_gemm_backward(int32_t n, const void *X, int32_t ldx, int32_t dtype, int32_t d_in, const void *W,
                                 int32_t d_out, const void *Z, int32_t ldz, int32_t z_dtype, const float *dZ,
                                 int32_t lddz, void *dX, int32_t lddx, int32_t dx_dtype, float *dW, void *ws,
                                 size_t ws_bytes, void *stream)
{
    if (n < 0) return fail(FTC_EINVAL, "ftc_update_gemm_backward: negative n");
    if (n == 0) return FTC_OK;
    FTC_TRY(check_dense(X, ldx, dtype, d_in, "ftc_update_gemm_backward", "X"));
    FTC_TRY(check_dense(dZ, lddz, FTC_F32, d_out, "ftc_update_gemm_backward", "dZ"));
    if (Z) FTC_TRY(check_dense(Z, ldz, z_dtype, d_out, "ftc_update_gemm_backward", "Z"));
    if (dX) FTC_TRY(check_dense(dX, lddx, dx_dtype, d_in, "ftc_update_gemm_backward", "dX"));
    if (!W || !dW) return fail(FTC_EINVAL, "ftc_update_gemm_backward: W or dW is NULL");
    if (dX == X) return fail(FTC_EINVAL, "ftc_update_gemm_backward: dX aliases X");
    if (weight_grad_group(d_in, d_out) == 0) return fail(FTC_EUNSUPPORTED, "ftc_update_gemm_backward: need d_out <= 504");
    const size_t need = ftc_update_gemm_backward_workspace_bytes(n, d_in, d_out);
    if (!ws || ws_bytes < need)
        return fail(FTC_EWORKSPACE, "ftc_update_gemm_backward: workspace of %zu bytes needed", need);
    if (reinterpret_cast<uintptr_t>(ws) % 256 != 0)
        return fail(FTC_EALIGN, "ftc_update_gemm_backward: workspace must be 256-byte aligned");
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const float *dP = dZ;
    int ldp = lddz;
    char *p = static_cast<char *>(ws);
    if (Z) {  // ReLU: the gradient passes where the output was positive
        float *masked = reinterpret_cast<float *>(p);
        ldp = pad4(d_out);
        FTC_TRY(launch_mask_scale(n, d_out, dZ, lddz, Z, ldz, z_dtype, nullptr, masked, ldp, hs));
        dP = masked;
    }
    void *ws_wg = p + align_up(static_cast<size_t>(n) * pad4(d_out) * sizeof(float), 256);
    FTC_TRY(launch_weight_grad(n, X, ldx, dtype, d_in, dP, ldp, d_out, dW, ws_wg, hs));
    if (dX)
        FTC_TRY(launch_input_grad_any(n, dP, ldp, d_out, W, dtype, d_in, dX, lddx, dx_dtype,
                                      static_cast<char *>(ws_wg) + weight_grad_ws(n, d_in, d_out), hs));
    return FTC_OK;
}

size_t ftc_gcn_layer_backward_workspace_bytes(int32_t n, int32_t nnz, int32_t d_in, int32_t d_out)
{
    if (n < 0 || nnz < 0 || d_in < 1 || d_out < 1) return 0;
    const size_t mat = align_up(static_cast<size_t>(n) * pad4(d_out) * sizeof(float), 256);
    return 2 * mat + align_up(ftc_spmm_workspace_bytes(n, nnz, d_out), 256) + weight_grad_ws(n, d_in, d_out) +
           input_grad_ws(d_in, d_out);
}

int32_t ftc_gcn_layer_backward(const ftc_csr *gT, const ftc_windows *wT, const float *valsT, const float *dinv,
                               const void *X, int32_t ldx, int32_t dtype, int32_t d_in, const void *W, int32_t d_out,
                               const void *Y, int32_t ldy, int32_t y_dtype, const float *dY, int32_t lddy, float *dX,
                               int32_t lddx, float *dW, int32_t path, void *ws, size_t ws_bytes, void *stream)
{
    FTC_TRY(check_csr(gT, "ftc_gcn_layer_backward"));
    if (gT->n == 0) return FTC_OK;
    FTC_TRY(check_dense(X, ldx, dtype, d_in, "ftc_gcn_layer_backward", "X"));
    FTC_TRY(check_dense(dY, lddy, FTC_F32, d_out, "ftc_gcn_layer_backward", "dY"));
    if (Y) FTC_TRY(check_dense(Y, ldy, y_dtype, d_out, "ftc_gcn_layer_backward", "Y"));
    if (dX) FTC_TRY(check_dense(dX, lddx, FTC_F32, d_in, "ftc_gcn_layer_backward", "dX"));
    if (!W || !dW) return fail(FTC_EINVAL, "ftc_gcn_layer_backward: W or dW is NULL");
    if (weight_grad_group(d_in, d_out) == 0) return fail(FTC_EUNSUPPORTED, "ftc_gcn_layer_backward: need d_out <= 504");
    const size_t need = ftc_gcn_layer_backward_workspace_bytes(gT->n, gT->nnz, d_in, d_out);
    if (!ws || ws_bytes < need)
        return fail(FTC_EWORKSPACE, "ftc_gcn_layer_backward: workspace of %zu bytes needed", need);
    if (reinterpret_cast<uintptr_t>(ws) % 256 != 0)
        return fail(FTC_EALIGN, "ftc_gcn_layer_backward: workspace must be 256-byte aligned");
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const int n = gT->n, ldp = pad4(d_out);
    const size_t mat = align_up(static_cast<size_t>(n) * ldp * sizeof(float), 256);
    char *p = static_cast<char *>(ws);
    float *dP = reinterpret_cast<float *>(p);
    float *dZ = reinterpret_cast<float *>(p + mat);
    void *ws_spmm = p + 2 * mat;
    const size_t spmm_bytes = align_up(ftc_spmm_workspace_bytes(n, gT->nnz, d_out), 256);
    void *ws_wg = p + 2 * mat + spmm_bytes;
    // dP = dY where the output was positive, rows scaled by dinv in the factored form
    FTC_TRY(launch_mask_scale(n, d_out, dY, lddy, Y, ldy, y_dtype, dinv, dP, ldp, hs));
    // dZ = A^T dP on the transposed graph the caller hands over
    FTC_TRY(ftc_spmm(gT, wT, dinv ? nullptr : valsT, dP, ldp, FTC_F32, d_out, dZ, ldp, FTC_F32, dinv, 0, path,
                     ws_spmm, spmm_bytes, stream));
    FTC_TRY(launch_weight_grad(n, X, ldx, dtype, d_in, dZ, ldp, d_out, dW, ws_wg, hs));
    if (dX)
        FTC_TRY(launch_input_grad_any(n, dZ, ldp, d_out, W, dtype, d_in, dX, lddx, FTC_F32,
                                      static_cast<char *>(ws_wg) + weight_grad_ws(n, d_in, d_out), hs));
    return FTC_OK;
}

size_t ftc_agnn_layer_backward_workspace_bytes(int32_t n, int32_t nnz, int32_t D)
{
    if (n < 0 || nnz < 0 || D < 1) return 0;
    const size_t edge = align_up(static_cast<size_t>(nnz) * sizeof(float), 256);
    return 3 * edge + align_up(static_cast<size_t>(n) * sizeof(float), 256) +
           2 * align_up(static_cast<size_t>(n) * pad4(D) * sizeof(float), 256) +
           align_up(ftc_sddmm_workspace_bytes(n, nnz, D), 256) + align_up(ftc_spmm_workspace_bytes(n, nnz, D), 256) +
           align_up(softmax_seg_ws(n, nnz), 256) + edge_dot_ws();
}

int32_t ftc_agnn_layer_backward(const ftc_csr *g, const ftc_windows *w, const int32_t *T, const void *H, int32_t ld,
                                int32_t dtype, int32_t D, float beta, const float *p, const void *dY, int32_t lddy,
                                void *dH, int32_t lddh, int32_t dh_dtype, float *dbeta, int32_t path, void *ws,
                                size_t ws_bytes, void *stream)
{
    FTC_TRY(check_csr(g, "ftc_agnn_layer_backward"));
    if (g->n == 0) return FTC_OK;
    FTC_TRY(check_dense(H, ld, dtype, D, "ftc_agnn_layer_backward", "H"));
    FTC_TRY(check_dense(dY, lddy, dtype, D, "ftc_agnn_layer_backward", "dY"));
    FTC_TRY(check_dense(dH, lddh, dh_dtype, D, "ftc_agnn_layer_backward", "dH"));
    if (!dbeta) return fail(FTC_EINVAL, "ftc_agnn_layer_backward: dbeta is NULL");
    if (g->nnz > 0 && (!T || !p)) return fail(FTC_EINVAL, "ftc_agnn_layer_backward: T or p is NULL");
    if (dH == H || dH == dY) return fail(FTC_EINVAL, "ftc_agnn_layer_backward: dH aliases an input");
    if (ld != lddy) return fail(FTC_EINVAL, "ftc_agnn_layer_backward: H and dY need the same leading dimension");
    const size_t need = ftc_agnn_layer_backward_workspace_bytes(g->n, g->nnz, D);
    if (!ws || ws_bytes < need)
        return fail(FTC_EWORKSPACE, "ftc_agnn_layer_backward: workspace of %zu bytes needed", need);
    if (reinterpret_cast<uintptr_t>(ws) % 256 != 0)
        return fail(FTC_EALIGN, "ftc_agnn_layer_backward: workspace must be 256-byte aligned");
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const int n = g->n, nnz = g->nnz, ldq = pad4(D);
    const size_t edge = align_up(static_cast<size_t>(nnz) * sizeof(float), 256);
    char *q8 = static_cast<char *>(ws);
    float *c = reinterpret_cast<float *>(q8); q8 += edge;       // cosines
    float *ds = reinterpret_cast<float *>(q8); q8 += edge;      // dL/dp, then dL/ds
    float *v = reinterpret_cast<float *>(q8); q8 += edge;       // edge values of the two transposed products
    float *rinv = reinterpret_cast<float *>(q8); q8 += align_up(static_cast<size_t>(n) * sizeof(float), 256);
    float *q = reinterpret_cast<float *>(q8); q8 += align_up(static_cast<size_t>(n) * ldq * sizeof(float), 256);
    float *agg = reinterpret_cast<float *>(q8); q8 += align_up(static_cast<size_t>(n) * ldq * sizeof(float), 256);
    void *ws_sd = q8; const size_t sd = align_up(ftc_sddmm_workspace_bytes(n, nnz, D), 256); q8 += sd;
    void *ws_sp = q8; const size_t sp = align_up(ftc_spmm_workspace_bytes(n, nnz, D), 256); q8 += sp;
    void *ws_sm = q8; const size_t sm = align_up(softmax_seg_ws(n, nnz), 256); q8 += sm;
    void *ws_dot = q8;
    FTC_TRY(launch_row_rnorm(n, H, ld, dtype, D, rinv, hs));
    // c_e = cos(h_i, h_j);  dp_e = <dY_i, h_j>  (y_i = sum_e p_e h_j)
    FTC_TRY(ftc_sddmm(g, w, H, H, ld, dtype, D, nullptr, nullptr, 1.f, 1, c, path, ws_sd, sd, stream));
    FTC_TRY(ftc_sddmm(g, w, dY, H, ld, dtype, D, nullptr, nullptr, 1.f, 0, ds, path, ws_sd, sd, stream));
    FTC_TRY(ftc_edge_softmax_backward(g, w, p, ds, ds, ws_sm, sm, stream));
    FTC_TRY(launch_edge_dot(nnz, ds, c, dbeta, ws_dot, hs));  // s = beta * c, so dL/dbeta = sum_e ds_e c_e
    // gradient with respect to the normalised rows: q_i = sum_e (dc_e + dc_T(e)) hn_j, dc = beta * ds,
    // hn_j = rinv_j h_j folded into the edge values so that H itself is the gathered matrix
    FTC_TRY(launch_edge_combine(nnz, ds, T, 1.f, 1.f, beta, rinv, g->col_idx, v, hs));
    FTC_TRY(ftc_spmm(g, w, v, H, ld, dtype, D, q, ldq, FTC_F32, nullptr, 0, path, ws_sp, sp, stream));
    // through the aggregated rows: dH = P^T dY, (P^T)_e = p_T(e) on the symmetric pattern
    FTC_TRY(launch_edge_combine(nnz, p, T, 0.f, 1.f, 1.f, nullptr, g->col_idx, v, hs));
    FTC_TRY(ftc_spmm(g, w, v, dY, lddy, dtype, D, agg, ldq, FTC_F32, nullptr, 0, path, ws_sp, sp, stream));
    // ... plus the derivative of the normalisation, rounded once to the requested type
    return launch_cos_backward_rows(n, H, ld, dtype, D, rinv, q, ldq, agg, ldq, dH, lddh, dh_dtype, hs);
}

size_t ftc_agnn_layer_backward_fused_workspace_bytes(int32_t n, int32_t nnz, int32_t D)
{
    if (n < 0 || nnz < 0 || D < 1) return 0;
    return agnn_backward_fused_ws(n, nnz, D);
}

int32_t ftc_agnn_layer_backward_fused(const ftc_csr *g, const ftc_windows *w, const void *H, int32_t ld, int32_t dtype,
                                      int32_t D, float beta, const float *row_z, const void *Y, int32_t ldy,
                                      int32_t y_dtype, const void *dY, int32_t lddy, void *dH, int32_t lddh,
                                      int32_t dh_dtype, float *dbeta, const int32_t *pattern_flag, void *ws,
                                      size_t ws_bytes, void *stream)
{
    FTC_TRY(check_csr(g, "ftc_agnn_layer_backward_fused"));
    if (g->n == 0) return FTC_OK;
    FTC_TRY(check_dense(H, ld, dtype, D, "ftc_agnn_layer_backward_fused", "H"));
    FTC_TRY(check_dense(dY, lddy, dtype, D, "ftc_agnn_layer_backward_fused", "dY"));
    FTC_TRY(check_dense(Y, ldy, y_dtype, D, "ftc_agnn_layer_backward_fused", "Y"));
    FTC_TRY(check_dense(dH, lddh, dh_dtype, D, "ftc_agnn_layer_backward_fused", "dH"));
    if (!dbeta || !row_z) return fail(FTC_EINVAL, "ftc_agnn_layer_backward_fused: dbeta or row_z is NULL");
    if (dH == H || dH == dY || dH == Y) return fail(FTC_EINVAL, "ftc_agnn_layer_backward_fused: dH aliases an input");
    if (ld != lddy)
        return fail(FTC_EINVAL, "ftc_agnn_layer_backward_fused: H and dY need the same leading dimension");
    if (!w) return fail(FTC_EINVAL, "ftc_agnn_layer_backward_fused: the window index is required");
    FTC_TRY(check_windows(g, w, "ftc_agnn_layer_backward_fused", false));
    if (g->nnz > 0 && !w->edge_to_row) return fail(FTC_EINVAL, "ftc_agnn_layer_backward_fused: edge_to_row is NULL");
    const bool rows16 = aligned16(H) && aligned16(dY) && (static_cast<int64_t>(ld) * elem_size(dtype)) % 16 == 0;
    if (!rows16 || !agnn_backward_fused_shape(dtype, D) || !(fabsf(beta) < AGNN_FUSED_MAX_BETA))
        return fail(FTC_EUNSUPPORTED,
                    "ftc_agnn_layer_backward_fused: needs |beta| < 43, 16-byte aligned rows and a width the "
                    "edge-balanced kernels cover with 2 * D <= 256 padded slots; use ftc_agnn_layer_backward");
    const size_t need = agnn_backward_fused_ws(g->n, g->nnz, D);
    if (!ws || ws_bytes < need)
        return fail(FTC_EWORKSPACE, "ftc_agnn_layer_backward_fused: workspace of %zu bytes needed", need);
    if (reinterpret_cast<uintptr_t>(ws) % 256 != 0)
        return fail(FTC_EALIGN, "ftc_agnn_layer_backward_fused: workspace must be 256-byte aligned");
    FTC_TRY(launch_agnn_backward_fused(*g, *w, H, dY, ld, dtype, D, beta, row_z, Y, ldy, y_dtype, dH, lddh, dh_dtype,
                                       dbeta, ws, static_cast<hipStream_t>(stream)));
    if (pattern_flag)  // not a symmetric pattern: NaN instead of a gradient of nothing
        return launch_poison_if_flag(pattern_flag, g->n, D, dH, lddh, dh_dtype, dbeta, static_cast<hipStream_t>(stream));
    return FTC_OK;
}

// ---- locality reordering (preprocessing) ---------------------------------------------------------
size_t ftc_reorder_workspace_bytes(int32_t n, int32_t nnz)
{
    if (n < 0 || nnz < 0) return 0;
    return reorder_ws(n, nnz);
}

static int32_t check_reorder_ws(const char *who, int n, int nnz, void *ws, size_t ws_bytes)
{
    const size_t need = reorder_ws(n, nnz);
    if (!ws || ws_bytes < need) return fail(FTC_EWORKSPACE, "%s: workspace of %zu bytes needed", who, need);
    if (reinterpret_cast<uintptr_t>(ws) % 256 != 0) return fail(FTC_EALIGN, "%s: workspace must be 256-byte aligned", who);
    return FTC_OK;
}

int32_t ftc_degree_order(const ftc_csr *g, int32_t mode, int32_t *perm, int32_t *inv, void *ws, size_t ws_bytes,
                         void *stream)
{
    FTC_TRY(check_csr(g, "ftc_degree_order"));
    if (mode != FTC_ORDER_DEGREE && mode != FTC_ORDER_DEGREE_CLASSES)
        return fail(FTC_EINVAL, "ftc_degree_order: unknown mode %d", mode);
    if (g->n == 0) return FTC_OK;
    if (!perm || !inv) return fail(FTC_EINVAL, "ftc_degree_order: perm or inv is NULL");
    FTC_TRY(check_reorder_ws("ftc_degree_order", g->n, g->nnz, ws, ws_bytes));
    return launch_degree_order(*g, mode, perm, inv, ws, static_cast<hipStream_t>(stream));
}

int32_t ftc_order_by_key(int32_t n, const int32_t *keys, int32_t *perm, int32_t *inv, int32_t *flag, void *ws,
                         size_t ws_bytes, void *stream)
{
    if (n < 0) return fail(FTC_EINVAL, "ftc_order_by_key: negative n");
    if (!flag) return fail(FTC_EINVAL, "ftc_order_by_key: flag is NULL");
    if (n > 0 && (!keys || !perm || !inv)) return fail(FTC_EINVAL, "ftc_order_by_key: keys, perm or inv is NULL");
    FTC_TRY(check_reorder_ws("ftc_order_by_key", n, 0, ws, ws_bytes));
    return launch_order_by_key(n, keys, perm, inv, flag, ws, static_cast<hipStream_t>(stream));
}

int32_t ftc_label_propagation(const ftc_csr *g, int32_t rounds, int32_t *labels, void *ws, size_t ws_bytes, void *stream)
{
    FTC_TRY(check_csr(g, "ftc_label_propagation"));
    if (rounds < 0) return fail(FTC_EINVAL, "ftc_label_propagation: negative number of rounds");
    if (g->n == 0) return FTC_OK;
    if (!labels) return fail(FTC_EINVAL, "ftc_label_propagation: labels is NULL");
    FTC_TRY(check_reorder_ws("ftc_label_propagation", g->n, g->nnz, ws, ws_bytes));
    return launch_label_propagation(*g, rounds, labels, ws, static_cast<hipStream_t>(stream));
}

int32_t ftc_permute_graph(const ftc_csr *g, const int32_t *perm, const int32_t *inv, int32_t *row_ptr_out,
                          int32_t *col_idx_out, int32_t *flag, void *ws, size_t ws_bytes, void *stream)
{
    FTC_TRY(check_csr(g, "ftc_permute_graph"));
    if (!flag) return fail(FTC_EINVAL, "ftc_permute_graph: flag is NULL");
    if (!row_ptr_out) return fail(FTC_EINVAL, "ftc_permute_graph: row_ptr_out is NULL");
    if (g->n > 0 && (!perm || !inv)) return fail(FTC_EINVAL, "ftc_permute_graph: perm or inv is NULL");
    if (g->nnz > 0 && !col_idx_out) return fail(FTC_EINVAL, "ftc_permute_graph: col_idx_out is NULL");
    if (row_ptr_out == g->row_ptr || (col_idx_out && col_idx_out == g->col_idx))
        return fail(FTC_EINVAL, "ftc_permute_graph: the output aliases the input graph");
    FTC_TRY(check_reorder_ws("ftc_permute_graph", g->n, g->nnz, ws, ws_bytes));
    return launch_permute_graph(*g, perm, inv, row_ptr_out, col_idx_out, flag, ws, static_cast<hipStream_t>(stream));
}

int32_t ftc_permute_rows(int32_t n, const void *X, int32_t ldx, int32_t dtype, int32_t D, const int32_t *map, void *out,
                         int32_t ldo, void *stream)
{
    if (n < 0) return fail(FTC_EINVAL, "ftc_permute_rows: negative n");
    if (n == 0) return FTC_OK;
    FTC_TRY(check_dense(X, ldx, dtype, D, "ftc_permute_rows", "X"));
    FTC_TRY(check_dense(out, ldo, dtype, D, "ftc_permute_rows", "out"));
    if (!map) return fail(FTC_EINVAL, "ftc_permute_rows: map is NULL");
    if (out == X) return fail(FTC_EINVAL, "ftc_permute_rows: out aliases X");
    return launch_permute_rows(n, X, ldx, dtype, D, map, out, ldo, static_cast<hipStream_t>(stream));
}

// ---- per-graph plan --------------------------------------------------------------------------------
int32_t ftc_degree_stats(const ftc_csr *g, int64_t *stats, void *stream)
{
    FTC_TRY(check_csr(g, "ftc_degree_stats"));
    if (!stats) return fail(FTC_EINVAL, "ftc_degree_stats: stats is NULL");
    return launch_degree_stats(*g, stats, static_cast<hipStream_t>(stream));
}

// Thresholds of the plan, from measurements on the benchmark graphs (bench.py --reorder, --sweep):
// relabelling by degree class paid 5 to 17 % on the gather kernels of the graphs with skew 7.8, 9.3
// and 70 and nothing on those with skew 1.03 and 1.1; it cannot pay while the whole feature matrix
// fits the 4 MiB L2 of one XCD.  With flat degrees only a community ordering can help (block-model
// graph: -28 to -52 % after ten rounds of label propagation); whether the graph has communities is
// not visible in these statistics, so the plan proposes a trial.
static constexpr double PLAN_SKEW_MIN = 2.0;
static constexpr double PLAN_L2_BYTES = 4.0 * 1024 * 1024;

int32_t ftc_plan_graph(int32_t n, int32_t nnz, int64_t sum_deg_sq, int64_t sum_uniq, int32_t D, int32_t dtype,
                       ftc_plan *plan)
{
    if (!plan) return fail(FTC_EINVAL, "ftc_plan_graph: plan is NULL");
    if (n < 0 || nnz < 0 || D < 1 || !valid_dtype(dtype) || sum_deg_sq < 0 || sum_uniq < 0 || sum_uniq > nnz)
        return fail(FTC_EINVAL, "ftc_plan_graph: bad argument");
    plan->skew = nnz > 0 ? static_cast<double>(n) * static_cast<double>(sum_deg_sq) /
                               (static_cast<double>(nnz) * static_cast<double>(nnz))
                         : 0.0;
    plan->reuse = sum_uniq > 0 ? static_cast<double>(nnz) / static_cast<double>(sum_uniq) : 0.0;
    const double feature_bytes = static_cast<double>(n) * D * elem_size(dtype);
    plan->reorder = FTC_ORDER_NONE;
    if (feature_bytes > PLAN_L2_BYTES) {
        if (plan->skew >= PLAN_SKEW_MIN) plan->reorder = FTC_ORDER_DEGREE_CLASSES;
        else if (nnz >= 8.0 * n) plan->reorder = FTC_ORDER_COMMUNITIES;  // flat degrees: only communities can help
    }
    int vec, lpr;
    const bool seg = seg_shape(dtype, D, &vec, &lpr);
    plan->agnn_single_pass = seg ? 1 : 0;
    plan->agnn_backward_single_pass = agnn_backward_fused_shape(dtype, D) ? 1 : 0;
    // FTC_PATH_AUTO splits the windows between the two kernels only where the matrix cores can win
    plan->spmm_mfma_windows = (mfma_shape_ok(dtype, D) && spmm_mfma_reuse(D) >= 0.f) ? 1 : 0;
    plan->sddmm_mfma_windows = (mfma_shape_ok(dtype, D) && sddmm_mfma_reuse(D) >= 0.f) ? 1 : 0;
    plan->mfma_min_reuse = sddmm_mfma_reuse(D);
    return FTC_OK;
}

}  // extern "C"
