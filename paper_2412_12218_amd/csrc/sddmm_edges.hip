// Edge-parallel sparse edge feature computation (SDDMM, Section V.A) on the vector units.
//
// The output has one value per stored entry (`EdgeValList`), so equal numbers of EDGES per wave
// balance the work however skewed the rows are; edge_to_row of the window index gives each
// edge its row.  A wave stages the (column, row) pairs of SEG_R consecutive edges in LDS, groups
// of LPR lanes walk contiguous runs of them, SD_B edges at a time: SD_B independent gathers of
// Y rows in flight per lane, the X row is re-read only when the row changes.  Dot products are
// reduced inside the group with DPP lane shuffles, parked in LDS, and written back scaled
// (alpha * row_scale[i] * col_scale[j]) with fully coalesced stores.
#include "ftc_common.hpp"

namespace ftc {

constexpr int SD_R = 512;  // edges per wave
constexpr int SD_B = 4;    // edges per batch

bool seg_shape(int dtype, int D, int *vec, int *lpr);  // spmm_seg.hip: same lane layout

// COS: the scores are cosines: every dot product is divided by the Euclidean norms of its two rows
// (clamped at 1e-12), which are recomputed from the row slices that are in registers anyway (one more
// packed dot product and lane-group sum per edge) instead of being gathered, 4 bytes at a time,
// from arrays of inverse norms: on a graph without locality that gather moves a 64-byte sector per edge.
template <class T, int VEC, int LPR, bool COS>
__global__ __launch_bounds__(256) void sddmm_edges_kernel(int nnz, int n_ranges, const int *__restrict__ row_ptr,
                                                          const int *__restrict__ col_idx,
                                                          const int *__restrict__ edge_to_row,
                                                          const void *__restrict__ X,
                                                          const void *__restrict__ Y, int ld, int D,
                                                          const float *__restrict__ rs,
                                                          const float *__restrict__ cs, float alpha,
                                                          float *__restrict__ out,
                                                          const uint8_t *__restrict__ dense)
{
    constexpr int NG = 64 / LPR;
    constexpr int RUN = SD_R / NG;
    constexpr int RP = SD_R + NG;
    __shared__ int s_col_all[4][RP];
    __shared__ int s_row_all[4][RP];
    __shared__ float s_dot_all[4][RP];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int g = lane / LPR, sub = lane % LPR;
    int *s_col = s_col_all[wave];
    int *s_row = s_row_all[wave];
    float *s_dot = s_dot_all[wave];

    const int v = xcd_chunked_block(blockIdx.x, gridDim.x) * 4 + wave;
    const bool active = v < n_ranges;
    const int base = active ? v * SD_R : 0;
    const int n_valid = active ? min(SD_R, nnz - base) : 0;
    int rows[SD_R / 64];
    const bool from_starts = n_valid == SD_R && rows_from_starts<SD_R>(row_ptr, edge_to_row, base, lane, rows);
#pragma unroll
    for (int j = 0; j < SD_R / 64; ++j) {
        const int i = j * 64 + lane;
        if (i < n_valid) {
            const int p = i + i / RUN;
            const int er = from_starts ? rows[j] : edge_to_row[base + i];
            const bool skip = dense && dense[er >> 4];  // that window goes to the matrix cores
            s_col[p] = skip ? -1 : __builtin_nontemporal_load(col_idx + base + i);  // streamed once
            s_row[p] = skip ? -1 : er;
        }
    }
    __syncthreads();

    const int rs0 = g * RUN;
    const int re = min(rs0 + RUN, n_valid);
    const bool live = sub * VEC < D;
    RawVec<T, VEC> xi;  // slice of X[i,:] of the current row, as loaded
    zero_raw(xi);
    float ri = 0.f;     // COS: 1 / max(||X[i,:]||, 1e-12)
    int cur = -1;
    // every group runs the same number of batches so that the lane shuffles stay converged
    for (int b = rs0; b < rs0 + RUN; b += SD_B) {
        int c[SD_B], r[SD_B];
        bool need[SD_B];
        RawVec<T, VEC> y[SD_B], xs[SD_B];
#pragma unroll
        for (int k = 0; k < SD_B; ++k) {
            const bool ok = b + k < re;
            const int p = (ok ? b + k : 0) + (ok ? g : 0);
            c[k] = ok ? s_col[p] : -1;
            r[k] = ok ? s_row[p] : -1;
        }
        int prev = cur;
#pragma unroll
        for (int k = 0; k < SD_B; ++k) {
            need[k] = r[k] >= 0 && r[k] != prev;
            if (r[k] >= 0) prev = r[k];
        }
#pragma unroll
        for (int k = 0; k < SD_B; ++k) {
            if (c[k] >= 0 && live) load_raw<T, VEC>(Y, static_cast<int64_t>(c[k]) * ld + sub * VEC, y[k]);
            else zero_raw(y[k]);
            if (need[k] && live) load_raw<T, VEC>(X, static_cast<int64_t>(r[k]) * ld + sub * VEC, xs[k]);
            else zero_raw(xs[k]);
        }
#pragma unroll
        for (int k = 0; k < SD_B; ++k) {
            if (need[k]) {  // the group's lanes branch together
                xi = xs[k];
                if constexpr (COS) ri = __frsqrt_rn(fmaxf(group_sum_dpp<LPR>(dot_raw<T, VEC>(xi, xi, 0.f)), 1e-24f));
            }
            float d = group_sum_dpp<LPR>(dot_raw<T, VEC>(xi, y[k], 0.f));
            if constexpr (COS)
                d *= ri * __frsqrt_rn(fmaxf(group_sum_dpp<LPR>(dot_raw<T, VEC>(y[k], y[k], 0.f)), 1e-24f));
            if (sub == 0 && r[k] >= 0) s_dot[b + k + g] = d;
        }
        cur = prev;
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < SD_R / 64; ++j) {
        const int i = j * 64 + lane;
        const int pp = i + i / RUN;
        if (i < n_valid && s_col[pp] >= 0) {
            const int p = pp;
            const float scale = alpha * (rs ? rs[s_row[p]] : 1.f) * (cs ? cs[s_col[p]] : 1.f);
            __builtin_nontemporal_store(scale * s_dot[p], out + base + i);  // written once, not read here
        }
    }
}

template <class T>
static void launch_edges_t(int vec, int lpr, unsigned grid, hipStream_t s, int nnz, int n_ranges,
                           const ftc_csr &g, const int *e2r, const void *X, const void *Y, int ld, int D,
                           const float *rs, const float *cs, float alpha, float *out, const uint8_t *dense,
                           bool cosine)
{
    constexpr int VM = T::VEC;
#define FTC_SD(V, L)                                                                                           \
    do {                                                                                                       \
        if (cosine)                                                                                            \
            hipLaunchKernelGGL((sddmm_edges_kernel<T, V, L, true>), dim3(grid), dim3(256), 0, s, nnz, n_ranges, \
                               g.row_ptr, g.col_idx, e2r, X, Y, ld, D, nullptr, nullptr, alpha, out, dense);   \
        else                                                                                                   \
            hipLaunchKernelGGL((sddmm_edges_kernel<T, V, L, false>), dim3(grid), dim3(256), 0, s, nnz,         \
                               n_ranges, g.row_ptr, g.col_idx, e2r, X, Y, ld, D, rs, cs, alpha, out, dense);   \
    } while (0)
    if (vec == VM) {
        if (lpr == 4) FTC_SD(VM, 4);
        else if (lpr == 8) FTC_SD(VM, 8);
        else if (lpr == 16) FTC_SD(VM, 16);
        else FTC_SD(VM, 32);
    } else if (vec == VM / 2) {
        FTC_SD(VM / 2, 4);
    } else {
        FTC_SD(VM / 4, 4);
    }
#undef FTC_SD
}

// Caller has checked: window index present, seg_shape() accepts (dt, D), rows 16-byte aligned.
int32_t launch_sddmm_edges(const ftc_csr &g, const ftc_windows &w, const void *X, const void *Y, int ld, int dt,
                           int D, const float *rs, const float *cs, float alpha, float *out, const uint8_t *dense,
                           bool cosine, hipStream_t s)
{
    if (g.nnz == 0) return FTC_OK;
    int vec = 0, lpr = 0;
    seg_shape(dt, D, &vec, &lpr);
    const int n_ranges = ceil_div(g.nnz, SD_R);
    const unsigned grid = static_cast<unsigned>((n_ranges + 3) / 4);
    if (dt == FTC_F32)
        launch_edges_t<F32>(vec, lpr, grid, s, g.nnz, n_ranges, g, w.edge_to_row, X, Y, ld, D, rs, cs, alpha, out, dense, cosine);
    else if (dt == FTC_F16)
        launch_edges_t<F16>(vec, lpr, grid, s, g.nnz, n_ranges, g, w.edge_to_row, X, Y, ld, D, rs, cs, alpha, out, dense, cosine);
    else
        launch_edges_t<BF16>(vec, lpr, grid, s, g.nnz, n_ranges, g, w.edge_to_row, X, Y, ld, D, rs, cs, alpha,
                             out, dense, cosine);
    return launch_status("sddmm_edges");
}

}  // namespace ftc
