// GCN edge values A^_ij = (d~_i d~_j)^-1/2 for a pattern that already holds the self-loops,
// and a device-side CSR validity check.
#include "ftc_common.hpp"

namespace ftc {

__device__ __forceinline__ float inv_sqrt_deg(const int *row_ptr, int r)
{
    const int d = row_ptr[r + 1] - row_ptr[r];
    return d > 0 ? 1.f / sqrtf(static_cast<float>(d)) : 0.f;
}

__global__ __launch_bounds__(256) void dinv_kernel(int n, const int *__restrict__ row_ptr,
                                                   float *__restrict__ dinv)
{
    const int64_t r = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (r < n) dinv[r] = inv_sqrt_deg(row_ptr, static_cast<int>(r));
}

// One thread per edge; the row of an edge comes from the window index.
__global__ __launch_bounds__(256) void gcn_vals_edges_kernel(int nnz, const int *__restrict__ row_ptr,
                                                             const int *__restrict__ col_idx,
                                                             const int *__restrict__ edge_to_row,
                                                             float *__restrict__ vals)
{
    const int64_t e = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (e >= nnz) return;
    vals[e] = inv_sqrt_deg(row_ptr, edge_to_row[e]) * inv_sqrt_deg(row_ptr, col_idx[e]);
}

// Same with the per-node factors already in memory: one 4-byte gather per endpoint.
__global__ __launch_bounds__(256) void gcn_vals_edges_dinv_kernel(int nnz, const int *__restrict__ col_idx,
                                                                  const int *__restrict__ edge_to_row,
                                                                  const float *__restrict__ dinv,
                                                                  float *__restrict__ vals)
{
    const int64_t e = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (e >= nnz) return;
    vals[e] = dinv[edge_to_row[e]] * dinv[col_idx[e]];
}

// Without a window index: 16 lanes per row.
__global__ __launch_bounds__(256) void gcn_vals_rows_kernel(int n, const int *__restrict__ row_ptr,
                                                            const int *__restrict__ col_idx,
                                                            float *__restrict__ vals)
{
    const int sub = threadIdx.x & 15;
    const int64_t r = static_cast<int64_t>(blockIdx.x) * 16 + (threadIdx.x >> 4);
    if (r >= n) return;
    const float di = inv_sqrt_deg(row_ptr, static_cast<int>(r));
    for (int e = row_ptr[r] + sub; e < row_ptr[r + 1]; e += 16) vals[e] = di * inv_sqrt_deg(row_ptr, col_idx[e]);
}

int32_t launch_gcn_norm(const ftc_csr &g, const ftc_windows *w, float *vals, float *dinv, hipStream_t s)
{
    if (g.n == 0) return FTC_OK;
    if (dinv) {
        hipLaunchKernelGGL(dinv_kernel, dim3((g.n + 255) / 256), dim3(256), 0, s, g.n, g.row_ptr, dinv);
        const int32_t st = launch_status("gcn_norm dinv");
        if (st != FTC_OK) return st;
    }
    if (vals && g.nnz > 0) {
        if (w && dinv) {
            hipLaunchKernelGGL(gcn_vals_edges_dinv_kernel, dim3(ceil_div(g.nnz, 256)), dim3(256), 0, s, g.nnz,
                               g.col_idx, w->edge_to_row, dinv, vals);
        } else if (w) {
            hipLaunchKernelGGL(gcn_vals_edges_kernel, dim3(ceil_div(g.nnz, 256)), dim3(256), 0, s, g.nnz,
                               g.row_ptr, g.col_idx, w->edge_to_row, vals);
        } else {
            hipLaunchKernelGGL(gcn_vals_rows_kernel, dim3((g.n + 15) / 16), dim3(256), 0, s, g.n, g.row_ptr,
                               g.col_idx, vals);
        }
        return launch_status("gcn_norm vals");
    }
    return FTC_OK;
}

// ------------------------------------------------------------------------------------------------
__global__ void clear_flag_kernel(int32_t *flag) { *flag = 0; }

__global__ __launch_bounds__(256) void validate_kernel(int n, int nnz, const int *__restrict__ row_ptr,
                                                       const int *__restrict__ col_idx, int32_t *flag)
{
    const int64_t t = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    int bad = 0;
    if (t < n && row_ptr[t] > row_ptr[t + 1]) bad |= 1;
    if (t == 0 && (row_ptr[0] != 0 || row_ptr[n] != nnz)) bad |= 1;
    if (t <= n && (row_ptr[t] < 0 || row_ptr[t] > nnz)) bad |= 1;
    if (t < nnz && (col_idx[t] < 0 || col_idx[t] >= n)) bad |= 2;
    if (bad) atomicOr(flag, bad);
}

int32_t launch_validate(const ftc_csr &g, int32_t *flag, hipStream_t s)
{
    hipLaunchKernelGGL(clear_flag_kernel, dim3(1), dim3(1), 0, s, flag);
    const int64_t m = (g.n + 1 > g.nnz ? g.n + 1 : g.nnz);
    hipLaunchKernelGGL(validate_kernel, dim3(static_cast<unsigned>((m + 255) / 256)), dim3(256), 0, s, g.n,
                       g.nnz, g.row_ptr, g.col_idx, flag);
    return launch_status("validate_csr");
}

}  // namespace ftc
