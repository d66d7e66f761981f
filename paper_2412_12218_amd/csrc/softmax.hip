// Edge softmax over the stored entries of each CSR row.  Row lengths range from 1 to tens of
// thousands (power-law graphs), so a workgroup takes 256 consecutive rows and treats them in
// three classes: short rows by one lane each, medium rows by one wave each, long rows by the
// whole workgroup.  Every row's reduction order depends only on its length, so results are
// reproducible from run to run.
#include "ftc_common.hpp"

namespace ftc {

constexpr int SM_SHORT = 16;    // <= : one lane per row
constexpr int SM_MEDIUM = 2048; // <= : one wave per row; above: the workgroup

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    return v;
}

__global__ __launch_bounds__(256) void edge_softmax_kernel(int n, const int *__restrict__ row_ptr,
                                                           const float *in, float *out)
{
    __shared__ int mid_rows[256];
    __shared__ int big_rows[256];
    __shared__ int n_mid, n_big;
    __shared__ float red[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) { n_mid = 0; n_big = 0; }
    __syncthreads();
    const int64_t row = static_cast<int64_t>(blockIdx.x) * 256 + tid;
    int e0 = 0, e1 = 0;
    if (row < n) { e0 = row_ptr[row]; e1 = row_ptr[row + 1]; }
    const int len = e1 - e0;
    if (len > 0 && len <= SM_SHORT) {
        float m = -INFINITY;
        for (int e = e0; e < e1; ++e) m = fmaxf(m, in[e]);
        float z = 0.f;
        for (int e = e0; e < e1; ++e) z += expf(in[e] - m);
        const float inv = 1.f / z;
        for (int e = e0; e < e1; ++e) out[e] = expf(in[e] - m) * inv;
    } else if (len > SM_SHORT && len <= SM_MEDIUM) {
        mid_rows[atomicAdd(&n_mid, 1)] = static_cast<int>(row);
    } else if (len > SM_MEDIUM) {
        big_rows[atomicAdd(&n_big, 1)] = static_cast<int>(row);
    }
    __syncthreads();
    const int nm = n_mid, nb = n_big;
    for (int i = wave; i < nm; i += 4) {
        const int r = mid_rows[i];
        const int a = row_ptr[r], b = row_ptr[r + 1];
        float m = -INFINITY;
        for (int e = a + lane; e < b; e += 64) m = fmaxf(m, in[e]);
        m = wave_max(m);
        float z = 0.f;
        for (int e = a + lane; e < b; e += 64) z += expf(in[e] - m);
        z = wave_sum(z);
        const float inv = 1.f / z;
        for (int e = a + lane; e < b; e += 64) out[e] = expf(in[e] - m) * inv;
    }
    for (int i = 0; i < nb; ++i) {  // nb is uniform over the workgroup
        const int r = big_rows[i];
        const int a = row_ptr[r], b = row_ptr[r + 1];
        float m = -INFINITY;
        for (int e = a + tid; e < b; e += 256) m = fmaxf(m, in[e]);
        m = wave_max(m);
        __syncthreads();
        if (lane == 0) red[wave] = m;
        __syncthreads();
        m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        float z = 0.f;
        for (int e = a + tid; e < b; e += 256) z += expf(in[e] - m);
        z = wave_sum(z);
        __syncthreads();
        if (lane == 0) red[wave] = z;
        __syncthreads();
        z = (red[0] + red[1]) + (red[2] + red[3]);
        const float inv = 1.f / z;
        for (int e = a + tid; e < b; e += 256) out[e] = expf(in[e] - m) * inv;
    }
}

int32_t launch_softmax(const ftc_csr &g, const float *in, float *out, hipStream_t s)
{
    if (g.n == 0 || g.nnz == 0) return FTC_OK;
    const unsigned grid = static_cast<unsigned>((static_cast<int64_t>(g.n) + 255) / 256);
    hipLaunchKernelGGL(edge_softmax_kernel, dim3(grid), dim3(256), 0, s, g.n, g.row_ptr, in, out);
    return launch_status("edge_softmax");
}

// ------------------------------------------------------------------------------------------------
// Edge-balanced variant for graphs with a window index (edge_to_row known for every edge).
//
//   1. stats kernel: a wave takes SMS_R consecutive edges, 64 at a time.  The pair
//      (running maximum m, sum of exp(s - m)) is an associative reduction, so a segmented
//      inclusive scan over the 64 lanes (segments = runs of equal row id, found with
//      edge_to_row) gives every row piece its pair.  Rows that end inside the wave's range and
//      did not start before it are final and go to stats[row]; the piece entering from the left
//      and the piece leaving to the right go to a carry buffer.
//   2. fix-up kernel: pieces of a row cut by range boundaries are combined in edge order.
//   3. apply kernel: p[e] = exp(s[e] - m[row]) / z[row], one thread per edge.
constexpr int SMS_R = 1024;

struct MZ {
    float m, z;
};

__device__ __forceinline__ MZ mz_combine(MZ a, MZ b)
{
    // exp of a non-positive number only; the larger maximum keeps its sum unscaled
    MZ r;
    if (a.m >= b.m) { r.m = a.m; r.z = a.z + b.z * __expf(b.m - a.m); }
    else { r.m = b.m; r.z = b.z + a.z * __expf(a.m - b.m); }
    return r;
}

__global__ __launch_bounds__(256) void softmax_stats_kernel(int nnz, int n_ranges,
                                                            const int *__restrict__ edge_to_row,
                                                            const float *__restrict__ in,
                                                            float2 *__restrict__ stats,
                                                            float2 *__restrict__ carry,  // [n_ranges][2]
                                                            int *__restrict__ carry_tail_row)
{
    const int lane = threadIdx.x & 63;
    const int v = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (v >= n_ranges) return;  // no workgroup barrier below
    const int base = v * SMS_R;
    const int n_valid = min(SMS_R, nnz - base);
    const int prev_row = base > 0 ? edge_to_row[base - 1] : -1;
    // the open piece carried from chunk to chunk (same value in every lane)
    MZ cmz = {-INFINITY, 0.f};
    int crow = -1;
    for (int c0 = 0; c0 < n_valid; c0 += 64) {
        const int i = c0 + lane;
        const bool ok = i < n_valid;
        const int row = ok ? edge_to_row[base + i] : -2 - lane;  // distinct ids for the padding lanes
        MZ x = {ok ? in[base + i] : -INFINITY, ok ? 1.f : 0.f};
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            MZ y;
            y.m = __shfl_up(x.m, d, 64);
            y.z = __shfl_up(x.z, d, 64);
            const int yr = __shfl_up(row, d, 64);
            if (lane >= d && yr == row) x = mz_combine(y, x);
        }
        const int first_row = __shfl(row, 0, 64);
        if (crow >= 0) {
            if (row == crow) {
                x = mz_combine(cmz, x);  // lanes of the first segment continue the carried piece
            } else if (first_row != crow && lane == 0) {
                // the carried piece ended exactly at the chunk boundary
                if (crow == prev_row) carry[2 * static_cast<size_t>(v)] = make_float2(cmz.m, cmz.z);
                else stats[crow] = make_float2(cmz.m, cmz.z);
            }
        }
        const int last_lane = min(63, n_valid - c0 - 1);
        const int next_row = __shfl_down(row, 1, 64);
        if (ok && lane < last_lane && next_row != row) {  // a piece that ends inside the chunk
            if (row == prev_row) carry[2 * static_cast<size_t>(v)] = make_float2(x.m, x.z);
            else stats[row] = make_float2(x.m, x.z);
        }
        crow = __shfl(row, last_lane, 64);
        cmz.m = __shfl(x.m, last_lane, 64);
        cmz.z = __shfl(x.z, last_lane, 64);
    }
    if (lane == 0) {
        const bool right_open = base + n_valid < nnz && edge_to_row[base + n_valid] == crow;
        int tail = -1;
        if (crow == prev_row) {
            carry[2 * static_cast<size_t>(v)] = make_float2(cmz.m, cmz.z);  // closed or spanning the range
        } else if (right_open) {
            carry[2 * static_cast<size_t>(v) + 1] = make_float2(cmz.m, cmz.z);
            tail = crow;
        } else {
            stats[crow] = make_float2(cmz.m, cmz.z);
        }
        carry_tail_row[v] = tail;
    }
}

__global__ __launch_bounds__(256) void softmax_fixup_kernel(int n_ranges, const int *__restrict__ row_ptr,
                                                            const float2 *__restrict__ carry,
                                                            const int *__restrict__ carry_tail_row,
                                                            float2 *__restrict__ stats)
{
    const int v = blockIdx.x * 256 + threadIdx.x;
    if (v >= n_ranges) return;
    const int r = carry_tail_row[v];
    if (r < 0) return;
    const int last = (row_ptr[r + 1] - 1) / SMS_R;
    float2 t = carry[2 * static_cast<size_t>(v) + 1];
    MZ acc = {t.x, t.y};
    for (int u = v + 1; u <= last; ++u) {
        t = carry[2 * static_cast<size_t>(u)];
        acc = mz_combine(acc, MZ{t.x, t.y});
    }
    stats[r] = make_float2(acc.m, acc.z);
}

__global__ __launch_bounds__(256) void softmax_apply_kernel(int nnz, const int *__restrict__ edge_to_row,
                                                            const float2 *__restrict__ stats, const float *in,
                                                            float *out)
{
    const int64_t e = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (e >= nnz) return;
    const float2 st = stats[edge_to_row[e]];
    out[e] = expf(in[e] - st.x) / st.y;
}

size_t softmax_seg_ws(int n, int nnz)
{
    const size_t n_ranges = (static_cast<size_t>(nnz) + SMS_R - 1) / SMS_R;
    return align_up(static_cast<size_t>(n) * sizeof(float2), 256) + align_up(n_ranges * 2 * sizeof(float2), 256) +
           align_up(n_ranges * sizeof(int), 256);
}

int32_t launch_softmax_seg(const ftc_csr &g, const ftc_windows &w, const float *in, float *out, void *ws,
                           hipStream_t s)
{
    if (g.n == 0 || g.nnz == 0) return FTC_OK;
    const int n_ranges = (g.nnz + SMS_R - 1) / SMS_R;
    char *p = static_cast<char *>(ws);
    float2 *stats = reinterpret_cast<float2 *>(p);
    p += align_up(static_cast<size_t>(g.n) * sizeof(float2), 256);
    float2 *carry = reinterpret_cast<float2 *>(p);
    p += align_up(static_cast<size_t>(n_ranges) * 2 * sizeof(float2), 256);
    int *tail_row = reinterpret_cast<int *>(p);
    hipLaunchKernelGGL(softmax_stats_kernel, dim3((n_ranges + 3) / 4), dim3(256), 0, s, g.nnz, n_ranges,
                       w.edge_to_row, in, stats, carry, tail_row);
    int32_t st = launch_status("edge_softmax stats");
    if (st != FTC_OK) return st;
    hipLaunchKernelGGL(softmax_fixup_kernel, dim3((n_ranges + 255) / 256), dim3(256), 0, s, n_ranges, g.row_ptr,
                       carry, tail_row, stats);
    st = launch_status("edge_softmax fixup");
    if (st != FTC_OK) return st;
    hipLaunchKernelGGL(softmax_apply_kernel, dim3((g.nnz + 255) / 256), dim3(256), 0, s, g.nnz, w.edge_to_row,
                       stats, in, out);
    return launch_status("edge_softmax apply");
}

// ------------------------------------------------------------------------------------------------
// Inverse row norms for the AGNN cosine: a group of LPR lanes per row.
template <class T, int LPR>
__global__ __launch_bounds__(256) void row_rnorm_kernel(int n, const void *__restrict__ H, int ld, int D,
                                                        float *__restrict__ rinv)
{
    constexpr int V = T::VEC;
    constexpr int GROUPS = 256 / LPR;
    const int sub = threadIdx.x % LPR;
    const int64_t row = static_cast<int64_t>(blockIdx.x) * GROUPS + threadIdx.x / LPR;
    float q = 0.f;
    if (row < n && sub * V < D) {
        float h[V];
        load_vec<T>(H, row * ld + sub * V, h);
#pragma unroll
        for (int k = 0; k < V; ++k) q = fmaf(h[k], h[k], q);
    }
#pragma unroll
    for (int m = LPR / 2; m >= 1; m >>= 1) q += __shfl_xor(q, m, 64);
    if (row < n && sub == 0) rinv[row] = 1.f / fmaxf(sqrtf(q), 1e-12f);
}

__global__ __launch_bounds__(256) void row_rnorm_generic_kernel(int n, const void *H, int ld, int dt, int D,
                                                                float *rinv)
{
    const int64_t row = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (row >= n) return;
    float q = 0.f;
    for (int k = 0; k < D; ++k) {
        const float h = load_elem(H, row * ld + k, dt);
        q = fmaf(h, h, q);
    }
    rinv[row] = 1.f / fmaxf(sqrtf(q), 1e-12f);
}

template <class T>
static void rnorm_t(int lpr, int n, const void *H, int ld, int D, float *rinv, hipStream_t s)
{
#define FTC_CASE(L)                                                                                    \
    case L: {                                                                                          \
        const unsigned grid = static_cast<unsigned>((static_cast<int64_t>(n) + 256 / L - 1) / (256 / L)); \
        hipLaunchKernelGGL((row_rnorm_kernel<T, L>), dim3(grid), dim3(256), 0, s, n, H, ld, D, rinv);  \
    } break;
    switch (lpr) {
        FTC_CASE(1)
        FTC_CASE(2)
        FTC_CASE(4)
        FTC_CASE(8)
        FTC_CASE(16)
        FTC_CASE(32)
    }
#undef FTC_CASE
}

int32_t launch_row_rnorm(int n, const void *H, int ld, int dt, int D, float *rinv, hipStream_t s)
{
    if (n == 0) return FTC_OK;
    const int v = dt == FTC_F32 ? 4 : 8;
    if (aligned16(H) && (static_cast<int64_t>(ld) * elem_size(dt)) % 16 == 0 && D % v == 0 && D / v <= 32) {
        int lpr = 1;
        while (lpr * v < D) lpr *= 2;
        if (dt == FTC_F32) rnorm_t<F32>(lpr, n, H, ld, D, rinv, s);
        else if (dt == FTC_F16) rnorm_t<F16>(lpr, n, H, ld, D, rinv, s);
        else rnorm_t<BF16>(lpr, n, H, ld, D, rinv, s);
    } else {
        hipLaunchKernelGGL(row_rnorm_generic_kernel, dim3((n + 255) / 256), dim3(256), 0, s, n, H, ld, dt, D,
                           rinv);
    }
    return launch_status("row_rnorm");
}

}  // namespace ftc
