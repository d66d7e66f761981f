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
