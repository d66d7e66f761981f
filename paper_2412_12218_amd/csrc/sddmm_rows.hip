// Row-oriented SDDMM on the plain CSR: a group of LPR lanes owns one row i, keeps its slice of
// X[i,:] in registers and visits the stored entries (i, j), gathering Y[j,:] and reducing the
// partial dot products inside the group.  Output has the layout of col_idx (`EdgeValList`,
// Section V.A, sparse edge feature computation).
#include "ftc_common.hpp"

namespace ftc {

template <int LPR>
__device__ __forceinline__ float group_sum(float v)
{
#pragma unroll
    for (int m = LPR / 2; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    return v;
}

template <class T, int LPR>
__global__ __launch_bounds__(256) void sddmm_rows_kernel(int n, const int *__restrict__ row_ptr,
                                                         const int *__restrict__ col_idx,
                                                         const void *__restrict__ X,
                                                         const void *__restrict__ Y, int ld, int D,
                                                         const float *__restrict__ rs,
                                                         const float *__restrict__ cs, float alpha,
                                                         float *__restrict__ out)
{
    constexpr int V = T::VEC;
    constexpr int GROUPS = 256 / LPR;
    const int sub = threadIdx.x % LPR;
    const int grp = threadIdx.x / LPR;
    int64_t row = static_cast<int64_t>(blockIdx.x) * GROUPS + grp;
    // keep whole waves alive for the shuffles: out-of-range groups work on an empty row
    const bool in_range = row < n;
    if (!in_range) row = 0;
    const bool live = sub * V < D;
    const int e0 = in_range ? row_ptr[row] : 0, e1 = in_range ? row_ptr[row + 1] : 0;
    float xi[V];
#pragma unroll
    for (int k = 0; k < V; ++k) xi[k] = 0.f;
    if (live && in_range) load_vec<T>(X, row * ld + sub * V, xi);
    const float ri = (rs && in_range) ? rs[row] : 1.f;
    // all lanes of a wave iterate to the longest row of the wave so the shuffles stay converged
    int len = e1 - e0, maxlen = len;
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) maxlen = max(maxlen, __shfl_xor(maxlen, m, 64));
    for (int t = 0; t < maxlen; ++t) {
        const bool act = t < len;
        const int j = act ? col_idx[e0 + t] : 0;
        float y[V];
#pragma unroll
        for (int k = 0; k < V; ++k) y[k] = 0.f;
        if (act && live) load_vec<T>(Y, static_cast<int64_t>(j) * ld + sub * V, y);
        float d = 0.f;
#pragma unroll
        for (int k = 0; k < V; ++k) d = fmaf(xi[k], y[k], d);
        d = group_sum<LPR>(d);
        if (act && sub == 0) out[e0 + t] = alpha * ri * (cs ? cs[j] : 1.f) * d;
    }
}

__global__ __launch_bounds__(256) void sddmm_generic_kernel(int n, const int *__restrict__ row_ptr,
                                                            const int *__restrict__ col_idx, const void *X,
                                                            const void *Y, int ld, int dt, int D,
                                                            const float *rs, const float *cs, float alpha,
                                                            float *out)
{
    const int64_t row = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (row >= n) return;
    for (int e = row_ptr[row]; e < row_ptr[row + 1]; ++e) {
        const int j = col_idx[e];
        float d = 0.f;
        for (int k = 0; k < D; ++k)
            d = fmaf(load_elem(X, row * ld + k, dt), load_elem(Y, static_cast<int64_t>(j) * ld + k, dt), d);
        out[e] = alpha * (rs ? rs[row] : 1.f) * (cs ? cs[j] : 1.f) * d;
    }
}

template <class T>
static void launch_t(int lpr, const ftc_csr &g, const void *X, const void *Y, int ld, int D, const float *rs,
                     const float *cs, float alpha, float *out, hipStream_t s)
{
#define FTC_CASE(L)                                                                                  \
    case L: {                                                                                        \
        const int groups = 256 / L;                                                                  \
        const unsigned grid = static_cast<unsigned>((static_cast<int64_t>(g.n) + groups - 1) / groups); \
        hipLaunchKernelGGL((sddmm_rows_kernel<T, L>), dim3(grid), dim3(256), 0, s, g.n, g.row_ptr,   \
                           g.col_idx, X, Y, ld, D, rs, cs, alpha, out);                             \
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

int32_t launch_sddmm_rows(const ftc_csr &g, const void *X, const void *Y, int ld, int dt, int D,
                          const float *rs, const float *cs, float alpha, float *out, hipStream_t s)
{
    if (g.n == 0 || g.nnz == 0) return FTC_OK;
    const int v = dt == FTC_F32 ? 4 : 8;
    const bool vec = aligned16(X) && aligned16(Y) && (static_cast<int64_t>(ld) * elem_size(dt)) % 16 == 0 &&
                     D % v == 0 && D / v <= 32;
    if (vec) {
        int lpr = 1;
        while (lpr * v < D) lpr *= 2;
        if (dt == FTC_F32) launch_t<F32>(lpr, g, X, Y, ld, D, rs, cs, alpha, out, s);
        else if (dt == FTC_F16) launch_t<F16>(lpr, g, X, Y, ld, D, rs, cs, alpha, out, s);
        else launch_t<BF16>(lpr, g, X, Y, ld, D, rs, cs, alpha, out, s);
    } else {
        const unsigned grid = static_cast<unsigned>((static_cast<int64_t>(g.n) + 255) / 256);
        hipLaunchKernelGGL(sddmm_generic_kernel, dim3(grid), dim3(256), 0, s, g.n, g.row_ptr, g.col_idx, X, Y,
                           ld, dt, D, rs, cs, alpha, out);
    }
    return launch_status("sddmm_rows");
}

}  // namespace ftc
