// Row-oriented SpMM on the plain CSR (no window index needed): a group of LPR lanes owns one
// output row and walks its stored entries, every lane holding one 16-byte slice of the
// feature row.  This is the definition C = A x B of Section I.A.2 evaluated row by row; it is
// the path taken when the caller has no window index, and the reference the balanced
// segmented kernels are compared with.
#include "ftc_common.hpp"

namespace ftc {

template <class T, int LPR>
__global__ __launch_bounds__(256) void spmm_rows_kernel(int n, const int *__restrict__ row_ptr,
                                                        const int *__restrict__ col_idx,
                                                        const float *__restrict__ vals,
                                                        const void *__restrict__ X, int ldx, int D,
                                                        void *__restrict__ out, int ldo, int odt, Epi epi)
{
    constexpr int V = T::VEC;
    constexpr int GROUPS = 256 / LPR;
    const int sub = threadIdx.x % LPR;
    const int grp = threadIdx.x / LPR;
    const int64_t row = static_cast<int64_t>(blockIdx.x) * GROUPS + grp;
    if (row >= n) return;
    const bool live = sub * V < D;  // D may be smaller than LPR * V (D = 24, 40, ...)
    const int e0 = row_ptr[row], e1 = row_ptr[row + 1];
    float acc[V];
#pragma unroll
    for (int k = 0; k < V; ++k) acc[k] = 0.f;
    if (live) {
        int e = e0;
        for (; e + 4 <= e1; e += 4) {
            int c[4];
            float a[4];
            float x[4][V];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                c[u] = col_idx[e + u];
                a[u] = vals ? vals[e + u] : 1.f;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) load_vec<T>(X, static_cast<int64_t>(c[u]) * ldx + sub * V, x[u]);
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int k = 0; k < V; ++k) acc[k] = fmaf(a[u], x[u][k], acc[k]);
        }
        for (; e < e1; ++e) {
            float x[V];
            const float a = vals ? vals[e] : 1.f;
            load_vec<T>(X, static_cast<int64_t>(col_idx[e]) * ldx + sub * V, x);
#pragma unroll
            for (int k = 0; k < V; ++k) acc[k] = fmaf(a, x[k], acc[k]);
        }
        const float f = epi.factor(row);
#pragma unroll
        for (int k = 0; k < V; ++k) acc[k] = epi.apply(f, acc[k]);
        store_vec<V>(out, row * ldo + sub * V, odt, acc);
    }
}

// Any D, any alignment: one thread per output element.
__global__ __launch_bounds__(256) void spmm_generic_kernel(int n, const int *__restrict__ row_ptr,
                                                           const int *__restrict__ col_idx,
                                                           const float *__restrict__ vals, const void *X,
                                                           int ldx, int xdt, int D, void *out, int ldo,
                                                           int odt, Epi epi)
{
    const int64_t t = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (t >= static_cast<int64_t>(n) * D) return;
    const int64_t row = t / D;
    const int k = static_cast<int>(t - row * D);
    float acc = 0.f;
    for (int e = row_ptr[row]; e < row_ptr[row + 1]; ++e)
        acc = fmaf(vals ? vals[e] : 1.f, load_elem(X, static_cast<int64_t>(col_idx[e]) * ldx + k, xdt), acc);
    acc = epi.apply(epi.factor(row), acc);
    store_elem(out, row * ldo + k, odt, acc);
}

template <class T>
static void launch_rows_t(int lpr, const ftc_csr &g, const float *vals, const void *X, int ldx, int D,
                          void *out, int ldo, int odt, Epi epi, hipStream_t s)
{
#define FTC_CASE(L)                                                                                  \
    case L: {                                                                                        \
        const int groups = 256 / L;                                                                  \
        const unsigned grid = static_cast<unsigned>((static_cast<int64_t>(g.n) + groups - 1) / groups); \
        hipLaunchKernelGGL((spmm_rows_kernel<T, L>), dim3(grid), dim3(256), 0, s, g.n, g.row_ptr,    \
                           g.col_idx, vals, X, ldx, D, out, ldo, odt, epi);                        \
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

// Vector path usable? (alignment and shape); mirrors the rule stated in ftc.h.
static bool vec_ok(const void *p, int ld, int dt, int D)
{
    const int v = dt == FTC_F32 ? 4 : 8;
    return aligned16(p) && (static_cast<int64_t>(ld) * elem_size(dt)) % 16 == 0 && D % v == 0 && D / v <= 32;
}

int32_t launch_spmm_rows(const ftc_csr &g, const float *vals, const void *X, int ldx, int xdt, int D,
                         void *out, int ldo, int odt, Epi epi, hipStream_t s)
{
    if (g.n == 0) return FTC_OK;
    const int v = xdt == FTC_F32 ? 4 : 8;
    // output rows are written in slices of v elements: 16 B (fp32, v=4), 32 B (fp32, v=8),
    // 8 or 16 B (16-bit); requiring 16-byte aligned rows covers all of them
    if (vec_ok(X, ldx, xdt, D) && aligned16(out) && (static_cast<int64_t>(ldo) * elem_size(odt)) % 16 == 0) {
        int lpr = 1;
        while (lpr * v < D) lpr *= 2;
        if (xdt == FTC_F32) launch_rows_t<F32>(lpr, g, vals, X, ldx, D, out, ldo, odt, epi, s);
        else if (xdt == FTC_F16) launch_rows_t<F16>(lpr, g, vals, X, ldx, D, out, ldo, odt, epi, s);
        else launch_rows_t<BF16>(lpr, g, vals, X, ldx, D, out, ldo, odt, epi, s);
    } else {
        const int64_t total = static_cast<int64_t>(g.n) * D;
        const unsigned grid = static_cast<unsigned>((total + 255) / 256);
        hipLaunchKernelGGL(spmm_generic_kernel, dim3(grid), dim3(256), 0, s, g.n, g.row_ptr, g.col_idx, vals,
                           X, ldx, xdt, D, out, ldo, odt, epi);
    }
    return launch_status("spmm_rows");
}

}  // namespace ftc
