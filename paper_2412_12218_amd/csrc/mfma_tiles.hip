// Matrix-core path on condensed row windows (Section V.A, sparse neighbour aggregation and
// sparse edge feature computation), for windows dense enough to pay for it.
//
// A window is 16 rows; its condensed column list S_w (win_cols) maps tile columns to rows of the
// feature matrix (`sparse_AToX_index`).  One 64-lane workgroup handles one window with
// v_mfma_f32_16x16x32_{f16,bf16} (fp32 accumulate):
//
//   SDDMM  scores[16 x |S_w|] = X[window rows] * Y[S_w]^T.  The contraction runs over the feature
//          dimension, which is contiguous in memory for both operands, so A and B operands are
//          16-byte global loads with no staging.  The dense score tile goes to LDS and every edge
//          of the window picks its value by (edge_to_row, edge_to_col).  Each neighbour row is
//          gathered once per window instead of once per edge.
//   SpMM   out[16 x D] = A_w[16 x |S_w|] * X[S_w].  The contraction runs over condensed columns,
//          32 per step: the edge values are added into an fp32 tile in LDS by the lane that owns
//          the cell (storage order, so duplicates add reproducibly), every tile value is split
//          into two bf16 pieces (full fp32 exponent range, 2^-17 relative accuracy per value,
//          no common scale) and the 32 gathered rows are staged row-major in LDS and read back
//          element-wise in operand order.
//
// Windows are selected by a per-window flag (see win_classify_kernel); the vector kernels skip
// exactly the flagged windows.
#include "ftc_common.hpp"

namespace ftc {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef __bf16 bhalf8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));

template <class T>
__device__ __forceinline__ float4v mfma16x16x32(const uint4 &a, const uint4 &b, float4v c)
{
    if constexpr (std::is_same<T, F16>::value)
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, a), __builtin_bit_cast(half8, b), c,
                                                      0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bhalf8, a), __builtin_bit_cast(bhalf8, b),
                                                       c, 0, 0, 0);
}

// flags[w] = 1 when window w goes to the matrix cores: it has edges, at most max_edges of them,
// and at least `reuse` edges per condensed column on average.
__global__ __launch_bounds__(256) void win_classify_kernel(int n, int n_windows, const int *__restrict__ row_ptr,
                                                           const int *__restrict__ win_col_ptr, float reuse,
                                                           int max_edges, uint8_t *__restrict__ flags)
{
    const int w = blockIdx.x * 256 + threadIdx.x;
    if (w >= n_windows) return;
    const int r0 = w * 16;
    const int cnt = row_ptr[min(n, r0 + 16)] - row_ptr[r0];
    const int uniq = win_col_ptr[w + 1] - win_col_ptr[w];
    flags[w] = (cnt > 0 && cnt <= max_edges && static_cast<float>(cnt) >= reuse * static_cast<float>(uniq)) ? 1 : 0;
}

int32_t launch_classify(const ftc_csr &g, const ftc_windows &w, float reuse, int max_edges, uint8_t *flags,
                        hipStream_t s)
{
    if (w.n_windows == 0) return FTC_OK;
    hipLaunchKernelGGL(win_classify_kernel, dim3((w.n_windows + 255) / 256), dim3(256), 0, s, g.n, w.n_windows,
                       g.row_ptr, w.win_col_ptr, reuse, max_edges, flags);
    return launch_status("win_classify");
}

// ------------------------------------------------------------------------------------------------
constexpr int SDM_CH = 64;   // condensed columns per LDS chunk (small: LDS per window bounds occupancy)
constexpr int SDM_NU = 4;    // 16-column tiles gathered before their MFMAs are issued

template <class T, int KS>  // KS = ceil(D / 32)
__global__ __launch_bounds__(64) void sddmm_mfma_kernel(int n, const int *__restrict__ row_ptr,
                                                        const int *__restrict__ edge_to_row,
                                                        const int *__restrict__ edge_to_col,
                                                        const int *__restrict__ win_col_ptr,
                                                        const int *__restrict__ win_cols,
                                                        const uint16_t *__restrict__ X,
                                                        const uint16_t *__restrict__ Y, int ld, int D,
                                                        const float *__restrict__ rs, const float *__restrict__ cs,
                                                        float alpha, float *__restrict__ out,
                                                        const uint8_t *__restrict__ flags)
{
    __shared__ float S[16][SDM_CH + 1];
    const int w = blockIdx.x;
    const int r0 = w * 16;
    const int e0 = row_ptr[r0], e1 = row_ptr[min(n, r0 + 16)];
    if (!flags[w]) return;
    const int u0 = win_col_ptr[w];
    const int uniq = win_col_ptr[w + 1] - u0;
    const int lane = threadIdx.x, m = lane & 15, kb = lane >> 4;

    uint4 a[KS];
    {
        const int row = min(r0 + m, n - 1);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int k = ks * 32 + kb * 8;
            a[ks] = k < D ? *reinterpret_cast<const uint4 *>(X + static_cast<size_t>(row) * ld + k)
                          : make_uint4(0u, 0u, 0u, 0u);
        }
    }
    float rsv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) rsv[i] = alpha * (rs ? rs[min(r0 + kb * 4 + i, n - 1)] : 1.f);

    for (int cb = 0; cb < uniq; cb += SDM_CH) {
        const int nch = min(SDM_CH, uniq - cb);
        for (int t0 = 0; t0 * 16 < nch; t0 += SDM_NU) {
            uint4 b[SDM_NU][KS];
            float csv[SDM_NU];
#pragma unroll
            for (int u = 0; u < SDM_NU; ++u) {
                const int c = cb + (t0 + u) * 16 + m;
                const int colv = win_cols[u0 + min(c, uniq - 1)];
                csv[u] = cs ? cs[colv] : 1.f;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const int k = ks * 32 + kb * 8;
                    b[u][ks] = k < D ? *reinterpret_cast<const uint4 *>(Y + static_cast<size_t>(colv) * ld + k)
                                     : make_uint4(0u, 0u, 0u, 0u);
                }
            }
#pragma unroll
            for (int u = 0; u < SDM_NU; ++u) {
                float4v acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) acc = mfma16x16x32<T>(a[ks], b[u][ks], acc);
                const int cc = (t0 + u) * 16 + m;
                if (cc < nch) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) S[kb * 4 + i][cc] = rsv[i] * csv[u] * acc[i];
                }
            }
        }
        __syncthreads();
        for (int e = e0 + lane; e < e1; e += 64) {
            const int cc = edge_to_col[e] - cb;
            if (cc >= 0 && cc < nch) out[e] = S[edge_to_row[e] - r0][cc];
        }
        __syncthreads();
    }
}

// ------------------------------------------------------------------------------------------------
// An fp32 value as the sum of two bf16 pieces.  bf16 keeps the exponent range of fp32, so the pair
// carries every value with a relative error of at most 2^-17 whatever its magnitude: no scale is
// needed and a small value next to a large one in the same tile keeps its own accuracy.
__device__ __forceinline__ void split_bf16_pair(float v, uint32_t &hi, uint32_t &lo)
{
    hi = f32_to_bf16_bits(v);
    const bool finite = (hi & 0x7f80u) != 0x7f80u;
    lo = finite ? f32_to_bf16_bits(v - __uint_as_float(hi << 16)) : 0u;
}

// The tile product always runs on v_mfma_f32_16x16x32_bf16.  bf16 features enter as they are (two
// MFMAs per step: value high and low piece).  An fp16 feature (11 significant bits) is the exact sum
// of two bf16 pieces; three MFMAs per step (high x high, low x high, high x low) leave out only the
// low x low product, 2^-18 of a term.
template <class T, int NT>  // NT = ceil(D / 16)
__global__ __launch_bounds__(64) void spmm_mfma_kernel(int n, const int *__restrict__ row_ptr,
                                                       const int *__restrict__ edge_to_col,
                                                       const int *__restrict__ win_col_ptr,
                                                       const int *__restrict__ win_cols,
                                                       const float *__restrict__ vals,
                                                       const uint16_t *__restrict__ X, int ldx, int D,
                                                       void *__restrict__ out, int ldo, int odt, Epi epi,
                                                       const uint8_t *__restrict__ flags)
{
    constexpr bool SPLIT_X = std::is_same<T, F16>::value;
    constexpr int DP = NT * 16 + 8;  // 16-bit elements per staged row (16-byte pad)
    __shared__ float As[16][36];     // 16 rows x 32 condensed columns (+pad)
    __shared__ __attribute__((aligned(16))) uint16_t Xs[(SPLIT_X ? 2 : 1) * 32 * DP];
    uint16_t *const Xlo = Xs + 32 * DP;  // low pieces of fp16 features
    const int w = blockIdx.x;
    const int r0 = w * 16;
    if (!flags[w]) return;
    const int u0 = win_col_ptr[w];
    const int uniq = win_col_ptr[w + 1] - u0;
    const int lane = threadIdx.x, m = lane & 15, kb = lane >> 4;

    // Lane (m, kb) owns the tile cells (m, c) with c % 4 == kb and adds the entries of row r0 + m
    // that fall into them in storage order: no atomics, duplicates add in one fixed order.  With
    // ascending condensed columns in every row of the window (the usual case) a cursor per row walks
    // each entry once; otherwise every chunk scans the whole row.
    const int rb = row_ptr[min(n, r0 + m)], re = row_ptr[min(n, r0 + m + 1)];
    bool ascending = true;
    for (int e = rb + 1 + kb; e < re; e += 4) ascending = ascending && edge_to_col[e - 1] <= edge_to_col[e];
    const bool cursor_mode = __builtin_amdgcn_ballot_w64(!ascending) == 0ull;
    int cur = rb;

    float4v acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = float4v{0.f, 0.f, 0.f, 0.f};
    const int pieces = NT * 2;  // 16-byte pieces per staged row (D padded to a multiple of 16)

    for (int c0 = 0; c0 < uniq; c0 += 32) {
        for (int t = lane; t < 16 * 36; t += 64) (&As[0][0])[t] = 0.f;
        __syncthreads();
        if (cursor_mode) {
            int e = cur;
            for (; e < re; ++e) {
                const int cc = edge_to_col[e] - c0;  // >= 0: earlier chunks took everything below c0
                if (cc >= 32) break;
                if ((cc & 3) == kb) As[m][cc] += vals ? vals[e] : 1.f;
            }
            cur = e;
        } else {
            for (int e = rb; e < re; ++e) {
                const int cc = edge_to_col[e] - c0;
                if (cc >= 0 && cc < 32 && (cc & 3) == kb) As[m][cc] += vals ? vals[e] : 1.f;
            }
        }
        for (int t = lane; t < 32 * pieces; t += 64) {
            const int k = t / pieces, piece = t % pieces;
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (c0 + k < uniq && piece * 8 < D)
                v = *reinterpret_cast<const uint4 *>(X + static_cast<size_t>(win_cols[u0 + c0 + k]) * ldx + piece * 8);
            if constexpr (SPLIT_X) {
                const uint32_t in[4] = {v.x, v.y, v.z, v.w};
                uint32_t h[4], l[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    uint32_t h0, l0, h1, l1;
                    split_bf16_pair(f16_bits_to_f32(in[j] & 0xffffu), h0, l0);
                    split_bf16_pair(f16_bits_to_f32(in[j] >> 16), h1, l1);
                    h[j] = h0 | (h1 << 16);
                    l[j] = l0 | (l1 << 16);
                }
                *reinterpret_cast<uint4 *>(&Xs[k * DP + piece * 8]) = make_uint4(h[0], h[1], h[2], h[3]);
                *reinterpret_cast<uint4 *>(&Xlo[k * DP + piece * 8]) = make_uint4(l[0], l[1], l[2], l[3]);
            } else {
                *reinterpret_cast<uint4 *>(&Xs[k * DP + piece * 8]) = v;
            }
        }
        __syncthreads();
        uint32_t hi[8], lo[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) split_bf16_pair(As[m][kb * 8 + j], hi[j], lo[j]);
        const uint4 ahi = make_uint4(hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16), hi[4] | (hi[5] << 16),
                                     hi[6] | (hi[7] << 16));
        const uint4 alo = make_uint4(lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16), lo[4] | (lo[5] << 16),
                                     lo[6] | (lo[7] << 16));
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            uint32_t x[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) x[j] = Xs[(kb * 8 + j) * DP + t * 16 + m];
            const uint4 b = make_uint4(x[0] | (x[1] << 16), x[2] | (x[3] << 16), x[4] | (x[5] << 16),
                                       x[6] | (x[7] << 16));
            acc[t] = mfma16x16x32<BF16>(alo, b, acc[t]);
            if constexpr (SPLIT_X) {
#pragma unroll
                for (int j = 0; j < 8; ++j) x[j] = Xlo[(kb * 8 + j) * DP + t * 16 + m];
                const uint4 bl = make_uint4(x[0] | (x[1] << 16), x[2] | (x[3] << 16), x[4] | (x[5] << 16),
                                            x[6] | (x[7] << 16));
                acc[t] = mfma16x16x32<BF16>(ahi, bl, acc[t]);
            }
            acc[t] = mfma16x16x32<BF16>(ahi, b, acc[t]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int col = t * 16 + m;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = r0 + kb * 4 + i;
            if (row < n && col < D)
                store_elem(out, static_cast<int64_t>(row) * ldo + col, odt, epi.apply(epi.factor(row), acc[t][i]));
        }
    }
}

bool mfma_shape_ok(int dtype, int D)
{
    if (dtype != FTC_F16 && dtype != FTC_BF16) return false;
    if (D % 8 != 0 || D > 256) return false;
    const int nt = (D + 15) / 16;
    return nt <= 4 || nt == 6 || nt == 8 || nt == 12 || nt == 16;
}

// Caller has checked: blk_h == 16, mfma_shape_ok(dtype, D), rows 16-byte aligned, flags filled.
int32_t launch_sddmm_mfma(const ftc_csr &g, const ftc_windows &w, const void *X, const void *Y, int ld, int dt,
                          int D, const float *rs, const float *cs, float alpha, float *out, const uint8_t *flags,
                          hipStream_t s)
{
    if (w.n_windows == 0 || g.nnz == 0) return FTC_OK;
    const int ks = (D + 31) / 32;
    const uint16_t *x = static_cast<const uint16_t *>(X);
    const uint16_t *y = static_cast<const uint16_t *>(Y);
#define FTC_SM(K)                                                                                               \
    case K:                                                                                                     \
        if (dt == FTC_F16)                                                                                      \
            hipLaunchKernelGGL((sddmm_mfma_kernel<F16, K>), dim3(w.n_windows), dim3(64), 0, s, g.n, g.row_ptr,  \
                               w.edge_to_row, w.edge_to_col, w.win_col_ptr, w.win_cols, x, y, ld, D, rs, cs,    \
                               alpha, out, flags);                                                   \
        else                                                                                                    \
            hipLaunchKernelGGL((sddmm_mfma_kernel<BF16, K>), dim3(w.n_windows), dim3(64), 0, s, g.n, g.row_ptr, \
                               w.edge_to_row, w.edge_to_col, w.win_col_ptr, w.win_cols, x, y, ld, D, rs, cs,    \
                               alpha, out, flags);                                                   \
        break;
    switch (ks) {
        FTC_SM(1) FTC_SM(2) FTC_SM(3) FTC_SM(4) FTC_SM(5) FTC_SM(6) FTC_SM(7) FTC_SM(8)
    }
#undef FTC_SM
    return launch_status("sddmm_mfma");
}

int32_t launch_spmm_mfma(const ftc_csr &g, const ftc_windows &w, const float *vals, const void *X, int ldx, int dt,
                         int D, void *out, int ldo, int odt, Epi epi, const uint8_t *flags, hipStream_t s)
{
    if (w.n_windows == 0) return FTC_OK;
    const int nt = (D + 15) / 16;
    const uint16_t *x = static_cast<const uint16_t *>(X);
#define FTC_PM(N)                                                                                              \
    case N:                                                                                                    \
        if (dt == FTC_F16)                                                                                     \
            hipLaunchKernelGGL((spmm_mfma_kernel<F16, N>), dim3(w.n_windows), dim3(64), 0, s, g.n, g.row_ptr,  \
                               w.edge_to_col, w.win_col_ptr, w.win_cols, vals, x, ldx, D, out, ldo, odt, epi, \
                               flags);                                                                         \
        else                                                                                                   \
            hipLaunchKernelGGL((spmm_mfma_kernel<BF16, N>), dim3(w.n_windows), dim3(64), 0, s, g.n, g.row_ptr, \
                               w.edge_to_col, w.win_col_ptr, w.win_cols, vals, x, ldx, D, out, ldo, odt, epi, \
                               flags);                                                                         \
        break;
    switch (nt) {
        FTC_PM(1) FTC_PM(2) FTC_PM(3) FTC_PM(4) FTC_PM(6) FTC_PM(8) FTC_PM(12) FTC_PM(16)
        default:
            set_error("spmm_mfma: feature width %d not instantiated", D);
            return FTC_EUNSUPPORTED;
    }
#undef FTC_PM
    return launch_status("spmm_mfma");
}

}  // namespace ftc
