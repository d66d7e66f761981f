// Kernels of the backward pass of the two layers that have no forward counterpart.  The sparse
// products of the backward pass (A^T dP, P^T dY, the edge scores <dY_i, h_j>, ...) reuse the forward
// SpMM / SDDMM kernels; what is here is the glue around them:
//   transposed index of a symmetric pattern, derivative of the row-wise softmax, the ReLU mask,
//   the weight gradient X^T G, the input gradient G W^T, edge-wise combinations and the derivative
//   of the row normalisation of the AGNN cosine.
// The paper speaks of training (Sections II and V) but gives no gradient formulas; these are the
// derivatives of the forward definitions.  Gradients are fp32.
#include "ftc_common.hpp"

namespace ftc {

// ---- T[e] = position of (j, i) for e = (i, j) -----------------------------------------------------
__global__ __launch_bounds__(256) void transpose_index_kernel(int n, int nnz, const int *__restrict__ row_ptr,
                                                              const int *__restrict__ col_idx,
                                                              const int *__restrict__ edge_to_row,
                                                              int *__restrict__ T, int *flag)
{
    const int64_t e = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (e >= nnz) return;
    int i;
    if (edge_to_row) {
        i = edge_to_row[e];
    } else {  // last row with row_ptr[i] <= e
        int a = 0, b = n;
        while (b - a > 1) {
            const int mid = (a + b) >> 1;
            if (row_ptr[mid] <= e) a = mid; else b = mid;
        }
        i = a;
    }
    const int j = col_idx[e];
    int lo = row_ptr[j], hi = row_ptr[j + 1];  // first position in row j with column >= i
    const int end = hi;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (col_idx[mid] < i) lo = mid + 1; else hi = mid;
    }
    const bool found = lo < end && col_idx[lo] == i;
    T[e] = found ? lo : -1;
    if (!found) atomicOr(flag, 1);
}

__global__ void set_int_kernel(int *p, int v) { *p = v; }

int32_t launch_transpose_index(const ftc_csr &g, const int *edge_to_row, int *T, int *flag, hipStream_t s)
{
    hipLaunchKernelGGL(set_int_kernel, dim3(1), dim3(1), 0, s, flag, 0);
    if (g.nnz > 0)
        hipLaunchKernelGGL(transpose_index_kernel, dim3(ceil_div(g.nnz, 256)), dim3(256), 0, s, g.n, g.nnz, g.row_ptr,
                           g.col_idx, edge_to_row, T, flag);
    return launch_status("transpose_index");
}

// ---- ds = p * (dp - sum over the row of p * dp) ----------------------------------------------------
// Row classes as in the row-wise softmax: a lane, a wave or the workgroup per row, by length; the
// order of every row's sum depends on its length alone.
__device__ __forceinline__ float bw_wave_sum(float v)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    return v;
}

__global__ __launch_bounds__(256) void softmax_backward_kernel(int n, const int *__restrict__ row_ptr, const float *p,
                                                               const float *dp, float *ds)
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
    if (len > 0 && len <= 16) {
        float t = 0.f;
        for (int e = e0; e < e1; ++e) t += p[e] * dp[e];
        for (int e = e0; e < e1; ++e) ds[e] = p[e] * (dp[e] - t);
    } else if (len > 16 && len <= 2048) {
        mid_rows[atomicAdd(&n_mid, 1)] = static_cast<int>(row);
    } else if (len > 2048) {
        big_rows[atomicAdd(&n_big, 1)] = static_cast<int>(row);
    }
    __syncthreads();
    const int nm = n_mid, nb = n_big;
    for (int i = wave; i < nm; i += 4) {
        const int r = mid_rows[i];
        const int a = row_ptr[r], b = row_ptr[r + 1];
        float t = 0.f;
        for (int e = a + lane; e < b; e += 64) t += p[e] * dp[e];
        t = bw_wave_sum(t);
        for (int e = a + lane; e < b; e += 64) ds[e] = p[e] * (dp[e] - t);
    }
    for (int i = 0; i < nb; ++i) {  // nb is uniform over the workgroup
        const int r = big_rows[i];
        const int a = row_ptr[r], b = row_ptr[r + 1];
        float t = 0.f;
        for (int e = a + tid; e < b; e += 256) t += p[e] * dp[e];
        t = bw_wave_sum(t);
        __syncthreads();
        if (lane == 0) red[wave] = t;
        __syncthreads();
        t = (red[0] + red[1]) + (red[2] + red[3]);
        for (int e = a + tid; e < b; e += 256) ds[e] = p[e] * (dp[e] - t);
    }
}

int32_t launch_softmax_backward(const ftc_csr &g, const float *p, const float *dp, float *ds, hipStream_t s)
{
    if (g.n == 0 || g.nnz == 0) return FTC_OK;
    hipLaunchKernelGGL(softmax_backward_kernel, dim3((g.n + 255) / 256), dim3(256), 0, s, g.n, g.row_ptr, p, dp, ds);
    return launch_status("edge_softmax_backward");
}

// ---- out = dY * [Y > 0] * scale[row] (fp32) --------------------------------------------------------
__global__ __launch_bounds__(256) void mask_scale_kernel(int n, int d, const float *__restrict__ dY, int lddy,
                                                         const void *__restrict__ Y, int ldy, int ydt,
                                                         const float *__restrict__ scale, float *__restrict__ out,
                                                         int ldo)
{
    const int64_t t = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (t >= static_cast<int64_t>(n) * d) return;
    const int64_t row = t / d;
    const int k = static_cast<int>(t % d);
    float v = dY[row * lddy + k];
    if (Y && !(load_elem(Y, row * ldy + k, ydt) > 0.f)) v = 0.f;
    if (scale) v *= scale[row];
    out[row * ldo + k] = v;
}

int32_t launch_mask_scale(int n, int d, const float *dY, int lddy, const void *Y, int ldy, int ydt,
                          const float *scale, float *out, int ldo, hipStream_t s)
{
    const int64_t total = static_cast<int64_t>(n) * d;
    if (total == 0) return FTC_OK;
    hipLaunchKernelGGL(mask_scale_kernel, dim3(static_cast<unsigned>((total + 255) / 256)), dim3(256), 0, s, n, d, dY,
                       lddy, Y, ldy, ydt, scale, out, ldo);
    return launch_status("mask_scale");
}

// ---- dW = X^T G -----------------------------------------------------------------------------------
// A workgroup walks a contiguous share of the rows, WG_ROWS at a time staged in LDS as fp32; a
// thread owns 4 x 4 tiles of the d_in x d_out result (two 16-byte LDS reads per 16 multiply-adds)
// and keeps them in registers for all of its rows.  When the result has fewer than 256 tiles the
// threads form 256 / tiles slices that split the staged rows between them, and the slices' tiles
// are added in slice order through LDS at the end.  The workgroups' partial results are added by
// a second kernel in workgroup order: reproducible, no floating-point atomics.
constexpr int WG_ROWS = 32;
constexpr int WG_MAX_BLOCKS = 1024;
constexpr int WG_TILES = 4;  // 4 x 4 tiles per thread at most: d_in * d_out <= 256 * 16 * WG_TILES

__global__ __launch_bounds__(256) void weight_grad_kernel(int n, const void *__restrict__ X, int ldx, int xdt, int d_in,
                                                          const float *__restrict__ G, int ldg, int d_out,
                                                          float *__restrict__ partial, int x_vec, int g_vec)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int dip = (d_in + 3) / 4 * 4, dop = (d_out + 3) / 4 * 4;
    float *Xs = lds;                  // [WG_ROWS][dip]
    float *Gs = lds + WG_ROWS * dip;  // [WG_ROWS][dop]
    const int tid = threadIdx.x;
    const int tiles_b = dop / 4, n_tiles = (dip / 4) * tiles_b;
    const int slices = n_tiles < 256 ? 256 / n_tiles : 1;
    const int slice = n_tiles < 256 ? tid / n_tiles : 0;
    const int tile0 = n_tiles < 256 ? tid % n_tiles : tid;
    const bool worker = slice < slices;
    float acc[WG_TILES][16];
#pragma unroll
    for (int u = 0; u < WG_TILES; ++u)
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[u][q] = 0.f;
    const int64_t per = (static_cast<int64_t>(n) + gridDim.x - 1) / gridDim.x;
    const int64_t r_begin = per * blockIdx.x, r_end = min(static_cast<int64_t>(n), r_begin + per);
    const int xv = xdt == FTC_F32 ? 4 : 8;  // elements per 16-byte piece of X
    for (int64_t r0 = r_begin; r0 < r_end; r0 += WG_ROWS) {
        __syncthreads();  // the previous rows are consumed
        if (x_vec) {      // d_in is a multiple of the piece, rows are 16-byte aligned
            const int ppr = d_in / xv;
            for (int t = tid; t < WG_ROWS * ppr; t += 256) {
                const int r = t / ppr, a = (t % ppr) * xv;
                float f[8];
                const bool ok = r0 + r < r_end;
                if (xdt == FTC_F32) {
                    const float4 v = ok ? *reinterpret_cast<const float4 *>(static_cast<const float *>(X) + (r0 + r) * ldx + a)
                                        : make_float4(0.f, 0.f, 0.f, 0.f);
                    *reinterpret_cast<float4 *>(&Xs[r * dip + a]) = v;
                } else {
                    if (ok) {
                        if (xdt == FTC_F16) load_vec<F16>(X, (r0 + r) * ldx + a, f);
                        else load_vec<BF16>(X, (r0 + r) * ldx + a, f);
                    } else {
#pragma unroll
                        for (int q = 0; q < 8; ++q) f[q] = 0.f;
                    }
                    *reinterpret_cast<float4 *>(&Xs[r * dip + a]) = make_float4(f[0], f[1], f[2], f[3]);
                    *reinterpret_cast<float4 *>(&Xs[r * dip + a + 4]) = make_float4(f[4], f[5], f[6], f[7]);
                }
            }
        } else {
            for (int t = tid; t < WG_ROWS * dip; t += 256) {
                const int r = t / dip, a = t % dip;
                Xs[t] = (r0 + r < r_end && a < d_in) ? load_elem(X, (r0 + r) * ldx + a, xdt) : 0.f;
            }
        }
        if (g_vec) {  // d_out is a multiple of 4, rows of G are 16-byte aligned
            for (int t = tid; t < WG_ROWS * tiles_b; t += 256) {
                const int r = t / tiles_b, b = (t % tiles_b) * 4;
                *reinterpret_cast<float4 *>(&Gs[r * dop + b]) =
                    r0 + r < r_end ? *reinterpret_cast<const float4 *>(G + (r0 + r) * ldg + b) : make_float4(0.f, 0.f, 0.f, 0.f);
            }
        } else {
            for (int t = tid; t < WG_ROWS * dop; t += 256) {
                const int r = t / dop, b = t % dop;
                Gs[t] = (r0 + r < r_end && b < d_out) ? G[(r0 + r) * ldg + b] : 0.f;
            }
        }
        __syncthreads();
        if (worker) {
#pragma unroll
            for (int u = 0; u < WG_TILES; ++u) {
                const int tile = tile0 + u * 256;
                if (tile < n_tiles && (u == 0 || n_tiles >= 256)) {
                    const int a0 = (tile / tiles_b) * 4, b0 = (tile % tiles_b) * 4;
                    for (int r = slice; r < WG_ROWS; r += slices) {
                        const float4 x = *reinterpret_cast<const float4 *>(&Xs[r * dip + a0]);
                        const float4 gq = *reinterpret_cast<const float4 *>(&Gs[r * dop + b0]);
                        const float xq[4] = {x.x, x.y, x.z, x.w}, gv[4] = {gq.x, gq.y, gq.z, gq.w};
#pragma unroll
                        for (int i = 0; i < 4; ++i)
#pragma unroll
                            for (int j = 0; j < 4; ++j) acc[u][i * 4 + j] = fmaf(xq[i], gv[j], acc[u][i * 4 + j]);
                    }
                }
            }
        }
    }
    float *out = partial + static_cast<size_t>(blockIdx.x) * d_in * d_out;
    if (n_tiles < 256) {
        // add the slices' tiles in slice order; red[slice][tile][16] reuses the staging memory
        __syncthreads();
        float *red = lds;
        if (worker) {
#pragma unroll
            for (int q = 0; q < 16; ++q) red[(slice * n_tiles + tile0) * 16 + q] = acc[0][q];
        }
        __syncthreads();
        for (int e = tid; e < n_tiles * 16; e += 256) {
            float t = 0.f;
            for (int sl = 0; sl < slices; ++sl) t += red[sl * n_tiles * 16 + e];
            const int tile = e / 16, q = e % 16;
            const int a = (tile / tiles_b) * 4 + q / 4, b = (tile % tiles_b) * 4 + q % 4;
            if (a < d_in && b < d_out) out[a * d_out + b] = t;
        }
        return;
    }
#pragma unroll
    for (int u = 0; u < WG_TILES; ++u) {
        const int tile = tid + u * 256;
        if (tile < n_tiles) {
            const int a0 = (tile / tiles_b) * 4, b0 = (tile % tiles_b) * 4;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (a0 + i < d_in && b0 + j < d_out) out[(a0 + i) * d_out + b0 + j] = acc[u][i * 4 + j];
        }
    }
}

__global__ __launch_bounds__(256) void sum_partials_kernel(int count, int n_partials, const float *__restrict__ partial,
                                                           float *__restrict__ out)
{
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= count) return;
    float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    int b = 0;
    for (; b + 7 < n_partials; b += 8) {
#pragma unroll
        for (int k = 0; k < 8; ++k) s[k] += partial[static_cast<size_t>(b + k) * count + t];
    }
    for (; b < n_partials; ++b) s[0] += partial[static_cast<size_t>(b) * count + t];
    out[t] = ((s[0] + s[1]) + (s[2] + s[3])) + ((s[4] + s[5]) + (s[6] + s[7]));
}

static int weight_grad_blocks(int n)
{
    const int by_rows = (n + 4 * WG_ROWS - 1) / (4 * WG_ROWS);  // at least four row groups per workgroup
    return by_rows < 1 ? 1 : (by_rows > WG_MAX_BLOCKS ? WG_MAX_BLOCKS : by_rows);
}

bool weight_grad_shape_ok(int d_in, int d_out)
{
    // register tiles of one workgroup cover the result; the staged rows fit 64 KB of LDS
    return d_in >= 1 && d_out >= 1 && ((d_in + 3) / 4) * ((d_out + 3) / 4) <= 256 * WG_TILES &&
           (d_in + 3) / 4 * 4 + (d_out + 3) / 4 * 4 <= 512;
}

// Input columns that one pass covers next to d_out output columns: all of them when the register tiles
// and the staged rows allow it, else the largest multiple of 8 that does (at most 256); 0 if none.
int weight_grad_group(int d_in, int d_out)
{
    if (weight_grad_shape_ok(d_in, d_out)) return d_in;
    for (int gk = 256; gk >= 8; gk -= 8)
        if (gk < d_in && weight_grad_shape_ok(gk, d_out)) return gk;
    return 0;
}

size_t weight_grad_ws(int n, int d_in, int d_out)
{
    const int gk = weight_grad_group(d_in, d_out);
    return align_up(static_cast<size_t>(weight_grad_blocks(n)) * (gk > 0 ? gk : d_in) * d_out * sizeof(float), 256);
}

// dW = X^T G.  A wider X is taken in groups of input columns: rows [k0, k0 + gk) of dW are one contiguous
// block, each pass reads its columns of X and all of G, and the passes share the workspace (they run
// one after the other on the stream).
int32_t launch_weight_grad(int n, const void *X, int ldx, int xdt, int d_in, const float *G, int ldg, int d_out,
                           float *dW, void *ws, hipStream_t s)
{
    const int blocks = weight_grad_blocks(n);
    const int group = weight_grad_group(d_in, d_out);
    const int dop = (d_out + 3) / 4 * 4;
    const int xv = xdt == FTC_F32 ? 4 : 8;
    const int g_vec = d_out % 4 == 0 && ldg % 4 == 0 && aligned16(G);
    float *partial = static_cast<float *>(ws);
    for (int k0 = 0; k0 < d_in; k0 += group) {
        const int dk = d_in - k0 < group ? d_in - k0 : group;
        const int dip = (dk + 3) / 4 * 4;
        const int n_tiles = (dip / 4) * (dop / 4);
        size_t lds = static_cast<size_t>(WG_ROWS) * (dip + dop) * sizeof(float);
        if (n_tiles < 256) {  // room for the slices' tiles
            const size_t red = static_cast<size_t>(256 / n_tiles) * n_tiles * 16 * sizeof(float);
            if (red > lds) lds = red;
        }
        const void *Xk = static_cast<const char *>(X) + static_cast<size_t>(k0) * elem_size(xdt);
        const int x_vec = dk % xv == 0 && (static_cast<int64_t>(ldx) * elem_size(xdt)) % 16 == 0 && aligned16(Xk);
        hipLaunchKernelGGL(weight_grad_kernel, dim3(blocks), dim3(256), lds, s, n, Xk, ldx, xdt, dk, G, ldg, d_out,
                           partial, x_vec, g_vec);
        hipLaunchKernelGGL(sum_partials_kernel, dim3((dk * d_out + 255) / 256), dim3(256), 0, s, dk * d_out, blocks,
                           partial, dW + static_cast<size_t>(k0) * d_out);
    }
    return launch_status("weight_grad");
}

// ---- dX = G W^T -----------------------------------------------------------------------------------
// A thread owns one input feature a and keeps row a of W in registers; the rows of G are staged in
// LDS and read as broadcasts.
constexpr int IG_ROWS = 64;

template <int DOUT>  // d_out padded to a multiple of 4
__global__ __launch_bounds__(256) void input_grad_kernel(int n, const float *__restrict__ G, int ldg, int d_out,
                                                         const void *__restrict__ W, int wdt, int d_in,
                                                         void *__restrict__ dX, int lddx, int dx_dt)
{
    __shared__ __attribute__((aligned(16))) float Gs[IG_ROWS * DOUT];
    const int tid = threadIdx.x;
    const int64_t r0 = static_cast<int64_t>(blockIdx.x) * IG_ROWS;
    for (int t = tid; t < IG_ROWS * DOUT; t += 256) {
        const int r = t / DOUT, b = t % DOUT;
        Gs[t] = (r0 + r < n && b < d_out) ? G[(r0 + r) * ldg + b] : 0.f;
    }
    __syncthreads();
    for (int a = tid; a < d_in; a += 256) {
        float w[DOUT];
#pragma unroll
        for (int b = 0; b < DOUT; ++b) w[b] = b < d_out ? load_elem(W, static_cast<int64_t>(a) * d_out + b, wdt) : 0.f;
        for (int r = 0; r < IG_ROWS && r0 + r < n; ++r) {
            float acc = 0.f;
#pragma unroll
            for (int b = 0; b < DOUT; b += 4) {
                const float4 z = *reinterpret_cast<const float4 *>(&Gs[r * DOUT + b]);
                acc = fmaf(z.x, w[b], acc);
                acc = fmaf(z.y, w[b + 1], acc);
                acc = fmaf(z.z, w[b + 2], acc);
                acc = fmaf(z.w, w[b + 3], acc);
            }
            store_elem(dX, (r0 + r) * lddx + a, dx_dt, acc);
        }
    }
}

int32_t launch_input_grad(int n, const float *G, int ldg, int d_out, const void *W, int wdt, int d_in, void *dX,
                          int lddx, int dx_dt, hipStream_t s)
{
    if (n == 0) return FTC_OK;
    const unsigned grid = static_cast<unsigned>((static_cast<int64_t>(n) + IG_ROWS - 1) / IG_ROWS);
#define FTC_IG(P)                                                                                               \
    hipLaunchKernelGGL(input_grad_kernel<P>, dim3(grid), dim3(256), 0, s, n, G, ldg, d_out, W, wdt, d_in, dX, lddx, \
                       dx_dt)
    if (d_out <= 8) FTC_IG(8);
    else if (d_out <= 16) FTC_IG(16);
    else if (d_out <= 32) FTC_IG(32);
    else FTC_IG(64);
#undef FTC_IG
    return launch_status("input_grad");
}

// More than 64 output columns: dX = G W^T is the dense update of the fp32 matrix G with the weights W^T, so
// W is transposed into the workspace as fp32 (d_out x d_in) and the forward kernels do the rest.
__global__ __launch_bounds__(256) void transpose_weights_kernel(int d_in, int d_out, const void *__restrict__ W,
                                                                int wdt, float *__restrict__ Wt)
{
    const int64_t t = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (t >= static_cast<int64_t>(d_in) * d_out) return;
    const int b = static_cast<int>(t / d_in), a = static_cast<int>(t % d_in);  // consecutive threads write consecutive entries
    Wt[t] = load_elem(W, static_cast<int64_t>(a) * d_out + b, wdt);
}

size_t input_grad_ws(int d_in, int d_out)
{
    return d_out > 64 ? align_up(static_cast<size_t>(d_in) * d_out * sizeof(float), 256) : 0;
}

// ws: input_grad_ws(d_in, d_out) bytes, used when d_out > 64
int32_t launch_input_grad_any(int n, const float *G, int ldg, int d_out, const void *W, int wdt, int d_in, void *dX,
                              int lddx, int dx_dt, void *ws, hipStream_t s)
{
    if (d_out <= 64) return launch_input_grad(n, G, ldg, d_out, W, wdt, d_in, dX, lddx, dx_dt, s);
    if (n == 0) return FTC_OK;
    float *Wt = static_cast<float *>(ws);
    const int64_t total = static_cast<int64_t>(d_in) * d_out;
    hipLaunchKernelGGL(transpose_weights_kernel, dim3(static_cast<unsigned>((total + 255) / 256)), dim3(256), 0, s, d_in,
                       d_out, W, wdt, Wt);
    const int32_t st = launch_status("input_grad transpose");
    if (st != FTC_OK) return st;
    return launch_gemm(n, G, ldg, FTC_F32, d_out, Wt, d_in, dX, lddx, dx_dt, Epi{0, nullptr}, s);
}

// ---- out[e] = alpha * (wa * a[e] + wb * a[T[e]]) * cs[col[e]] -------------------------------------
__global__ __launch_bounds__(256) void edge_combine_kernel(int nnz, const float *__restrict__ a,
                                                           const int *__restrict__ T, float wa, float wb, float alpha,
                                                           const float *__restrict__ cs,
                                                           const int *__restrict__ col_idx, float *__restrict__ out)
{
    const int64_t e = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (e >= nnz) return;
    const int t = T[e];  // -1 where the pattern has no partner: that term is dropped, nothing is read
    float v = alpha * (wa * a[e] + ((t >= 0 && t < nnz) ? wb * a[t] : 0.f));
    if (cs) v *= cs[col_idx[e]];
    out[e] = v;
}

int32_t launch_edge_combine(int nnz, const float *a, const int *T, float wa, float wb, float alpha, const float *cs,
                            const int *col_idx, float *out, hipStream_t s)
{
    if (nnz == 0) return FTC_OK;
    hipLaunchKernelGGL(edge_combine_kernel, dim3(ceil_div(nnz, 256)), dim3(256), 0, s, nnz, a, T, wa, wb, alpha, cs,
                       col_idx, out);
    return launch_status("edge_combine");
}

// ---- out = sum_e a[e] * b[e], in a fixed order ----------------------------------------------------
constexpr int DOT_BLOCKS = 1024;

__global__ __launch_bounds__(256) void edge_dot_kernel(int nnz, const float *__restrict__ a, const float *__restrict__ b,
                                                       float *__restrict__ partial)
{
    __shared__ float red[4];
    const int64_t per = (static_cast<int64_t>(nnz) + gridDim.x - 1) / gridDim.x;
    const int64_t lo = per * blockIdx.x, hi = min(static_cast<int64_t>(nnz), lo + per);
    float t = 0.f;
    for (int64_t e = lo + threadIdx.x; e < hi; e += 256) t = fmaf(a[e], b[e], t);
    t = bw_wave_sum(t);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = t;
    __syncthreads();
    if (threadIdx.x == 0) partial[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

__global__ __launch_bounds__(256) void sum_scalar_kernel(int count, const float *__restrict__ partial, float *out)
{
    __shared__ float red[4];
    float t = 0.f;
    for (int i = threadIdx.x; i < count; i += 256) t += partial[i];
    t = bw_wave_sum(t);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = t;
    __syncthreads();
    if (threadIdx.x == 0) *out = (red[0] + red[1]) + (red[2] + red[3]);
}

size_t edge_dot_ws() { return align_up(DOT_BLOCKS * sizeof(float), 256); }

int32_t launch_edge_dot(int nnz, const float *a, const float *b, float *out, void *ws, hipStream_t s)
{
    float *partial = static_cast<float *>(ws);
    hipLaunchKernelGGL(edge_dot_kernel, dim3(DOT_BLOCKS), dim3(256), 0, s, nnz, a, b, partial);
    hipLaunchKernelGGL(sum_scalar_kernel, dim3(1), dim3(256), 0, s, DOT_BLOCKS, partial, out);
    return launch_status("edge_dot");
}

// ---- guard of the single-pass AGNN backward: a pattern that is not symmetric gets NaN, not numbers ------
// *flag != 0 (the flag of ftc_transpose_index): every element of the n x D matrix M and *scalar become NaN.
// With *flag == 0 every thread returns after one load.
__global__ __launch_bounds__(256) void poison_if_flag_kernel(const int32_t *__restrict__ flag, int n, int D,
                                                             void *__restrict__ M, int ld, int dt,
                                                             float *__restrict__ scalar)
{
    if (*flag == 0) return;
    const float nan = __int_as_float(0x7fc00000);
    const int64_t total = static_cast<int64_t>(n) * D;
    for (int64_t t = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; t < total; t += static_cast<int64_t>(gridDim.x) * 256)
        store_elem(M, (t / D) * ld + t % D, dt, nan);
    if (blockIdx.x == 0 && threadIdx.x == 0) *scalar = nan;
}

int32_t launch_poison_if_flag(const int32_t *flag, int n, int D, void *M, int ld, int dt, float *scalar, hipStream_t s)
{
    hipLaunchKernelGGL(poison_if_flag_kernel, dim3(256), dim3(256), 0, s, flag, n, D, M, ld, dt, scalar);
    return launch_status("poison_if_flag");
}

// ---- dH = base + rinv * (q - hn <hn, q>), hn = rinv * h --------------------------------------------
// q is the gradient with respect to the normalised rows, base the part of dH that reaches h through
// the aggregated rows; eight lanes per row.  A row whose norm was clamped (|h| <= 1e-12) is a plain
// scaling: no projection; a row of one element gets nothing through its direction unless clamped.
// base may be dH itself (fp32, in place).
// VEC4: four consecutive elements per lane and step (16-byte loads of q and base; every leading
// dimension a multiple of 4, D too, pointers 16-byte aligned), else element by element.
template <bool VEC4>
__global__ __launch_bounds__(256) void cos_backward_rows_kernel(int n, const void *__restrict__ H, int ld, int dt, int D,
                                                                const float *__restrict__ rinv,
                                                                const float *__restrict__ q, int ldq,
                                                                const float *base, int ldb, void *dH, int lddh,
                                                                int dh_dt)
{
    constexpr int W = VEC4 ? 4 : 1;
    const int sub = threadIdx.x & 7;
    const int64_t row = (static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x) >> 3;
    const bool ok = row < n;
    const float ri = ok ? rinv[row] : 0.f;
    float proj = 0.f;
    // the row has at most 256 elements: 8 lanes x 4 elements x 8 steps, kept in registers between the passes
    float hq[VEC4 ? 8 : 1][W], qq[VEC4 ? 8 : 1][W];
    if (ok) {
        if constexpr (VEC4) {
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                const int k = (s * 8 + sub) * 4;
                if (k < D) {
                    const float4 q4 = *reinterpret_cast<const float4 *>(q + row * ldq + k);
                    qq[s][0] = q4.x; qq[s][1] = q4.y; qq[s][2] = q4.z; qq[s][3] = q4.w;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        hq[s][e] = load_elem(H, row * ld + k + e, dt) * ri;
                        proj = fmaf(hq[s][e], qq[s][e], proj);
                    }
                }
            }
        } else {
            for (int k = sub; k < D; k += 8) proj = fmaf(load_elem(H, row * ld + k, dt) * ri, q[row * ldq + k], proj);
        }
    }
    proj += __shfl_xor(proj, 1, 64);
    proj += __shfl_xor(proj, 2, 64);
    proj += __shfl_xor(proj, 4, 64);
    const bool clamped = ri >= 0.999e12f;  // the clamp of the row-norm kernel took effect
    if (clamped) proj = 0.f;
    // A one-element row normalises to its sign, whose derivative is zero: q - hn <hn, q> would leave the
    // rounding of hn * hn against 1, multiplied by 1 / |h|.
    const float ri_out = (D == 1 && !clamped) ? 0.f : ri;
    if (ok) {
        if constexpr (VEC4) {
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                const int k = (s * 8 + sub) * 4;
                if (k < D) {
                    const float4 b4 = *reinterpret_cast<const float4 *>(base + row * ldb + k);
                    const float bb[4] = {b4.x, b4.y, b4.z, b4.w};
                    float o[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = bb[e] + ri * (qq[s][e] - hq[s][e] * proj);
                    store_vec<4>(dH, row * lddh + k, dh_dt, o);
                }
            }
        } else {
            for (int k = sub; k < D; k += 8) {
                const float hn = load_elem(H, row * ld + k, dt) * ri;
                store_elem(dH, row * lddh + k, dh_dt, base[row * ldb + k] + ri_out * (q[row * ldq + k] - hn * proj));
            }
        }
    }
}

int32_t launch_cos_backward_rows(int n, const void *H, int ld, int dt, int D, const float *rinv, const float *q, int ldq,
                                 const float *base, int ldb, void *dH, int lddh, int dh_dt, hipStream_t s)
{
    if (n == 0) return FTC_OK;
    const unsigned grid = static_cast<unsigned>((static_cast<int64_t>(n) * 8 + 255) / 256);
    const bool vec4 = D % 4 == 0 && D <= 256 && ld % 4 == 0 && ldq % 4 == 0 && ldb % 4 == 0 && lddh % 4 == 0 &&
                      aligned16(q) && aligned16(base) && aligned16(dH) && aligned16(H);
    if (vec4)
        hipLaunchKernelGGL(cos_backward_rows_kernel<true>, dim3(grid), dim3(256), 0, s, n, H, ld, dt, D, rinv, q, ldq, base,
                           ldb, dH, lddh, dh_dt);
    else
        hipLaunchKernelGGL(cos_backward_rows_kernel<false>, dim3(grid), dim3(256), 0, s, n, H, ld, dt, D, rinv, q, ldq,
                           base, ldb, dH, lddh, dh_dt);
    return launch_status("cos_backward_rows");
}

}  // namespace ftc
