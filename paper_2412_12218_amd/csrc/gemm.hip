// Dense update phase Z = X * W for tall-skinny shapes (n rows, d_in <= 256, d_out <= 64):
// X is streamed once, W sits in LDS as fp32.
#include "ftc_common.hpp"

namespace ftc {

template <class T, int DOUT>
__global__ __launch_bounds__(256) void gemm_rows_kernel(int n, const void *__restrict__ X, int ldx, int d_in,
                                                        const void *__restrict__ W, int wdt, int d_out,
                                                        void *__restrict__ Z, int ldz, int zdt, int relu)
{
    constexpr int V = T::VEC;
    extern __shared__ float Ws[];  // d_in x DOUT, zero padded beyond d_out
    for (int t = threadIdx.x; t < d_in * DOUT; t += 256) {
        const int k = t / DOUT, o = t % DOUT;
        Ws[t] = o < d_out ? load_elem(W, static_cast<int64_t>(k) * d_out + o, wdt) : 0.f;
    }
    __syncthreads();
    const int64_t row = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (row >= n) return;
    float acc[DOUT];
#pragma unroll
    for (int o = 0; o < DOUT; ++o) acc[o] = 0.f;
    for (int k0 = 0; k0 < d_in; k0 += V) {
        float x[V];
        load_vec<T>(X, row * ldx + k0, x);
#pragma unroll
        for (int kk = 0; kk < V; ++kk) {
            const float4 *w4 = reinterpret_cast<const float4 *>(Ws + (k0 + kk) * DOUT);
#pragma unroll
            for (int o = 0; o < DOUT / 4; ++o) {
                const float4 w = w4[o];
                acc[4 * o] = fmaf(x[kk], w.x, acc[4 * o]);
                acc[4 * o + 1] = fmaf(x[kk], w.y, acc[4 * o + 1]);
                acc[4 * o + 2] = fmaf(x[kk], w.z, acc[4 * o + 2]);
                acc[4 * o + 3] = fmaf(x[kk], w.w, acc[4 * o + 3]);
            }
        }
    }
#pragma unroll
    for (int o = 0; o < DOUT; ++o)
        if (o < d_out) store_elem(Z, row * ldz + o, zdt, relu ? fmaxf(acc[o], 0.f) : acc[o]);
}

__global__ __launch_bounds__(256) void gemm_generic_kernel(int n, const void *X, int ldx, int dt, int d_in,
                                                           const void *W, int d_out, void *Z, int ldz,
                                                           int zdt, int relu)
{
    const int64_t t = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (t >= static_cast<int64_t>(n) * d_out) return;
    const int64_t row = t / d_out;
    const int o = static_cast<int>(t - row * d_out);
    float acc = 0.f;
    for (int k = 0; k < d_in; ++k)
        acc = fmaf(load_elem(X, row * ldx + k, dt), load_elem(W, static_cast<int64_t>(k) * d_out + o, dt), acc);
    store_elem(Z, row * ldz + o, zdt, relu ? fmaxf(acc, 0.f) : acc);
}

template <class T>
static void gemm_t(int dpad, int n, const void *X, int ldx, int d_in, const void *W, int wdt, int d_out,
                   void *Z, int ldz, int zdt, int relu, hipStream_t s)
{
    const unsigned grid = static_cast<unsigned>((static_cast<int64_t>(n) + 255) / 256);
    const size_t lds = static_cast<size_t>(d_in) * dpad * sizeof(float);
#define FTC_CASE(P)                                                                                     \
    case P:                                                                                             \
        hipLaunchKernelGGL((gemm_rows_kernel<T, P>), dim3(grid), dim3(256), lds, s, n, X, ldx, d_in, W, \
                           wdt, d_out, Z, ldz, zdt, relu);                                              \
        break;
    switch (dpad) {
        FTC_CASE(8)
        FTC_CASE(16)
        FTC_CASE(32)
        FTC_CASE(64)
    }
#undef FTC_CASE
}

int32_t launch_gemm(int n, const void *X, int ldx, int dt, int d_in, const void *W, int d_out, void *Z,
                    int ldz, int zdt, int relu, hipStream_t s)
{
    if (n == 0) return FTC_OK;
    const int v = dt == FTC_F32 ? 4 : 8;
    int dpad = 8;
    while (dpad < d_out) dpad *= 2;
    const bool fast = aligned16(X) && (static_cast<int64_t>(ldx) * elem_size(dt)) % 16 == 0 && d_in % v == 0 &&
                      dpad <= 64 && static_cast<int64_t>(d_in) * dpad <= 8192;
    if (fast) {
        if (dt == FTC_F32) gemm_t<F32>(dpad, n, X, ldx, d_in, W, dt, d_out, Z, ldz, zdt, relu, s);
        else if (dt == FTC_F16) gemm_t<F16>(dpad, n, X, ldx, d_in, W, dt, d_out, Z, ldz, zdt, relu, s);
        else gemm_t<BF16>(dpad, n, X, ldx, d_in, W, dt, d_out, Z, ldz, zdt, relu, s);
    } else {
        const int64_t total = static_cast<int64_t>(n) * d_out;
        hipLaunchKernelGGL(gemm_generic_kernel, dim3(static_cast<unsigned>((total + 255) / 256)), dim3(256), 0,
                           s, n, X, ldx, dt, d_in, W, d_out, Z, ldz, zdt, relu);
    }
    return launch_status("update_gemm");
}

}  // namespace ftc
