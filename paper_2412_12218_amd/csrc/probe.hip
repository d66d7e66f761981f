// Measurement aid, not part of the method: the bare gather pattern of the aggregation kernels
// (512 row indices per wave, groups of lanes fetch 16 bytes each of a row, eight loads in flight
// per lane) with no arithmetic and no output.  Timing it on a graph's own column indices gives
// the rate at which this GPU can deliver those rows at all, which is the ceiling the SpMM / SDDMM /
// AGNN kernels are measured against next to the HBM roofline.
#include "ftc_common.hpp"

namespace ftc {

template <int LPR>
__global__ __launch_bounds__(256) void gather_probe_kernel(const int *__restrict__ idx, int64_t n_waves,
                                                           const uint4 *__restrict__ X, int stride16,
                                                           float *sink)
{
    constexpr int NG = 64 / LPR, B = 8;
    const int lane = threadIdx.x & 63, g = lane / LPR, sub = lane % LPR;
    const int64_t wave = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (wave >= n_waves) return;
    const int *my = idx + wave * 512;
    float acc = 0.f;
    for (int b = g; b < 512; b += NG * B) {
        int c[B];
        uint4 v[B];
#pragma unroll
        for (int k = 0; k < B; ++k) c[k] = my[b + k * NG];
#pragma unroll
        for (int k = 0; k < B; ++k) v[k] = X[static_cast<int64_t>(c[k]) * stride16 + sub];
#pragma unroll
        for (int k = 0; k < B; ++k) acc += __uint_as_float(v[k].x) + __uint_as_float(v[k].w);
    }
    if (acc == 123.456f) *sink = acc;  // keeps the loads alive; never true for zero-filled X
}

}  // namespace ftc

extern "C" int32_t ftc_gather_probe(const int32_t *idx, int64_t n_idx, const void *X, int32_t row_bytes,
                                    int32_t stride_bytes, float *sink, void *stream)
{
    using namespace ftc;
    if (!idx || !X || !sink || n_idx < 0) {
        set_error("ftc_gather_probe: NULL pointer or negative count");
        return FTC_EINVAL;
    }
    if ((row_bytes != 16 && row_bytes != 32 && row_bytes != 64 && row_bytes != 128) || stride_bytes < row_bytes ||
        stride_bytes % 16 != 0) {
        set_error("ftc_gather_probe: rows of 16, 32, 64 or 128 bytes, stride a multiple of 16 not below the row");
        return FTC_EUNSUPPORTED;
    }
    if (!aligned16(X)) {
        set_error("ftc_gather_probe: X must be 16-byte aligned");
        return FTC_EALIGN;
    }
    const int64_t n_waves = n_idx / 512;  // a trailing partial group of indices is ignored
    if (n_waves == 0) return FTC_OK;
    const unsigned grid = static_cast<unsigned>((n_waves + 3) / 4);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint4 *x = static_cast<const uint4 *>(X);
    const int s16 = stride_bytes / 16;
    switch (row_bytes) {
        case 16: hipLaunchKernelGGL(gather_probe_kernel<1>, dim3(grid), dim3(256), 0, s, idx, n_waves, x, s16, sink); break;
        case 32: hipLaunchKernelGGL(gather_probe_kernel<2>, dim3(grid), dim3(256), 0, s, idx, n_waves, x, s16, sink); break;
        case 64: hipLaunchKernelGGL(gather_probe_kernel<4>, dim3(grid), dim3(256), 0, s, idx, n_waves, x, s16, sink); break;
        default: hipLaunchKernelGGL(gather_probe_kernel<8>, dim3(grid), dim3(256), 0, s, idx, n_waves, x, s16, sink); break;
    }
    return launch_status("gather_probe");
}
