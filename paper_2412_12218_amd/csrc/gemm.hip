// Dense update phase Z = X * W for tall-skinny shapes: X is streamed once, W sits in LDS.  The shapes of
// the benchmark models (d_in <= 256, d_out <= 64) keep all of W on chip for the whole kernel; wider
// inputs (the feature matrices of citation graphs have thousands of columns) go through the same
// kernels in chunks of the contraction dimension, wider outputs in groups of 64 columns.
#include "ftc_common.hpp"

namespace ftc {

// One row of X per thread, DOUT accumulators.  W columns [col0, col0 + d_out) of a matrix with w_ld columns;
// K_CHUNK rows of W are staged at a time (all of them when d_in <= K_CHUNK).
template <class T, int DOUT>
__global__ __launch_bounds__(256) void gemm_rows_kernel(int n, const void *__restrict__ X, int ldx, int d_in,
                                                        const void *__restrict__ W, int wdt, int w_ld, int col0,
                                                        int d_out, void *__restrict__ Z, int ldz, int zdt, Epi epi)
{
    constexpr int V = T::VEC;
    constexpr int K_CHUNK = 8192 / DOUT;  // 32 KB of fp32; a multiple of V
    extern __shared__ float Ws[];         // min(d_in, K_CHUNK) x DOUT, zero padded beyond d_out
    const int64_t row = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    float acc[DOUT];
#pragma unroll
    for (int o = 0; o < DOUT; ++o) acc[o] = 0.f;
    for (int kc0 = 0; kc0 < d_in; kc0 += K_CHUNK) {  // uniform
        const int kn = d_in - kc0 < K_CHUNK ? d_in - kc0 : K_CHUNK;
        if (kc0 > 0) __syncthreads();  // the previous chunk has been consumed
        for (int t = threadIdx.x; t < kn * DOUT; t += 256) {
            const int k = t / DOUT, o = t % DOUT;
            Ws[t] = o < d_out ? load_elem(W, static_cast<int64_t>(kc0 + k) * w_ld + col0 + o, wdt) : 0.f;
        }
        __syncthreads();
        if (row < n) {
            for (int k0 = 0; k0 < kn; k0 += V) {
                float x[V];
                load_vec<T>(X, row * ldx + kc0 + k0, x);
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
        }
    }
    if (row >= n) return;
#pragma unroll
    for (int o = 0; o < DOUT; ++o)
        if (o < d_out) store_elem(Z, row * ldz + col0 + o, zdt, epi.apply(epi.factor(row), acc[o]));
}

// Any element type, any alignment (rows of X that are not 16-byte aligned, widths that are no multiple of
// the vector length): a workgroup takes 64 rows and up to 64 output columns [col0, col0 + d_out), and
// walks the contraction dimension in chunks of 64.  The chunk of X is read element by element with
// consecutive threads on consecutive columns and parked in LDS as fp32 next to the chunk of W; a thread
// then owns one row and 16 output columns.
constexpr int GU_ROWS = 64, GU_K = 64;

__global__ __launch_bounds__(256) void gemm_unaligned_kernel(int n, const void *__restrict__ X, int ldx, int dt, int d_in,
                                                             const void *__restrict__ W, int w_ld, int col0, int d_out,
                                                             void *__restrict__ Z, int ldz, int zdt, Epi epi)
{
    __shared__ float Xs[GU_ROWS][GU_K + 1];  // odd stride: the 64 rows read by a wave fall on different banks
    __shared__ __attribute__((aligned(16))) float Ws[GU_K][64];
    const int tid = threadIdx.x;
    const int64_t r0 = static_cast<int64_t>(blockIdx.x) * GU_ROWS;
    const int r = tid & 63, og = tid >> 6;  // row of the tile, group of 16 output columns
    float acc[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[j] = 0.f;
    for (int k0 = 0; k0 < d_in; k0 += GU_K) {  // uniform
        if (k0 > 0) __syncthreads();
        for (int t = tid; t < GU_ROWS * GU_K; t += 256) {
            const int rr = t / GU_K, kk = t % GU_K;
            Xs[rr][kk] = (r0 + rr < n && k0 + kk < d_in) ? load_elem(X, (r0 + rr) * ldx + k0 + kk, dt) : 0.f;
        }
        for (int t = tid; t < GU_K * 64; t += 256) {
            const int kk = t / 64, o = t % 64;
            Ws[kk][o] = (k0 + kk < d_in && o < d_out) ? load_elem(W, static_cast<int64_t>(k0 + kk) * w_ld + col0 + o, dt) : 0.f;
        }
        __syncthreads();
#pragma unroll 8
        for (int kk = 0; kk < GU_K; ++kk) {
            const float x = Xs[r][kk];
#pragma unroll
            for (int j = 0; j < 16; j += 4) {
                const float4 w = *reinterpret_cast<const float4 *>(&Ws[kk][og * 16 + j]);
                acc[j] = fmaf(x, w.x, acc[j]);
                acc[j + 1] = fmaf(x, w.y, acc[j + 1]);
                acc[j + 2] = fmaf(x, w.z, acc[j + 2]);
                acc[j + 3] = fmaf(x, w.w, acc[j + 3]);
            }
        }
    }
    const int64_t row = r0 + r;
    if (row >= n) return;
    const float f = epi.factor(static_cast<int>(row));
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        const int o = og * 16 + j;
        if (o < d_out) store_elem(Z, row * ldz + col0 + o, zdt, epi.apply(f, acc[j]));
    }
}

// ------------------------------------------------------------------------------------------------
// Matrix-core version for 16-bit inputs.  The update phase is a dense contraction, so it goes to
// MFMA (v_mfma_f32_16x16x32_{f16,bf16}, fp32 accumulate).  A wave owns tiles of 16 rows of X:
//   A operand  lane l holds X[row0 + l%16][k0 + (l/16)*8 .. +7]: one 16-byte global load, the four
//              lane groups of a row cover 64 contiguous bytes, so X streams in fully used lines;
//   B operand  lane l holds W[k0 + (l/16)*8 .. +7][n0 + l%16]: W is transposed once into LDS
//              (k contiguous, zero padded to multiples of 32 x 16) and read as 16-byte words;
//   C          lane l holds Z[row0 + (l/16)*4 + i][n0 + l%16], i = 0..3.
// The kernel is bound by streaming X from HBM; W (at most 256 x 64) is read once per workgroup.
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef __bf16 bhalf8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));

template <class T>
__device__ __forceinline__ float4v mfma16(const uint4 &a, const uint4 &b, float4v c)
{
    if constexpr (std::is_same<T, F16>::value)
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, a), __builtin_bit_cast(half8, b), c,
                                                      0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bhalf8, a), __builtin_bit_cast(bhalf8, b),
                                                       c, 0, 0, 0);
}

constexpr int GEMM_RT = 2;  // 16-row tiles per wave iteration

template <class T, int KS, int NT>  // KS = ceil(d_in / 32), NT = ceil(d_out / 16)
__global__ __launch_bounds__(256) void gemm_mfma_kernel(int n, const uint16_t *__restrict__ X, int ldx, int d_in,
                                                        const uint16_t *__restrict__ W, int d_out,
                                                        void *__restrict__ Z, int ldz, int zdt, Epi epi,
                                                        int n_tiles, bool vec_store)
{
    constexpr int KP = KS * 32 + 8;  // padded k extent of a W^T row (keeps 16-byte alignment, spreads banks)
    __shared__ __attribute__((aligned(16))) uint16_t Wt[NT * 16 * KP];
    for (int t = threadIdx.x; t < NT * 16 * KS * 32; t += 256) {
        const int nn = t / (KS * 32), k = t % (KS * 32);
        Wt[nn * KP + k] = (nn < d_out && k < d_in) ? W[static_cast<size_t>(k) * d_out + nn] : uint16_t(0);
    }
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 15, kb = lane >> 4;
    // B operands stay in registers for the whole kernel
    uint4 breg[KS][NT];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
            breg[ks][nt] = *reinterpret_cast<const uint4 *>(&Wt[(nt * 16 + m) * KP + ks * 32 + kb * 8]);

    constexpr int ZP = NT * 16 + 4;  // row stride of the output patch (16-byte aligned, spreads banks)
    __shared__ __attribute__((aligned(16))) float Zs[4][16 * ZP];
    const int stride = gridDim.x * 4 * GEMM_RT;
    for (int tile0 = (blockIdx.x * 4 + wave) * GEMM_RT; tile0 < n_tiles; tile0 += stride) {
        uint4 a[GEMM_RT][KS];
#pragma unroll
        for (int rt = 0; rt < GEMM_RT; ++rt) {
            const int row = min((tile0 + rt) * 16 + m, n - 1);  // clamped: the store is predicated
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const int k = ks * 32 + kb * 8;
                if (k < d_in) a[rt][ks] = *reinterpret_cast<const uint4 *>(X + static_cast<size_t>(row) * ldx + k);
                else a[rt][ks] = make_uint4(0u, 0u, 0u, 0u);
            }
        }
#pragma unroll
        for (int rt = 0; rt < GEMM_RT; ++rt) {
            float4v c[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                c[nt] = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) c[nt] = mfma16<T>(a[rt][ks], breg[ks][nt], c[nt]);
            }
            if (vec_store) {
                // The accumulators hold columns (lane = column, register = row): written as they are,
                // a 16-bit output would leave in 2-byte pieces, four store instructions per 16 x 16
                // tile.  The tile is turned through LDS instead (each wave has its own patch; LDS
                // operations of one wave execute in order) so that a lane holds 4 NT consecutive
                // columns of one row and the tile leaves in one or two 8- or 16-byte stores per lane.
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int i = 0; i < 4; ++i) Zs[wave][(kb * 4 + i) * ZP + nt * 16 + m] = c[nt][i];
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                const int r = lane >> 2, c0 = (lane & 3) * (4 * NT);
                const int row = (tile0 + rt) * 16 + r;
                float o[4 * NT];
#pragma unroll
                for (int q = 0; q < NT; ++q) {
                    const float4 v = *reinterpret_cast<const float4 *>(&Zs[wave][r * ZP + c0 + 4 * q]);
                    o[4 * q] = v.x; o[4 * q + 1] = v.y; o[4 * q + 2] = v.z; o[4 * q + 3] = v.w;
                }
                if (row < n && c0 < d_out) {
                    const float f = epi.factor(row);
#pragma unroll
                    for (int j = 0; j < 4 * NT; ++j) o[j] = epi.apply(f, o[j]);
                    if constexpr (NT == 1) {
                        store_vec<4>(Z, static_cast<int64_t>(row) * ldz + c0, zdt, reinterpret_cast<float(&)[4]>(o));
                    } else {
#pragma unroll
                        for (int q = 0; q < NT / 2; ++q)
                            store_vec<8>(Z, static_cast<int64_t>(row) * ldz + c0 + 8 * q, zdt,
                                         reinterpret_cast<float(&)[8]>(o[8 * q]));
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();  // the patch is rewritten by the next tile
            } else {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const int col = nt * 16 + m;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int row = (tile0 + rt) * 16 + kb * 4 + i;
                        if (row < n && col < d_out)
                            store_elem(Z, static_cast<int64_t>(row) * ldz + col, zdt,
                                       epi.apply(epi.factor(row), c[nt][i]));
                    }
                }
            }
        }
    }
}

// The same contraction for any d_in (rows of X 16-byte aligned; the last piece of a width that is no
// multiple of 8 is read element by element) and a group of up to 64 output columns [col0, col0 + d_out)
// of a W with w_ld columns: W^T is staged in chunks of 256 rows of W, a workgroup keeps the
// accumulators of 4 x RT tiles of 16 rows across the chunks, and B operands come from LDS.
constexpr int WIDE_KC = 256;

template <class T, int WIDE_RT>
__global__ __launch_bounds__(256) void gemm_mfma_wide_kernel(int n, const uint16_t *__restrict__ X, int ldx, int d_in,
                                                             const uint16_t *__restrict__ W, int w_ld, int col0,
                                                             int d_out, void *__restrict__ Z, int ldz, int zdt,
                                                             Epi epi, int n_batches)
{
    constexpr int NT = 4, KP = WIDE_KC + 8;
    __shared__ __attribute__((aligned(16))) uint16_t Wt[NT * 16 * KP];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = lane & 15, kb = lane >> 4;
    const int nt_n = (d_out + 15) / 16;
    for (int batch = blockIdx.x; batch < n_batches; batch += gridDim.x) {  // uniform over the workgroup
        const int tile0 = (batch * 4 + wave) * WIDE_RT;
        float4v c[WIDE_RT][NT];
#pragma unroll
        for (int rt = 0; rt < WIDE_RT; ++rt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) c[rt][nt] = float4v{0.f, 0.f, 0.f, 0.f};
        for (int kc0 = 0; kc0 < d_in; kc0 += WIDE_KC) {
            __syncthreads();  // the previous chunk (or batch) has been consumed
            const int nn_n = nt_n * 16;  // only the column tiles that are used
            for (int t = threadIdx.x; t < nn_n * WIDE_KC; t += 256) {
                const int k = t / nn_n, nn = t % nn_n;  // consecutive threads read consecutive columns of W
                Wt[nn * KP + k] = (nn < d_out && kc0 + k < d_in) ? W[static_cast<size_t>(kc0 + k) * w_ld + col0 + nn]
                                                                 : uint16_t(0);
            }
            __syncthreads();
#pragma unroll
            for (int ks = 0; ks < WIDE_KC / 32; ++ks) {
                const int k = kc0 + ks * 32 + kb * 8;
                uint4 a[WIDE_RT];
#pragma unroll
                for (int rt = 0; rt < WIDE_RT; ++rt) {
                    const int64_t row = min(static_cast<int64_t>(tile0 + rt) * 16 + m, static_cast<int64_t>(n) - 1);
                    if (k + 8 <= d_in) {
                        a[rt] = *reinterpret_cast<const uint4 *>(X + row * ldx + k);
                    } else {  // the last piece of a width that is no multiple of 8: element by element, nothing beyond d_in is read
                        unsigned h[8];
#pragma unroll
                        for (int j = 0; j < 8; ++j) h[j] = k + j < d_in ? X[row * ldx + k + j] : 0u;
                        a[rt] = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
                    }
                }
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    if (nt < nt_n) {
                        const uint4 b = *reinterpret_cast<const uint4 *>(&Wt[(nt * 16 + m) * KP + ks * 32 + kb * 8]);
#pragma unroll
                        for (int rt = 0; rt < WIDE_RT; ++rt) c[rt][nt] = mfma16<T>(a[rt], b, c[rt][nt]);
                    }
                }
            }
        }
#pragma unroll
        for (int rt = 0; rt < WIDE_RT; ++rt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const int col = nt * 16 + m;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int64_t row = static_cast<int64_t>(tile0 + rt) * 16 + kb * 4 + i;
                    if (row < n && col < d_out)
                        store_elem(Z, row * ldz + col0 + col, zdt, epi.apply(epi.factor(static_cast<int>(row)), c[rt][nt][i]));
                }
            }
    }
}

template <class T>
static void gemm_mfma_wide_t(int n, const void *X, int ldx, int d_in, const void *W, int d_out, void *Z, int ldz,
                             int zdt, Epi epi, hipStream_t s)
{
    const int64_t n_tiles = (static_cast<int64_t>(n) + 15) / 16;
    // four tiles per wave: W is re-staged once per 256 rows (one tile per wave was measured 2.4 times slower
    // at 100 k rows, although it starts four times as many workgroups)
    const int64_t n_batches = (n_tiles + 15) / 16;
    const unsigned grid = static_cast<unsigned>(n_batches < 256 * 4 ? n_batches : 256 * 4);
    for (int col0 = 0; col0 < d_out; col0 += 64) {
        const int cols = d_out - col0 < 64 ? d_out - col0 : 64;
        hipLaunchKernelGGL((gemm_mfma_wide_kernel<T, 4>), dim3(grid), dim3(256), 0, s, n,
                           static_cast<const uint16_t *>(X), ldx, d_in, static_cast<const uint16_t *>(W), d_out, col0,
                           cols, Z, ldz, zdt, epi, static_cast<int>(n_batches));
    }
}

template <class T>
static bool gemm_mfma_t(int n, const void *X, int ldx, int d_in, const void *W, int d_out, void *Z, int ldz,
                        int zdt, Epi epi, hipStream_t s)
{
    const int ks = (d_in + 31) / 32, nt = (d_out + 15) / 16;
    const int n_tiles = (n + 15) / 16;
    int grid = (n_tiles + 4 * GEMM_RT - 1) / (4 * GEMM_RT);
    if (grid > 256 * 8) grid = 256 * 8;
    const uint16_t *x = static_cast<const uint16_t *>(X);
    const uint16_t *w = static_cast<const uint16_t *>(W);
    // whole groups of 4 NT columns per lane, each group 8- or 16-byte aligned in the output
    const int zsize = zdt == FTC_F32 ? 4 : 2;
    const bool vec_store = d_out % (4 * nt) == 0 && aligned16(Z) && (static_cast<int64_t>(ldz) * zsize) % 16 == 0 &&
                           (nt == 1 || nt % 2 == 0);
#define FTC_G(K, N)                                                                                                 if (ks == K && nt == N) {                                                                                           hipLaunchKernelGGL((gemm_mfma_kernel<T, K, N>), dim3(grid), dim3(256), 0, s, n, x, ldx, d_in, w, d_out, Z,                            ldz, zdt, epi, n_tiles, vec_store);                                                                    return true;                                                                                                }
    FTC_G(1, 1) FTC_G(1, 2) FTC_G(2, 1) FTC_G(2, 2) FTC_G(4, 1) FTC_G(4, 2) FTC_G(4, 4) FTC_G(2, 4) FTC_G(1, 4)
    FTC_G(8, 1) FTC_G(8, 2) FTC_G(8, 4) FTC_G(3, 1) FTC_G(3, 2) FTC_G(3, 4)
#undef FTC_G
    return false;
}

template <class T>
static void gemm_t(int n, const void *X, int ldx, int d_in, const void *W, int wdt, int d_out, void *Z, int ldz, int zdt,
                   Epi epi, hipStream_t s)
{
    const unsigned grid = static_cast<unsigned>((static_cast<int64_t>(n) + 255) / 256);
    for (int col0 = 0; col0 < d_out; col0 += 64) {
        const int cols = d_out - col0 < 64 ? d_out - col0 : 64;
        int dpad = 8;
        while (dpad < cols) dpad *= 2;
        const int k_chunk = 8192 / dpad;
        const size_t lds = static_cast<size_t>(d_in < k_chunk ? d_in : k_chunk) * dpad * sizeof(float);
#define FTC_CASE(P)                                                                                          \
    case P:                                                                                                  \
        hipLaunchKernelGGL((gemm_rows_kernel<T, P>), dim3(grid), dim3(256), lds, s, n, X, ldx, d_in, W, wdt, \
                           d_out, col0, cols, Z, ldz, zdt, epi);                                             \
        break;
        switch (dpad) {
            FTC_CASE(8)
            FTC_CASE(16)
            FTC_CASE(32)
            FTC_CASE(64)
        }
#undef FTC_CASE
    }
}

int32_t launch_gemm(int n, const void *X, int ldx, int dt, int d_in, const void *W, int d_out, void *Z, int ldz,
                    int zdt, Epi epi, hipStream_t s)
{
    if (n == 0) return FTC_OK;
    const int v = dt == FTC_F32 ? 4 : 8;
    // vector loads of X: 16-byte aligned rows, whole vectors
    const bool fast = aligned16(X) && (static_cast<int64_t>(ldx) * elem_size(dt)) % 16 == 0 && d_in % v == 0;
    // 16-bit inputs: matrix cores (needs 16-byte row pieces of X)
    const bool rows16 = aligned16(X) && (static_cast<int64_t>(ldx) * elem_size(dt)) % 16 == 0;
    if (dt != FTC_F32 && rows16) {
        const bool done = fast && (dt == FTC_F16 ? gemm_mfma_t<F16>(n, X, ldx, d_in, W, d_out, Z, ldz, zdt, epi, s)
                                                 : gemm_mfma_t<BF16>(n, X, ldx, d_in, W, d_out, Z, ldz, zdt, epi, s));
        if (done) return launch_status("update_gemm mfma");
        // beyond the register-resident shapes, or a width that is no multiple of 8 in padded rows
        if (d_in > 256 || d_out > 64 || !fast) {
            if (dt == FTC_F16) gemm_mfma_wide_t<F16>(n, X, ldx, d_in, W, d_out, Z, ldz, zdt, epi, s);
            else gemm_mfma_wide_t<BF16>(n, X, ldx, d_in, W, d_out, Z, ldz, zdt, epi, s);
            return launch_status("update_gemm mfma (wide)");
        }
    }
    if (fast) {
        if (dt == FTC_F32) gemm_t<F32>(n, X, ldx, d_in, W, dt, d_out, Z, ldz, zdt, epi, s);
        else if (dt == FTC_F16) gemm_t<F16>(n, X, ldx, d_in, W, dt, d_out, Z, ldz, zdt, epi, s);
        else gemm_t<BF16>(n, X, ldx, d_in, W, dt, d_out, Z, ldz, zdt, epi, s);
    } else {
        const unsigned grid = static_cast<unsigned>((static_cast<int64_t>(n) + GU_ROWS - 1) / GU_ROWS);
        for (int col0 = 0; col0 < d_out; col0 += 64) {
            const int cols = d_out - col0 < 64 ? d_out - col0 : 64;
            hipLaunchKernelGGL(gemm_unaligned_kernel, dim3(grid), dim3(256), 0, s, n, X, ldx, dt, d_in, W, d_out, col0,
                               cols, Z, ldz, zdt, epi);
        }
    }
    return launch_status("update_gemm");
}

}  // namespace ftc
