// Shared host/device helpers of libftc (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "ftc.h"

namespace ftc {

constexpr int WAVE = 64;
constexpr int SEG_R = 512;  // edges per wave of the edge-balanced kernels (SpMM, fused AGNN forward / backward)

// ---- host side -------------------------------------------------------------------------------
void set_error(const char *fmt, ...);
int32_t launch_status(const char *what);  // FTC_OK or FTC_EHIP after a kernel launch

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int elem_size(int dtype) { return dtype == FTC_F32 ? 4 : 2; }
inline bool valid_dtype(int d) { return d == FTC_F32 || d == FTC_F16 || d == FTC_BF16; }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// ceil(a / b) for non-negative a up to INT32_MAX (the sum a + b - 1 would not fit)
inline int ceil_div(int a, int b) { return static_cast<int>((static_cast<int64_t>(a) + b - 1) / b); }

// Epilogue of the kernels that produce dense rows: out = act(scale[row] * value), scale optional.
struct Epi {
    int relu;
    const float *scale;
#if defined(__HIPCC__)
    __device__ __forceinline__ float factor(int64_t row) const { return scale ? scale[row] : 1.f; }
    __device__ __forceinline__ float apply(float f, float v) const
    {
        v *= f;
        return relu ? fmaxf(v, 0.f) : v;
    }
#endif
};

// Entry points implemented in the individual .hip files (host launchers, no validation).
int32_t launch_spmm_rows(const ftc_csr &g, const float *vals, const void *X, int ldx, int xdt, int D,
                         void *out, int ldo, int odt, Epi epi, hipStream_t s);
int32_t launch_sddmm_rows(const ftc_csr &g, const void *X, const void *Y, int ld, int dt, int D,
                          const float *rs, const float *cs, float alpha, float *out, hipStream_t s);
int32_t launch_softmax(const ftc_csr &g, const float *in, float *out, hipStream_t s);
size_t softmax_seg_ws(int n, int nnz);
int32_t launch_softmax_seg(const ftc_csr &g, const ftc_windows &w, const float *in, float *out, void *ws,
                           hipStream_t s);
int32_t launch_row_rnorm(int n, const void *H, int ld, int dt, int D, float *rinv, hipStream_t s);
int32_t launch_gemm(int n, const void *X, int ldx, int dt, int d_in, const void *W, int d_out, void *Z,
                    int ldz, int zdt, Epi epi, hipStream_t s);
int32_t launch_gcn_norm(const ftc_csr &g, const ftc_windows *w, float *vals, float *dinv, hipStream_t s);
int32_t launch_validate(const ftc_csr &g, int32_t *flag, hipStream_t s);
bool seg_shape(int dtype, int D, int *vec, int *lpr);
size_t spmm_seg_ws(int nnz, int D);
bool spmm_lane_shape(int xdt, int D, int ldx);
size_t spmm_lane_ws(int nnz);
int32_t launch_spmm_lane(const ftc_csr &g, const ftc_windows &w, const float *vals, const void *X, int ldx, int xdt,
                         int D, void *out, int ldo, int odt, Epi epi, void *ws, hipStream_t s);
int32_t launch_spmm_seg(const ftc_csr &g, const ftc_windows &w, const float *vals, const void *X, int ldx,
                        int xdt, int D, void *out, int ldo, int odt, Epi epi, void *ws, const uint8_t *dense,
                        hipStream_t s);
int32_t launch_sddmm_edges(const ftc_csr &g, const ftc_windows &w, const void *X, const void *Y, int ld, int dt,
                           int D, const float *rs, const float *cs, float alpha, float *out, const uint8_t *dense,
                           bool cosine, hipStream_t s);
size_t agnn_fused_ws(int nnz, int D);
int32_t launch_agnn_fused(const ftc_csr &g, const ftc_windows &w, const void *H, int ld, int dt, int D,
                          float beta, void *out, int ldo, int odt, float *row_z, float *out32, int ld32, void *ws,
                          hipStream_t s);
bool agnn_backward_fused_shape(int dtype, int D);
size_t agnn_backward_fused_ws(int n, int nnz, int D);
int32_t launch_agnn_backward_fused(const ftc_csr &g, const ftc_windows &w, const void *H, const void *dY, int ld, int dt,
                                   int D, float beta, const float *row_z, const void *Y, int ldy, int ydt, void *dH,
                                   int lddh, int dh_dt, float *dbeta, void *ws, hipStream_t s);
bool mfma_shape_ok(int dtype, int D);
int32_t launch_classify(const ftc_csr &g, const ftc_windows &w, float reuse, int max_edges, uint8_t *flags,
                        hipStream_t s);
int32_t launch_sddmm_mfma(const ftc_csr &g, const ftc_windows &w, const void *X, const void *Y, int ld, int dt,
                          int D, const float *rs, const float *cs, float alpha, float *out, const uint8_t *flags,
                          hipStream_t s);
int32_t launch_spmm_mfma(const ftc_csr &g, const ftc_windows &w, const float *vals, const void *X, int ldx, int dt,
                         int D, void *out, int ldo, int odt, Epi epi, const uint8_t *flags, hipStream_t s);
// backward.hip
int32_t launch_poison_if_flag(const int32_t *flag, int n, int D, void *M, int ld, int dt, float *scalar, hipStream_t s);
int32_t launch_transpose_index(const ftc_csr &g, const int *edge_to_row, int *T, int *flag, hipStream_t s);
int32_t launch_softmax_backward(const ftc_csr &g, const float *p, const float *dp, float *ds, hipStream_t s);
int32_t launch_softmax_backward_seg(const ftc_csr &g, const ftc_windows &w, const float *p, const float *dp, float *ds,
                                    void *ws, hipStream_t s);
int32_t launch_mask_scale(int n, int d, const float *dY, int lddy, const void *Y, int ldy, int ydt,
                          const float *scale, float *out, int ldo, hipStream_t s);
bool weight_grad_shape_ok(int d_in, int d_out);
int weight_grad_group(int d_in, int d_out);
size_t input_grad_ws(int d_in, int d_out);
int32_t launch_input_grad_any(int n, const float *G, int ldg, int d_out, const void *W, int wdt, int d_in, void *dX,
                              int lddx, int dx_dt, void *ws, hipStream_t s);
size_t weight_grad_ws(int n, int d_in, int d_out);
int32_t launch_weight_grad(int n, const void *X, int ldx, int xdt, int d_in, const float *G, int ldg, int d_out,
                           float *dW, void *ws, hipStream_t s);
int32_t launch_input_grad(int n, const float *G, int ldg, int d_out, const void *W, int wdt, int d_in, void *dX,
                          int lddx, int dx_dt, hipStream_t s);
int32_t launch_edge_combine(int nnz, const float *a, const int *T, float wa, float wb, float alpha, const float *cs,
                            const int *col_idx, float *out, hipStream_t s);
size_t edge_dot_ws();
int32_t launch_edge_dot(int nnz, const float *a, const float *b, float *out, void *ws, hipStream_t s);
int32_t launch_cos_backward_rows(int n, const void *H, int ld, int dt, int D, const float *rinv, const float *q, int ldq,
                                 const float *base, int ldb, void *dH, int lddh, int dh_dt, hipStream_t s);
// reorder.hip
size_t reorder_ws(int n, int nnz);
int32_t launch_degree_stats(const ftc_csr &g, int64_t *stats, hipStream_t s);
int32_t launch_order_by_key(int n, const int *keys, int *perm, int *inv, int *flag, void *ws, hipStream_t s);
int32_t launch_label_propagation(const ftc_csr &g, int iters, int *labels, void *ws, hipStream_t s);
int32_t launch_degree_order(const ftc_csr &g, int mode, int *perm, int *inv, void *ws, hipStream_t s);
int32_t launch_permute_graph(const ftc_csr &g, const int *perm, const int *inv, int *row_ptr_out, int *col_idx_out,
                             int *flag, void *ws, hipStream_t s);
int32_t launch_permute_rows(int n, const void *X, int ldx, int dt, int D, const int *map, void *out, int ldo,
                            hipStream_t s);
size_t build_windows_ws(int n, int nnz, int blk_h, int blk_w);
int32_t launch_build_windows(const ftc_csr &g, ftc_windows &w, void *ws, size_t ws_bytes, const ftc_side_streams *side,
                             hipStream_t s);

// ---- device side -----------------------------------------------------------------------------
#if defined(__HIPCC__)

// Element types.  A "vector" is one 16-byte load: 4 fp32 or 8 16-bit values.
struct F32 {
    static constexpr int VEC = 4;
    static constexpr int BYTES = 4;
};
struct F16 {
    static constexpr int VEC = 8;
    static constexpr int BYTES = 2;
};
struct BF16 {
    static constexpr int VEC = 8;
    static constexpr int BYTES = 2;
};

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;  // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);                               // round to nearest even
    return u >> 16;
}
__device__ __forceinline__ float f16_bits_to_f32(uint32_t b)
{
    return static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(b)));
}
__device__ __forceinline__ uint32_t f32_to_f16_bits(float f)
{
    return __builtin_bit_cast(uint16_t, static_cast<_Float16>(f));
}

// 16-byte vector load of T::VEC elements starting at element index `idx` (multiple of VEC).
template <class T>
__device__ __forceinline__ void load_vec(const void *base, int64_t idx, float (&f)[T::VEC]);

template <>
__device__ __forceinline__ void load_vec<F32>(const void *base, int64_t idx, float (&f)[4])
{
    float4 v = *reinterpret_cast<const float4 *>(static_cast<const float *>(base) + idx);
    f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
}
template <>
__device__ __forceinline__ void load_vec<F16>(const void *base, int64_t idx, float (&f)[8])
{
    uint4 v = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(base) + idx);
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        f[2 * k] = f16_bits_to_f32(w[k] & 0xffffu);
        f[2 * k + 1] = f16_bits_to_f32(w[k] >> 16);
    }
}
template <>
__device__ __forceinline__ void load_vec<BF16>(const void *base, int64_t idx, float (&f)[8])
{
    uint4 v = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(base) + idx);
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        f[2 * k] = __uint_as_float(w[k] << 16);
        f[2 * k + 1] = __uint_as_float(w[k] & 0xffff0000u);
    }
}

// Scalar element load / store with a run-time dtype (generic paths and epilogues).
__device__ __forceinline__ float load_elem(const void *base, int64_t idx, int dtype)
{
    if (dtype == FTC_F32) return static_cast<const float *>(base)[idx];
    uint32_t b = static_cast<const uint16_t *>(base)[idx];
    return dtype == FTC_F16 ? f16_bits_to_f32(b) : bf16_bits_to_f32(b);
}
__device__ __forceinline__ void store_elem(void *base, int64_t idx, int dtype, float v)
{
    if (dtype == FTC_F32) static_cast<float *>(base)[idx] = v;
    else if (dtype == FTC_F16) static_cast<uint16_t *>(base)[idx] = static_cast<uint16_t>(f32_to_f16_bits(v));
    else static_cast<uint16_t *>(base)[idx] = static_cast<uint16_t>(f32_to_bf16_bits(v));
}

// Narrow vector loads: NV elements (NV * sizeof(element) = 4, 8 or 16 bytes; 2 bytes for a
// single 16-bit element) starting at element index idx, which must be a multiple of NV.
// RawVec keeps the loaded words as they are; unpack() converts to fp32 at the point of use so
// that several loads can be in flight without holding their fp32 expansions in registers.
template <class T, int NV>
struct RawVec {
    static constexpr int WORDS = (NV * T::BYTES + 3) / 4;
    uint32_t w[WORDS];
};

template <class T, int NV>
__device__ __forceinline__ void zero_raw(RawVec<T, NV> &r)
{
#pragma unroll
    for (int k = 0; k < RawVec<T, NV>::WORDS; ++k) r.w[k] = 0u;
}

template <class T, int NV>
__device__ __forceinline__ void load_raw(const void *base, int64_t idx, RawVec<T, NV> &r)
{
    constexpr int BYTES = NV * T::BYTES;
    const char *p = static_cast<const char *>(base) + idx * T::BYTES;
    if constexpr (BYTES == 16) {
        const uint4 v = *reinterpret_cast<const uint4 *>(p);
        r.w[0] = v.x; r.w[1] = v.y; r.w[2] = v.z; r.w[3] = v.w;
    } else if constexpr (BYTES == 8) {
        const uint2 v = *reinterpret_cast<const uint2 *>(p);
        r.w[0] = v.x; r.w[1] = v.y;
    } else if constexpr (BYTES == 4) {
        r.w[0] = *reinterpret_cast<const uint32_t *>(p);
    } else {
        static_assert(BYTES == 2, "vector loads are 2, 4, 8 or 16 bytes");
        r.w[0] = *reinterpret_cast<const uint16_t *>(p);
    }
}

template <class T, int NV>
__device__ __forceinline__ void unpack(const RawVec<T, NV> &r, float (&f)[NV])
{
#pragma unroll
    for (int k = 0; k < NV; ++k) {
        if constexpr (T::BYTES == 4) {
            f[k] = __uint_as_float(r.w[k]);
        } else {
            const uint32_t word = r.w[k / 2];
            if constexpr (std::is_same<T, F16>::value) f[k] = f16_bits_to_f32((k & 1) ? (word >> 16) : (word & 0xffffu));
            else f[k] = (k & 1) ? __uint_as_float(word & 0xffff0000u) : __uint_as_float(word << 16);
        }
    }
}

// acc + sum_k a[k] * b[k] on the packed representation.  16-bit types use the packed dot-product
// instructions (v_dot2c_f32_f16 / v_dot2c_f32_bf16: two products per instruction, fp32 accumulate),
// which also saves unpacking the operands.
template <class T, int NV>
__device__ __forceinline__ float dot_raw(const RawVec<T, NV> &a, const RawVec<T, NV> &b, float acc)
{
    if constexpr (T::BYTES == 4) {
#pragma unroll
        for (int k = 0; k < NV; ++k) acc = fmaf(__uint_as_float(a.w[k]), __uint_as_float(b.w[k]), acc);
    } else {
        static_assert(NV % 2 == 0, "packed dot products take pairs");
        typedef _Float16 half2v __attribute__((ext_vector_type(2)));
        typedef __bf16 bhalf2v __attribute__((ext_vector_type(2)));
#pragma unroll
        for (int k = 0; k < NV / 2; ++k) {
            if constexpr (std::is_same<T, F16>::value)
                acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2v, a.w[k]), __builtin_bit_cast(half2v, b.w[k]),
                                             acc, false);
            else
                acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bhalf2v, a.w[k]),
                                                      __builtin_bit_cast(bhalf2v, b.w[k]), acc, false);
        }
    }
    return acc;
}

template <class T, int NV>
__device__ __forceinline__ void load_n(const void *base, int64_t idx, float (&f)[NV])
{
    RawVec<T, NV> r;
    load_raw<T, NV>(base, idx, r);
    unpack<T, NV>(r, f);
}

// Store NV consecutive floats (NV = 1, 2, 4 or 8) at element index idx (multiple of NV; rows are
// 16-byte aligned by the caller's checks) in the run-time output dtype.
template <int NV>
__device__ __forceinline__ void store_vec(void *base, int64_t idx, int dtype, const float (&f)[NV])
{
    if (dtype == FTC_F32) {
        float *p = static_cast<float *>(base) + idx;
        if constexpr (NV >= 4) {
#pragma unroll
            for (int k = 0; k < NV / 4; ++k)
                reinterpret_cast<float4 *>(p)[k] = make_float4(f[4 * k], f[4 * k + 1], f[4 * k + 2], f[4 * k + 3]);
        } else if constexpr (NV == 2) {
            *reinterpret_cast<float2 *>(p) = make_float2(f[0], f[1]);
        } else {
            *p = f[0];
        }
    } else {
        uint16_t *q = static_cast<uint16_t *>(base) + idx;
        if constexpr (NV == 1) {
            *q = static_cast<uint16_t>(dtype == FTC_F16 ? f32_to_f16_bits(f[0]) : f32_to_bf16_bits(f[0]));
        } else {
            uint32_t w[NV / 2];
#pragma unroll
            for (int k = 0; k < NV / 2; ++k) {
                const uint32_t lo = dtype == FTC_F16 ? f32_to_f16_bits(f[2 * k]) : f32_to_bf16_bits(f[2 * k]);
                const uint32_t hi = dtype == FTC_F16 ? f32_to_f16_bits(f[2 * k + 1]) : f32_to_bf16_bits(f[2 * k + 1]);
                w[k] = lo | (hi << 16);
            }
            if constexpr (NV == 8) *reinterpret_cast<uint4 *>(q) = make_uint4(w[0], w[1], w[2], w[3]);
            else if constexpr (NV == 4) *reinterpret_cast<uint2 *>(q) = make_uint2(w[0], w[1]);
            else *reinterpret_cast<uint32_t *>(q) = w[0];
        }
    }
}

// The same store with the non-temporal hint: rows that are written once and not read again by this kernel
// should not push gathered rows out of L2.
typedef uint32_t ftc_u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t ftc_u32x2 __attribute__((ext_vector_type(2)));
typedef float ftc_f32x4 __attribute__((ext_vector_type(4)));
template <int NV>
__device__ __forceinline__ void store_vec_nt(void *base, int64_t idx, int dtype, const float (&f)[NV])
{
    if (dtype == FTC_F32) {
        float *p = static_cast<float *>(base) + idx;
        if constexpr (NV >= 4) {
#pragma unroll
            for (int k = 0; k < NV / 4; ++k) {
                ftc_f32x4 v = {f[4 * k], f[4 * k + 1], f[4 * k + 2], f[4 * k + 3]};
                __builtin_nontemporal_store(v, reinterpret_cast<ftc_f32x4 *>(p) + k);
            }
        } else {
#pragma unroll
            for (int k = 0; k < NV; ++k) __builtin_nontemporal_store(f[k], p + k);
        }
    } else {
        uint16_t *q = static_cast<uint16_t *>(base) + idx;
        if constexpr (NV == 8 || NV == 4) {
            uint32_t w[NV / 2];
#pragma unroll
            for (int k = 0; k < NV / 2; ++k) {
                const uint32_t lo = dtype == FTC_F16 ? f32_to_f16_bits(f[2 * k]) : f32_to_bf16_bits(f[2 * k]);
                const uint32_t hi = dtype == FTC_F16 ? f32_to_f16_bits(f[2 * k + 1]) : f32_to_bf16_bits(f[2 * k + 1]);
                w[k] = lo | (hi << 16);
            }
            if constexpr (NV == 8) {
                ftc_u32x4 v = {w[0], w[1], w[2], w[3]};
                __builtin_nontemporal_store(v, reinterpret_cast<ftc_u32x4 *>(q));
            } else {
                ftc_u32x2 v = {w[0], w[1]};
                __builtin_nontemporal_store(v, reinterpret_cast<ftc_u32x2 *>(q));
            }
        } else {
            store_vec<NV>(base, idx, dtype, f);
        }
    }
}

template <int CTRL>
__device__ __forceinline__ float dpp_add(float v)
{
    const int moved = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false);
    return v + __int_as_float(moved);
}

// Sum over the LPR consecutive lanes of a group; every lane of the group gets the total.
template <int LPR>
__device__ __forceinline__ float group_sum_dpp(float v)
{
    if constexpr (LPR >= 32) v += __shfl_xor(v, 16, 64);
    if constexpr (LPR >= 16) v = dpp_add<0x140>(v);  // row_mirror: lane i <-> 15 - i
    if constexpr (LPR >= 8) v = dpp_add<0x141>(v);   // row_half_mirror: lane i <-> 7 - i
    if constexpr (LPR >= 4) v = dpp_add<0x4e>(v);    // quad_perm [2,3,0,1]
    if constexpr (LPR >= 2) v = dpp_add<0xb1>(v);    // quad_perm [1,0,3,2]
    return v;
}

// Second pass of the edge-balanced kernels (spmm_seg.hip): finishes the rows cut by a wave boundary
// from the carry buffer (rows of dp floats, dp a multiple of 4, 16-byte aligned) and zero-fills the rows
// without entries.
int32_t launch_seg_fixup(int n, int n_ranges, const int *row_ptr, const float *carry, const int *tail_row, int dp,
                         int D, void *out, int ldo, int odt, Epi epi, const uint8_t *dense, int seg_r, hipStream_t s,
                         const char *what);

// Workgroups are handed to the eight XCDs round-robin by their index, and every XCD has an L2 of its
// own.  The edge-balanced kernels walk the edges in order, so neighbouring workgroups gather
// neighbouring rows' columns: this maps the workgroups so that every XCD works on chunks of
// XCD_CHUNK consecutive logical blocks (the k-th workgroup of XCD x takes block k % XCD_CHUNK of chunk
// (k / XCD_CHUNK) * 8 + x) instead of on every eighth block.  Chunks, not one contiguous eighth of
// the edges per XCD: the cost of a block varies along the edge list of a skewed graph, and whole
// eighths were measured 10 to 40 % slower there.  The blocks beyond the last full group of eight
// chunks keep their index.
constexpr int XCD_CHUNK = 16;
__device__ __forceinline__ int xcd_chunked_block(int b, int grid)
{
    const int full = grid / (8 * XCD_CHUNK) * (8 * XCD_CHUNK);
    if (b >= full) return b;
    const int x = b & 7, k = b >> 3;
    return ((k / XCD_CHUNK) * 8 + x) * XCD_CHUNK + k % XCD_CHUNK;
}

// Rows of the R consecutive edges [base, base + R) of a FULL range, for a wave that stages edge 64 j + lane
// in step j: rows[j] = row of that edge.  Reading edge_to_row for every edge is a second 4-byte stream next
// to the column ids; the rows are also known from the range's first and last row and the starts of the
// rows in between: with at most 64 of those, every lane fetches one start and an edge's row is the first
// row plus the number of starts at or before it (empty rows count themselves in).  Returns false
// (wave-uniform) when the range holds more rows than that: the caller then reads edge_to_row.
template <int R>
__device__ __forceinline__ bool rows_from_starts(const int *__restrict__ row_ptr, const int *__restrict__ edge_to_row,
                                                 int base, int lane, int (&rows)[R / 64])
{
    const int r_first = edge_to_row[base], r_last = edge_to_row[base + R - 1];
    const int n_starts = r_last - r_first;  // rows r_first + 1 .. r_last begin inside the range
    if (n_starts > 64) return false;
    const int start = lane < n_starts ? row_ptr[r_first + 1 + lane] - base : INT32_MAX;
    int cnt[R / 64];
#pragma unroll
    for (int j = 0; j < R / 64; ++j) cnt[j] = 0;
    for (int t = 0; t < n_starts; ++t) {
        const int rel = __builtin_amdgcn_readlane(start, t) - lane;  // the start seen from this lane's edge of step 0
#pragma unroll
        for (int j = 0; j < R / 64; ++j) cnt[j] += rel <= j * 64 ? 1 : 0;
    }
#pragma unroll
    for (int j = 0; j < R / 64; ++j) rows[j] = r_first + cnt[j];
    return true;
}

// The same for a wave whose lanes own L CONSECUTIVE edges each (the lane's first edge is base + e0; lanes
// of one slot may share it): rows[k] = row of edge base + e0 + k, for a full range of `range` edges.
// Up to 256 row starts are held four per lane; a lane counts the starts at or before its first edge and
// marks those inside its L <= 32 edges.  An empty row shares its start with the next row, and a mark
// cannot say how many rows begin at one edge: such ranges, and ranges with more rows, return false
// (wave-uniform) and the caller reads edge_to_row.  All 64 lanes must be active.
template <int L>
__device__ __forceinline__ bool lane_rows_from_starts(const int *__restrict__ row_ptr,
                                                      const int *__restrict__ edge_to_row, int base, int range, int e0,
                                                      int lane, int (&rows)[L])
{
    static_assert(L <= 32, "one mark per edge in a 32-bit word");
    constexpr int Q = 4;  // starts per lane
    const int r_first = edge_to_row[base], r_last = edge_to_row[base + range - 1];
    const int n_starts = r_last - r_first;  // rows r_first + 1 .. r_last begin inside the range
    if (n_starts > 64 * Q) return false;
    int start_l[Q];
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        const int t = q * 64 + lane;
        start_l[q] = t < n_starts ? row_ptr[r_first + 1 + t] : INT32_MAX;
    }
    bool dup = false;
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        const int over = q + 1 < Q ? __shfl(start_l[q + 1 < Q ? q + 1 : q], 0, 64) : INT32_MAX;
        int nxt = __shfl_down(start_l[q], 1, 64);  // every lane takes part in both moves
        if (lane == 63) nxt = over;
        dup = dup || (start_l[q] != INT32_MAX && start_l[q] == nxt);
    }
    if (__builtin_amdgcn_ballot_w64(dup) != 0ull) return false;
    const int first_edge = base + e0;
    int before = 0;        // starts at or before the lane's first edge
    unsigned inside = 0u;  // bit k: a row starts at edge k of the lane (k = 1 .. L - 1)
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        const int n_q = n_starts - q * 64 < 64 ? n_starts - q * 64 : 64;
        for (int t = 0; t < n_q; ++t) {
            const int rel = __builtin_amdgcn_readlane(start_l[q], t) - first_edge;
            if (rel <= 0) ++before;
            else if (rel < L) inside |= 1u << rel;
        }
    }
#pragma unroll
    for (int k = 0; k < L; ++k) rows[k] = r_first + before + __popc(inside & ((2u << k) - 1u));
    return true;
}

// Inclusive prefix sum over the 64 lanes of a wave with data-parallel-primitive moves: shifts by
// 1, 2, 4, 8 inside rows of 16 lanes, then lane 15 of a row added to the next row (rows 1 and 3) and
// lane 31 added to rows 2 and 3.
__device__ __forceinline__ int wave_inclusive_scan(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);  // row_bcast:15 into rows 1, 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);  // row_bcast:31 into rows 2, 3
    return v;
}

#endif  // __HIPCC__
}  // namespace ftc
