// Sparse neighbour aggregation (SpMM, Section V.A) for narrow feature rows: at most 32 bytes per
// row (D <= 16 for 16-bit features, D <= 8 for fp32), the widths of the GCN hidden and output layers.
//
// The edge-balanced kernel of spmm_seg.hip puts four lanes on a row; with rows this narrow a lane
// then loads 4 or 8 bytes per edge and the per-edge bookkeeping outweighs the arithmetic.  Here a
// SLOT of LPE lanes owns SL_L consecutive edges, and each of its lanes loads one 16-byte piece of
// every row (LPE = 1: rows of 16 bytes; LPE = 2: rows of 32 bytes, the two halves in neighbouring
// lanes, so that a load instruction touches one contiguous segment per edge -- two loads per lane
// for the two halves were measured slower than the four-lane layout, 0.35 against 0.30 ms on the
// R-MAT benchmark graph: what costs is the number of separate segments a load instruction touches):
//   - the slot gathers the rows of its edges, eight loads in flight, and accumulates while the
//     output row stays the same; a row that begins and ends inside the slot is stored at once;
//   - the pieces of rows that continue from slot to slot are joined by ONE segmented scan over the
//     wave (data-parallel-primitive moves or lane shuffles, the row beginnings are the segment heads);
//   - the pieces of rows cut by a wave boundary go to the carry buffer of the edge-balanced
//     kernels and are finished by their fix-up kernel, in edge order.
// No floating-point atomics, no LDS: results are reproducible bit for bit.
#include "ftc_common.hpp"

namespace ftc {

constexpr int SL_L = 16;         // consecutive edges per lane
constexpr int SL_R = 64 * SL_L;  // edges per wave
constexpr int SL_B = 8;          // gathers issued together

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int sl_dpp(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, CTRL, ROW_MASK, 0xf, false);
}

// Segmented inclusive scan (sum) of N floats per lane over the lanes of a wave; head != 0 marks the
// first lane of a segment.  Shifts by 1, 2, 4, 8 inside rows of 16 lanes, then lane 15 of a row into
// the next row (rows 1 and 3) and lane 31 into rows 2 and 3; a lane stops taking from the left once
// a head lies in its span.
template <int N>
__device__ __forceinline__ void wave_segmented_sum(float (&x)[N], int head, int lane)
{
#define FTC_STEP(CTRL, ROW_MASK, VALID)                                                          \
    {                                                                                            \
        const int yh = sl_dpp<CTRL, ROW_MASK>(head);                                             \
        _Pragma("unroll") for (int j = 0; j < N; ++j)                                            \
        {                                                                                        \
            const float y = __int_as_float(sl_dpp<CTRL, ROW_MASK>(__float_as_int(x[j])));        \
            if ((VALID) && !head) x[j] += y;                                                     \
        }                                                                                        \
        if (VALID) head |= yh;                                                                   \
    }
    const int r16 = lane & 15;
    FTC_STEP(0x111, 0xf, r16 >= 1)
    FTC_STEP(0x112, 0xf, r16 >= 2)
    FTC_STEP(0x114, 0xf, r16 >= 4)
    FTC_STEP(0x118, 0xf, r16 >= 8)
    FTC_STEP(0x142, 0xa, (lane & 16) != 0)
    FTC_STEP(0x143, 0xc, lane >= 32)
#undef FTC_STEP
}

// Shuffle-based variant of the scan for slots of LPE lanes (a slot's lanes hold different pieces of the
// same rows and share the head flag): Kogge-Stone steps over distances of LPE, 2 LPE, ... lanes.
template <int N, int LPE>
__device__ __forceinline__ void wave_segmented_sum_slots(float (&x)[N], int head, int lane)
{
#pragma unroll
    for (int d = LPE; d < 64; d <<= 1) {
        const int yh = __shfl_up(head, d, 64);
        float y[N];
#pragma unroll
        for (int j = 0; j < N; ++j) y[j] = __shfl_up(x[j], d, 64);
        if (lane >= d) {
            if (!head) {
#pragma unroll
                for (int j = 0; j < N; ++j) x[j] += y[j];
            }
            head |= yh;
        }
    }
}

// LPE: lanes per edge (1: rows of one 16-byte piece; 2: rows of two pieces, neighbouring lanes load the two
// halves of a row, so a load instruction still touches one contiguous 32-byte segment per edge).
// VALS = false: all edge values are one.
template <class T, int LPE, bool VALS>
__global__ __launch_bounds__(256) void spmm_lane_kernel(int nnz, int n_ranges, const int *__restrict__ row_ptr,
                                                        const int *__restrict__ col_idx,
                                                        const int *__restrict__ edge_to_row,
                                                        const float *__restrict__ vals, const void *__restrict__ X,
                                                        int ldx, int D, void *__restrict__ out, int ldo, int odt, Epi epi,
                                                        float *__restrict__ carry, int *__restrict__ carry_tail_row,
                                                        int idx_vec, int out_vec)
{
    constexpr int V = T::VEC, DP = V, NV = 1;  // a lane holds one 16-byte piece of its rows
    constexpr int DPT = V * LPE;               // padded row width (carry rows)
    constexpr int RANGE = SL_R / LPE;          // edges per wave
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int slot = lane / LPE, piece = lane % LPE;
    const int v = xcd_chunked_block(blockIdx.x, gridDim.x) * 4 + wave;
    if (v >= n_ranges) return;  // no workgroup barrier below
    const int base = v * RANGE;
    const int n_valid = min(RANGE, nnz - base);
    const int prev_row = base > 0 ? edge_to_row[base - 1] : -1;
    const int next_row = base + n_valid < nnz ? edge_to_row[base + n_valid] : -1;
    const int far_row = static_cast<int64_t>(base) + 2 * RANGE < nnz ? edge_to_row[base + 2 * RANGE] : -1;
    const int e0 = slot * SL_L;
    int c[SL_L], r[SL_L];
    float a[VALS ? SL_L : 1];
    if (idx_vec && n_valid == RANGE) {
#pragma unroll
        for (int q = 0; q < SL_L / 4; ++q) {
            const int4 c4 = *reinterpret_cast<const int4 *>(col_idx + base + e0 + 4 * q);
            c[4 * q] = c4.x; c[4 * q + 1] = c4.y; c[4 * q + 2] = c4.z; c[4 * q + 3] = c4.w;
            if constexpr (VALS) {
                const float4 a4 = *reinterpret_cast<const float4 *>(vals + base + e0 + 4 * q);
                a[4 * q] = a4.x; a[4 * q + 1] = a4.y; a[4 * q + 2] = a4.z; a[4 * q + 3] = a4.w;
            }
        }
        // the rows of the lane's edges: from the row starts of the range where that works, else the per-entry stream
        if (!lane_rows_from_starts<SL_L>(row_ptr, edge_to_row, base, RANGE, e0, lane, r)) {
#pragma unroll
            for (int q = 0; q < SL_L / 4; ++q) {
                const int4 r4 = *reinterpret_cast<const int4 *>(edge_to_row + base + e0 + 4 * q);
                r[4 * q] = r4.x; r[4 * q + 1] = r4.y; r[4 * q + 2] = r4.z; r[4 * q + 3] = r4.w;
            }
        }
    } else {
#pragma unroll
        for (int k = 0; k < SL_L; ++k) {
            const bool ok = e0 + k < n_valid;
            c[k] = ok ? col_idx[base + e0 + k] : -1;
            r[k] = ok ? edge_to_row[base + e0 + k] : -2 - (e0 + k);  // padding: rows of their own, never stored
            if constexpr (VALS) a[k] = ok ? vals[base + e0 + k] : 0.f;
        }
    }
    int left;  // row of the edge before the slot's first
    if constexpr (LPE == 1) left = sl_dpp<0x138, 0xf>(r[SL_L - 1]);  // wave_shr:1
    else left = __shfl_up(r[SL_L - 1], LPE, 64);
    if (slot == 0) left = prev_row;

    auto store_row = [&](int row, const float(&s)[DP]) {
        if (row < 0) return;
        const float f = epi.factor(row);
        float o[DP];
#pragma unroll
        for (int j = 0; j < DP; ++j) o[j] = epi.apply(f, s[j]);
        if (out_vec) {  // D == DPT, rows of out 16-byte aligned
#pragma unroll
            for (int j = 0; j < DP; j += 4) {
                const float o4[4] = {o[j], o[j + 1], o[j + 2], o[j + 3]};
                store_vec<4>(out, static_cast<int64_t>(row) * ldo + piece * V + j, odt, o4);
            }
        } else {
#pragma unroll
            for (int j = 0; j < DP; ++j)
                if (piece * V + j < D) store_elem(out, static_cast<int64_t>(row) * ldo + piece * V + j, odt, o[j]);
        }
    };

    float acc[DP], first_piece[DP];
#pragma unroll
    for (int j = 0; j < DP; ++j) { acc[j] = 0.f; first_piece[j] = 0.f; }
    int nb = 0;  // row beginnings inside the slot
#pragma unroll
    for (int h = 0; h < SL_L / SL_B; ++h) {
        RawVec<T, V> y[SL_B][NV];
#pragma unroll
        for (int k = 0; k < SL_B; ++k) {
            const int ck = c[h * SL_B + k];
#pragma unroll
            for (int q = 0; q < NV; ++q) {
                if (ck >= 0) load_raw<T, V>(X, static_cast<int64_t>(ck) * ldx + piece * V + q * V, y[k][q]);
                else zero_raw(y[k][q]);
            }
        }
#pragma unroll
        for (int k = 0; k < SL_B; ++k) {
            const int i = h * SL_B + k;
            const int before = i == 0 ? left : r[i - 1];
            if (r[i] != before) {  // a row begins: the piece so far is finished
                if (nb == 0) {
#pragma unroll
                    for (int j = 0; j < DP; ++j) first_piece[j] = acc[j];  // joined with the lanes on the left below
                } else {
                    store_row(before, acc);  // began and ended inside this lane
                }
                ++nb;
#pragma unroll
                for (int j = 0; j < DP; ++j) acc[j] = 0.f;
            }
            if (c[i] >= 0) {
#pragma unroll
                for (int q = 0; q < NV; ++q) {
                    float yf[V];
                    unpack<T, V>(y[k][q], yf);
#pragma unroll
                    for (int j = 0; j < V; ++j) {
                        if constexpr (VALS) acc[q * V + j] = fmaf(a[i], yf[j], acc[q * V + j]);
                        else acc[q * V + j] += yf[j];
                    }
                }
            }
        }
    }
    if (nb == 0) {
#pragma unroll
        for (int j = 0; j < DP; ++j) first_piece[j] = acc[j];
    }
    // one segmented scan joins the lanes' last (or only) pieces
    float incl[DP];
#pragma unroll
    for (int j = 0; j < DP; ++j) incl[j] = acc[j];
    if constexpr (LPE == 1) wave_segmented_sum<DP>(incl, nb > 0 ? 1 : 0, lane);
    else wave_segmented_sum_slots<DP, LPE>(incl, nb > 0 ? 1 : 0, lane);
    // what flows into a slot from the left (every lane takes part in the shift)
    float t[DP];
#pragma unroll
    for (int j = 0; j < DP; ++j) {
        float fl;
        if constexpr (LPE == 1) fl = __int_as_float(sl_dpp<0x138, 0xf>(__float_as_int(incl[j])));  // wave_shr:1
        else fl = __shfl_up(incl[j], LPE, 64);
        if (slot == 0) fl = 0.f;
        t[j] = fl + first_piece[j];
    }
    float *carry_head = carry + (static_cast<size_t>(v) * 2) * DPT + piece * V;
    float *carry_tail = carry + (static_cast<size_t>(v) * 2 + 1) * DPT + piece * V;
    if (nb > 0) {  // the row that was open at the slot's start ends at the slot's first beginning
        if (left == prev_row) {  // it entered the wave from the left: the wave's head piece
#pragma unroll
            for (int j = 0; j < DP; ++j) carry_head[j] = t[j];
        } else {
            store_row(left, t);
        }
    }
    const bool any_begin = __builtin_amdgcn_ballot_w64(nb > 0) != 0ull;
    if (slot == 64 / LPE - 1) {  // the last slot holds the wave's last row
        const int last_row = r[SL_L - 1];
        const bool right_open = n_valid == RANGE && next_row == last_row;
        int tail_out = -1;
        if (!any_begin) {  // one row covers the whole wave (it entered from the left)
#pragma unroll
            for (int j = 0; j < DP; ++j) carry_head[j] = incl[j];
        } else if (right_open) {
#pragma unroll
            for (int j = 0; j < DP; ++j) carry_tail[j] = incl[j];
            tail_out = last_row;
        } else {
            store_row(last_row, incl);  // the last row ends with the wave
        }
        if (piece == 0) {
            carry_tail_row[2 * v] = tail_out;
            carry_tail_row[2 * v + 1] = (tail_out >= 0 && far_row != tail_out) ? 1 : 0;  // ends in range v + 1
        }
    }
}

// Row widths this kernel takes: one or two 16-byte pieces, rows of X at least that long.
bool spmm_lane_shape(int xdt, int D, int ldx)
{
    const int per = xdt == FTC_F32 ? 4 : 8;
    const int lpe = (D + per - 1) / per;
    return D >= 1 && lpe <= 2 && ldx >= lpe * per;
}

size_t spmm_lane_ws(int nnz)
{
    if (nnz == 0) return 0;
    const size_t n_ranges = (static_cast<size_t>(nnz) + SL_R / 2 - 1) / (SL_R / 2);  // the shorter ranges of LPE = 2
    return align_up(n_ranges * 2 * 16 * sizeof(float), 256) + align_up(n_ranges * 2 * sizeof(int), 256);
}

template <class T>
static void launch_lane_t(int lpe, unsigned grid, hipStream_t s, int nnz, int n_ranges, const ftc_csr &g, const int *e2r,
                          const float *vals, const void *X, int ldx, int D, void *out, int ldo, int odt, Epi epi,
                          float *carry, int *tail_row, int idx_vec, int out_vec)
{
#define FTC_LANE(LPE, VALS)                                                                                         \
    hipLaunchKernelGGL((spmm_lane_kernel<T, LPE, VALS>), dim3(grid), dim3(256), 0, s, nnz, n_ranges, g.row_ptr, g.col_idx, e2r, \
                       vals, X, ldx, D, out, ldo, odt, epi, carry, tail_row, idx_vec, out_vec)
    if (lpe == 1) {
        if (vals) FTC_LANE(1, true);
        else FTC_LANE(1, false);
    } else {
        if (vals) FTC_LANE(2, true);
        else FTC_LANE(2, false);
    }
#undef FTC_LANE
}

// Caller has checked: window index present, spmm_lane_shape(), rows of X 16-byte aligned, workspace
// of spmm_lane_ws() bytes.
int32_t launch_spmm_lane(const ftc_csr &g, const ftc_windows &w, const float *vals, const void *X, int ldx, int xdt,
                         int D, void *out, int ldo, int odt, Epi epi, void *ws, hipStream_t s)
{
    const int per = xdt == FTC_F32 ? 4 : 8;
    const int lpe = (D + per - 1) / per, dp = per * lpe, range = SL_R / lpe;
    const int n_ranges = ceil_div(g.nnz, range);
    float *carry = static_cast<float *>(ws);
    int *tail_row = reinterpret_cast<int *>(static_cast<char *>(ws) +
                                            align_up(static_cast<size_t>(n_ranges) * 2 * dp * sizeof(float), 256));
    const int idx_vec = aligned16(g.col_idx) && aligned16(w.edge_to_row) && (!vals || aligned16(vals));
    const int out_vec = D == dp && aligned16(out) && (static_cast<int64_t>(ldo) * elem_size(odt)) % 16 == 0;
    if (n_ranges > 0) {
        const unsigned grid = static_cast<unsigned>((n_ranges + 3) / 4);
        if (xdt == FTC_F32)
            launch_lane_t<F32>(lpe, grid, s, g.nnz, n_ranges, g, w.edge_to_row, vals, X, ldx, D, out, ldo, odt, epi, carry,
                               tail_row, idx_vec, out_vec);
        else if (xdt == FTC_F16)
            launch_lane_t<F16>(lpe, grid, s, g.nnz, n_ranges, g, w.edge_to_row, vals, X, ldx, D, out, ldo, odt, epi, carry,
                               tail_row, idx_vec, out_vec);
        else
            launch_lane_t<BF16>(lpe, grid, s, g.nnz, n_ranges, g, w.edge_to_row, vals, X, ldx, D, out, ldo, odt, epi, carry,
                                tail_row, idx_vec, out_vec);
        const int32_t st = launch_status("spmm_lane");
        if (st != FTC_OK) return st;
    }
    return launch_seg_fixup(g.n, n_ranges, g.row_ptr, carry, tail_row, dp, D, out, ldo, odt, epi, nullptr, range, s,
                            "spmm_lane fixup");
}

}  // namespace ftc
