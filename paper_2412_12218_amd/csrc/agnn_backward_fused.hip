// Backward of the AGNN propagation layer in one pass over the edges (symmetric pattern).
//
// Forward (agnn_fused.hip): y_i = sum_e p_e h_j, p_e = a_e / z_i, a_e = exp(beta c_e - |beta|),
// c_e = <hn_i, hn_j>, z_i = sum_e a_e.  The paper names training (Sections II and V) and gives no
// gradient formulas; these are the derivatives of that definition.  With t_i = sum_e p_e dp_e
// = <dY_i, y_i> and, for the stored entry T(e) = (j, i) that a symmetric pattern holds for every
// e = (i, j), c_T(e) = c_e and a_T(e) = a_e:
//     dp_e = <dY_i, h_j>                 ds_e    = p_e (dp_e - t_i)
//     p_T(e) = a_e / z_j                 ds_T(e) = p_T(e) (<h_i, dY_j> - t_j)
//     dbeta = sum_e ds_e c_e
//     q_i   = beta sum_e (ds_e + ds_T(e)) hn_j        (gradient w.r.t. the normalised row hn_i)
//     agg_i = sum_e p_T(e) dY_j                       (through the aggregated rows)
//     dH_i  = agg_i + (q_i - hn_i <hn_i, q_i>) / |h_i|
// so one sweep that gathers h_j and dY_j once per entry, plus the per-node pair (1 / z_j, t_j),
// yields everything: no edge array (scores, probabilities, transposed index) travels through HBM.
// z comes from the forward pass (row_z of ftc_agnn_layer), t from a row-wise dot product of dY and
// the forward output.  The same row pass copies h_i and dY_i side by side into one matrix HD
// (row i = [h_i | dY_i], each half padded to DP elements): every read that leaves L2 is a 128-byte
// line, so the two 64-byte rows an entry needs cost one line instead of two.
//
// Work partition, runs and the handling of rows cut by run / wave boundaries are those of the
// edge-balanced SpMM (spmm_seg.hip): the pair (q_i, agg_i) is one output row of width 2 * DP, cut
// rows go through the same carry buffer and are finished by the SpMM fix-up kernel; a row kernel
// (backward.hip) then applies the derivative of the normalisation.
#include "ftc_common.hpp"

namespace ftc {

constexpr int BW_B = 4;  // edges per batch

bool seg_shape(int dtype, int D, int *vec, int *lpr);

// stats[i] = (1 / z_i, <dY_i, Y_i>) and HD[i] = [h_i | dY_i] (element type of H, halves of DP
// elements, zero padded).  Eight lanes per row, 16 bytes of H and dY per lane and step (the caller
// guarantees 16-byte aligned rows of H and dY).  A row without entries gets (0, 0).
template <class T>
__global__ __launch_bounds__(256) void agnn_row_stats_kernel(int n, const void *__restrict__ H,
                                                             const void *__restrict__ dY, int ld,
                                                             const void *__restrict__ Y, int ldy, int ydt, int D, int DP,
                                                             const float *__restrict__ row_z, float2 *__restrict__ stats,
                                                             void *__restrict__ HD)
{
    constexpr int V = T::VEC;  // elements per 16 bytes
    const int sub = threadIdx.x & 7;
    const int64_t row = (static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x) >> 3;
    const bool y_vec = ydt == FTC_F32 && ldy % 4 == 0 && (reinterpret_cast<uintptr_t>(Y) & 15u) == 0;
    float t = 0.f;
    if (row < n) {
        char *dst = static_cast<char *>(HD) + row * 2 * DP * T::BYTES;
        for (int k = sub * V; k < DP; k += 8 * V) {  // DP is a multiple of V
            uint4 h = make_uint4(0u, 0u, 0u, 0u), d = h;
            if (k + V <= D) {
                h = *reinterpret_cast<const uint4 *>(static_cast<const char *>(H) + (row * ld + k) * T::BYTES);
                d = *reinterpret_cast<const uint4 *>(static_cast<const char *>(dY) + (row * ld + k) * T::BYTES);
                float df[V], yf[V];
                load_vec<T>(dY, row * ld + k, df);
                if (y_vec) {
#pragma unroll
                    for (int q = 0; q < V / 4; ++q) {
                        const float4 y4 = *reinterpret_cast<const float4 *>(static_cast<const float *>(Y) + row * ldy + k + 4 * q);
                        yf[4 * q] = y4.x; yf[4 * q + 1] = y4.y; yf[4 * q + 2] = y4.z; yf[4 * q + 3] = y4.w;
                    }
                } else {
#pragma unroll
                    for (int q = 0; q < V; ++q) yf[q] = load_elem(Y, row * ldy + k + q, ydt);
                }
#pragma unroll
                for (int q = 0; q < V; ++q) t = fmaf(df[q], yf[q], t);
            } else if (k < D) {  // a ragged last piece: element by element
                uint32_t hw[4] = {0u, 0u, 0u, 0u}, dw[4] = {0u, 0u, 0u, 0u};
                for (int q = 0; k + q < D; ++q) {
                    if constexpr (T::BYTES == 4) {
                        hw[q] = static_cast<const uint32_t *>(H)[row * ld + k + q];
                        dw[q] = static_cast<const uint32_t *>(dY)[row * ld + k + q];
                    } else {
                        hw[q / 2] |= static_cast<uint32_t>(static_cast<const uint16_t *>(H)[row * ld + k + q]) << (16 * (q & 1));
                        dw[q / 2] |= static_cast<uint32_t>(static_cast<const uint16_t *>(dY)[row * ld + k + q]) << (16 * (q & 1));
                    }
                    t = fmaf(load_elem(dY, row * ld + k + q, T::BYTES == 4 ? FTC_F32 : (std::is_same<T, F16>::value ? FTC_F16 : FTC_BF16)),
                             load_elem(Y, row * ldy + k + q, ydt), t);
                }
                h = make_uint4(hw[0], hw[1], hw[2], hw[3]);
                d = make_uint4(dw[0], dw[1], dw[2], dw[3]);
            }
            *reinterpret_cast<uint4 *>(dst + k * T::BYTES) = h;
            *reinterpret_cast<uint4 *>(dst + (DP + k) * T::BYTES) = d;
        }
    }
    t += __shfl_xor(t, 1, 64);
    t += __shfl_xor(t, 2, 64);
    t += __shfl_xor(t, 4, 64);
    if (row < n && sub == 0) {
        const float z = row_z[row];
        stats[row] = make_float2(z > 0.f ? 1.f / z : 0.f, t);
    }
}

template <class T, int VEC, int LPR>
__global__ __launch_bounds__(256) void agnn_backward_fused_kernel(
    int nnz, int n_ranges, const int *__restrict__ col_idx, const int *__restrict__ edge_to_row,
    const void *__restrict__ HD, int D, float beta, const float2 *__restrict__ stats, float *__restrict__ QA,
    float *__restrict__ carry, int *__restrict__ carry_tail_row, float *__restrict__ dbeta_part)
{
    constexpr int NG = 64 / LPR;
    constexpr int RUN = SEG_R / NG;
    constexpr int RP = SEG_R + NG;
    constexpr int DP = LPR * VEC;
    constexpr int DP2 = 2 * DP;  // q slots, then agg slots
    constexpr int IDX_WORDS = 4 * 2 * RP;
    static_assert(RUN % BW_B == 0, "runs are whole batches");
    constexpr int PART_WORDS = 4 * 2 * NG * DP2;
    __shared__ int smem[IDX_WORDS > PART_WORDS ? IDX_WORDS : PART_WORDS];
    __shared__ int s_meta[4][3][NG];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int g = lane / LPR, sub = lane % LPR;
    int *s_col = smem + wave * 2 * RP;
    int *s_row = s_col + RP;

    const int v = xcd_chunked_block(blockIdx.x, gridDim.x) * 4 + wave;
    const bool active = v < n_ranges;
    const int base = active ? v * SEG_R : 0;
    const int n_valid = active ? min(SEG_R, nnz - base) : 0;
    // (the rows could come from the row starts as in the forward kernels; measured 3 % slower here)
#pragma unroll
    for (int j = 0; j < SEG_R / 64; ++j) {
        const int i = j * 64 + lane;
        if (i < n_valid) {
            const int p = i + i / RUN;
            s_col[p] = __builtin_nontemporal_load(col_idx + base + i);  // streamed once: no need to keep them in L2
            s_row[p] = __builtin_nontemporal_load(edge_to_row + base + i);
        }
    }
    const int prev_row = (active && base > 0) ? edge_to_row[base - 1] : -1;
    const int next_row = (active && n_valid == SEG_R && base + SEG_R < nnz) ? edge_to_row[base + SEG_R] : -1;
    const int far_row = (active && static_cast<int64_t>(base) + 2 * SEG_R < nnz) ? edge_to_row[base + 2 * SEG_R] : -1;
    __syncthreads();

    const int rs = g * RUN;
    const int re = min(rs + RUN, n_valid);
    const bool has = rs < n_valid;
    const bool live = sub * VEC < D;
    const float absb = fabsf(beta);
    float acc[2 * VEC], hacc[2 * VEC];  // [0, VEC): q slice, [VEC, 2 VEC): agg slice
#pragma unroll
    for (int j = 0; j < 2 * VEC; ++j) { acc[j] = 0.f; hacc[j] = 0.f; }
    RawVec<T, VEC> xi, dxi;  // slices of H[i,:] and dY[i,:] of the current row, as loaded
    zero_raw(xi);
    zero_raw(dxi);
    float ri = 0.f, zi_inv = 0.f, ti = 0.f, dbeta_acc = 0.f;
    bool have_head = false, head_closed = false, have_tail = false;
    int head_row = -1, cur = -1;
    bool first = true;
    const int left_row = !has ? -2 : (rs == 0 ? prev_row : s_row[rs - 1 + g - 1]);

    auto direct_store = [&](int row) {
        if (live) {
            float q[VEC], a[VEC];
#pragma unroll
            for (int j = 0; j < VEC; ++j) { q[j] = acc[j]; a[j] = acc[VEC + j]; }
            store_vec<VEC>(QA, static_cast<int64_t>(row) * DP2 + sub * VEC, FTC_F32, q);
            store_vec<VEC>(QA, static_cast<int64_t>(row) * DP2 + DP + sub * VEC, FTC_F32, a);
        }
    };

    // every group runs the same number of batches: the lane-group sums need the whole wave; edges
    // beyond the group's run are masked
    for (int b = rs; b < rs + RUN; b += BW_B) {
        int c[BW_B], r[BW_B];
        bool need[BW_B];
        RawVec<T, VEC> y[BW_B], dy[BW_B];
        float2 st[BW_B];
#pragma unroll
        for (int k = 0; k < BW_B; ++k) {
            const bool ok = b + k < re;
            const int p = ok ? b + k + g : 0;
            c[k] = ok ? s_col[p] : -1;
            r[k] = ok ? s_row[p] : -1;
        }
        int prev = cur;
#pragma unroll
        for (int k = 0; k < BW_B; ++k) {
            need[k] = r[k] >= 0 && r[k] != prev;
            if (r[k] >= 0) prev = r[k];
        }
#pragma unroll
        for (int k = 0; k < BW_B; ++k) {
            if (c[k] >= 0 && live) {
                load_raw<T, VEC>(HD, static_cast<int64_t>(c[k]) * DP2 + sub * VEC, y[k]);
                load_raw<T, VEC>(HD, static_cast<int64_t>(c[k]) * DP2 + DP + sub * VEC, dy[k]);
            } else {
                zero_raw(y[k]);
                zero_raw(dy[k]);
            }
            st[k] = c[k] >= 0 ? stats[c[k]] : make_float2(0.f, 0.f);
        }
#pragma unroll
        for (int k = 0; k < BW_B; ++k) {
            if (need[k]) {  // a new row starts (the lanes of a group branch together)
                if (cur >= 0) {
                    if (first && left_row == cur) {
#pragma unroll
                        for (int j = 0; j < 2 * VEC; ++j) hacc[j] = acc[j];
                        have_head = true; head_closed = true; head_row = cur;
                    } else {
                        direct_store(cur);
                    }
                    first = false;
                }
                cur = r[k];
#pragma unroll
                for (int j = 0; j < 2 * VEC; ++j) acc[j] = 0.f;
                if (live) {
                    load_raw<T, VEC>(HD, static_cast<int64_t>(cur) * DP2 + sub * VEC, xi);
                    load_raw<T, VEC>(HD, static_cast<int64_t>(cur) * DP2 + DP + sub * VEC, dxi);
                } else {
                    zero_raw(xi);
                    zero_raw(dxi);
                }
                const float2 si = stats[cur];
                zi_inv = si.x;
                ti = si.y;
                ri = __frsqrt_rn(fmaxf(group_sum_dpp<LPR>(dot_raw<T, VEC>(xi, xi, 0.f)), 1e-24f));  // 1 / max(|h_i|, 1e-12)
            }
            const float d_hh = group_sum_dpp<LPR>(dot_raw<T, VEC>(xi, y[k], 0.f));
            const float qj = group_sum_dpp<LPR>(dot_raw<T, VEC>(y[k], y[k], 0.f));
            const float dp = group_sum_dpp<LPR>(dot_raw<T, VEC>(dxi, y[k], 0.f));
            const float dpt = group_sum_dpp<LPR>(dot_raw<T, VEC>(xi, dy[k], 0.f));
            if (r[k] >= 0) {
                const float rj = __frsqrt_rn(fmaxf(qj, 1e-24f));
                const float cs = ri * rj * d_hh;
                const float a = __expf(beta * cs - absb);
                const float ds = a * zi_inv * (dp - ti);
                const float pt = a * st[k].x;
                const float dst = pt * (dpt - st[k].y);
                const float coef = beta * (ds + dst) * rj;
                float yf[VEC], dyf[VEC];
                unpack<T, VEC>(y[k], yf);
                unpack<T, VEC>(dy[k], dyf);
#pragma unroll
                for (int j = 0; j < VEC; ++j) {
                    acc[j] = fmaf(coef, yf[j], acc[j]);
                    acc[VEC + j] = fmaf(pt, dyf[j], acc[VEC + j]);
                }
                if (sub == 0) dbeta_acc = fmaf(ds, cs, dbeta_acc);
            }
        }
    }
    if (has) {  // the run's last segment
        int right_row;
        if (re < n_valid) right_row = s_row[re + g + 1];
        else right_row = next_row;
        const bool right_open = right_row == cur;
        if (first && left_row == cur) {
#pragma unroll
            for (int j = 0; j < 2 * VEC; ++j) hacc[j] = acc[j];
            have_head = true; head_closed = !right_open; head_row = cur;
        } else if (!right_open) {
            direct_store(cur);
        } else {
            have_tail = true;
        }
    }
    // the wave's share of dbeta: lanes in a fixed order
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) dbeta_acc += __shfl_xor(dbeta_acc, m, 64);
    if (active && lane == 0) dbeta_part[v] = dbeta_acc;
    __syncthreads();  // staged indices are dead: the LDS is reused for partials

    float *part = reinterpret_cast<float *>(smem) + wave * 2 * NG * DP2;
    if (have_head) {
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
            part[(2 * g) * DP2 + sub * VEC + j] = hacc[j];
            part[(2 * g) * DP2 + DP + sub * VEC + j] = hacc[VEC + j];
        }
    }
    if (have_tail) {
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
            part[(2 * g + 1) * DP2 + sub * VEC + j] = acc[j];
            part[(2 * g + 1) * DP2 + DP + sub * VEC + j] = acc[VEC + j];
        }
    }
    if (sub == 0) {
        s_meta[wave][0][g] = have_head ? head_row : -1;
        s_meta[wave][1][g] = head_closed ? 1 : 0;
        s_meta[wave][2][g] = have_tail ? cur : -1;
    }
    __syncthreads();

    // Add the pieces of rows cut inside this wave, in edge order; one lane per output slot.
    if (active) {
        int tail_out = -1;
        for (int d = lane; d < DP2; d += 64) {
            float run = 0.f;
            int run_row = -1;
            bool from_outside = false;
            tail_out = -1;
            for (int q = 0; q < NG; ++q) {
                const int hr = s_meta[wave][0][q];
                if (hr >= 0) {
                    if (run_row < 0) { run_row = hr; run = 0.f; from_outside = true; }
                    run += part[(2 * q) * DP2 + d];
                    if (s_meta[wave][1][q]) {
                        if (from_outside) carry[(static_cast<size_t>(v) * 2) * DP2 + d] = run;
                        else QA[static_cast<int64_t>(run_row) * DP2 + d] = run;
                        run_row = -1;
                        from_outside = false;
                    }
                }
                const int tr = s_meta[wave][2][q];
                if (tr >= 0) { run_row = tr; run = part[(2 * q + 1) * DP2 + d]; from_outside = false; }
            }
            if (run_row >= 0) {
                if (from_outside) {
                    carry[(static_cast<size_t>(v) * 2) * DP2 + d] = run;  // the row covers the whole wave
                } else {
                    carry[(static_cast<size_t>(v) * 2 + 1) * DP2 + d] = run;
                    tail_out = run_row;
                }
            }
        }
        if (lane == 0) {
            carry_tail_row[2 * v] = tail_out;
            carry_tail_row[2 * v + 1] = (tail_out >= 0 && far_row != tail_out) ? 1 : 0;  // ends in range v + 1
        }
    }
}

// sum of the waves' shares in a fixed order: one workgroup of 1024 threads, four loads in flight each
__global__ __launch_bounds__(1024) void dbeta_sum_kernel(int count, const float *__restrict__ partial, float *out)
{
    __shared__ float red[16];
    float t0 = 0.f, t1 = 0.f, t2 = 0.f, t3 = 0.f;
    int i = threadIdx.x;
    for (; i + 3 * 1024 < count; i += 4 * 1024) {
        t0 += partial[i];
        t1 += partial[i + 1024];
        t2 += partial[i + 2048];
        t3 += partial[i + 3072];
    }
    for (; i < count; i += 1024) t0 += partial[i];
    float t = (t0 + t1) + (t2 + t3);
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) t += __shfl_xor(t, m, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = t;
    __syncthreads();
    if (threadIdx.x == 0) {
        float a = 0.f;
        for (int w = 0; w < 16; ++w) a += red[w];
        *out = a;
    }
}

// The fused pass covers the shapes of the edge-balanced kernels whose pair (q, agg) still fits the
// 256 slots of the fix-up kernel.
bool agnn_backward_fused_shape(int dtype, int D)
{
    int vec, lpr;
    return seg_shape(dtype, D, &vec, &lpr) && 2 * vec * lpr <= 256;
}

static size_t bw_dp2(int dtype, int D)
{
    int vec = 0, lpr = 0;
    seg_shape(dtype, D, &vec, &lpr);
    return 2 * static_cast<size_t>(vec) * lpr;
}

// [QA: n x DP2 fp32 | HD: n x DP2 elements | stats: n float2 | carry | tail rows | dbeta shares], DP2 of the
// widest element type
size_t agnn_backward_fused_ws(int n, int nnz, int D)
{
    size_t dp2 = 0;
    if (agnn_backward_fused_shape(FTC_F32, D)) dp2 = bw_dp2(FTC_F32, D);
    if (agnn_backward_fused_shape(FTC_F16, D) && bw_dp2(FTC_F16, D) > dp2) dp2 = bw_dp2(FTC_F16, D);
    if (dp2 == 0) return 0;
    const size_t n_ranges = (static_cast<size_t>(nnz) + SEG_R - 1) / SEG_R;
    return 2 * align_up(static_cast<size_t>(n) * dp2 * sizeof(float), 256) + align_up(static_cast<size_t>(n) * sizeof(float2), 256) +
           align_up(n_ranges * 2 * dp2 * sizeof(float), 256) + align_up(n_ranges * 2 * sizeof(int), 256) +
           align_up(n_ranges * sizeof(float), 256);
}

template <class T>
static void launch_bw_t(int vec, int lpr, unsigned grid, hipStream_t s, int nnz, int n_ranges, const ftc_csr &g,
                        const int *e2r, const void *HD, int D, float beta, const float2 *stats, float *QA, float *carry,
                        int *tail_row, float *dbeta_part)
{
    constexpr int VM = T::VEC;
#define FTC_BW(V, L)                                                                                                \
    hipLaunchKernelGGL((agnn_backward_fused_kernel<T, V, L>), dim3(grid), dim3(256), 0, s, nnz, n_ranges, g.col_idx, \
                       e2r, HD, D, beta, stats, QA, carry, tail_row, dbeta_part)
    if (vec == VM) {
        if (lpr == 4) FTC_BW(VM, 4);
        else if (lpr == 8) FTC_BW(VM, 8);
        else if (lpr == 16) FTC_BW(VM, 16);
        else FTC_BW(VM, 32);
    } else if (vec == VM / 2) {
        FTC_BW(VM / 2, 4);
    } else {
        FTC_BW(VM / 4, 4);
    }
#undef FTC_BW
}

// Caller has checked: window index present, agnn_backward_fused_shape(dt, D), rows of H and dY
// 16-byte aligned with the same leading dimension, workspace of agnn_backward_fused_ws() bytes.
int32_t launch_agnn_backward_fused(const ftc_csr &g, const ftc_windows &w, const void *H, const void *dY, int ld, int dt,
                                   int D, float beta, const float *row_z, const void *Y, int ldy, int ydt, void *dH,
                                   int lddh, int dh_dt, float *dbeta, void *ws, hipStream_t s)
{
    int vec = 0, lpr = 0;
    seg_shape(dt, D, &vec, &lpr);
    const int dp = vec * lpr, dp2 = 2 * dp;
    const int n = g.n;
    const int n_ranges = ceil_div(g.nnz, SEG_R);
    char *p = static_cast<char *>(ws);
    float *QA = reinterpret_cast<float *>(p);
    p += align_up(static_cast<size_t>(n) * dp2 * sizeof(float), 256);
    void *HD = p;
    p += align_up(static_cast<size_t>(n) * dp2 * sizeof(float), 256);
    float2 *stats = reinterpret_cast<float2 *>(p);
    p += align_up(static_cast<size_t>(n) * sizeof(float2), 256);
    float *carry = reinterpret_cast<float *>(p);
    p += align_up(static_cast<size_t>(n_ranges) * 2 * dp2 * sizeof(float), 256);
    int *tail_row = reinterpret_cast<int *>(p);
    p += align_up(static_cast<size_t>(n_ranges) * 2 * sizeof(int), 256);
    float *dbeta_part = reinterpret_cast<float *>(p);

    const unsigned grid_rows8 = static_cast<unsigned>((static_cast<int64_t>(n) * 8 + 255) / 256);
    if (dt == FTC_F32)
        hipLaunchKernelGGL(agnn_row_stats_kernel<F32>, dim3(grid_rows8), dim3(256), 0, s, n, H, dY, ld, Y, ldy, ydt, D, dp,
                           row_z, stats, HD);
    else if (dt == FTC_F16)
        hipLaunchKernelGGL(agnn_row_stats_kernel<F16>, dim3(grid_rows8), dim3(256), 0, s, n, H, dY, ld, Y, ldy, ydt, D, dp,
                           row_z, stats, HD);
    else
        hipLaunchKernelGGL(agnn_row_stats_kernel<BF16>, dim3(grid_rows8), dim3(256), 0, s, n, H, dY, ld, Y, ldy, ydt, D, dp,
                           row_z, stats, HD);
    if (n_ranges > 0) {
        const unsigned grid = static_cast<unsigned>((n_ranges + 3) / 4);
        if (dt == FTC_F32)
            launch_bw_t<F32>(vec, lpr, grid, s, g.nnz, n_ranges, g, w.edge_to_row, HD, D, beta, stats, QA, carry, tail_row,
                             dbeta_part);
        else if (dt == FTC_F16)
            launch_bw_t<F16>(vec, lpr, grid, s, g.nnz, n_ranges, g, w.edge_to_row, HD, D, beta, stats, QA, carry, tail_row,
                             dbeta_part);
        else
            launch_bw_t<BF16>(vec, lpr, grid, s, g.nnz, n_ranges, g, w.edge_to_row, HD, D, beta, stats, QA, carry, tail_row,
                              dbeta_part);
        const int32_t st = launch_status("agnn_backward_fused");
        if (st != FTC_OK) return st;
    }
    // rows cut by wave boundaries and rows without entries: the SpMM fix-up on the 2 * DP wide rows
    int32_t st = launch_seg_fixup(n, n_ranges, g.row_ptr, carry, tail_row, dp2, dp2, QA, dp2, FTC_F32, Epi{0, nullptr},
                                  nullptr, SEG_R, s, "agnn_backward_fused fixup");
    if (st != FTC_OK) return st;
    hipLaunchKernelGGL(dbeta_sum_kernel, dim3(1), dim3(1024), 0, s, n_ranges, dbeta_part, dbeta);
    st = launch_status("agnn_backward_fused dbeta");
    if (st != FTC_OK) return st;
    // dH = agg + (q - hn <hn, q>) / |h|, rounded once to the requested type
    float *rinv = reinterpret_cast<float *>(stats);  // the pairs are dead: their array takes the inverse norms
    st = launch_row_rnorm(n, H, ld, dt, D, rinv, s);
    if (st != FTC_OK) return st;
    return launch_cos_backward_rows(n, H, ld, dt, D, rinv, QA, dp2, QA + dp, dp2, dH, lddh, dh_dt, s);
}

}  // namespace ftc
