// AGNN propagation layer in one pass over the edges: edge scores (SDDMM), edge softmax and the
// weighted aggregation (SpMM) fused, so every neighbour row H[j,:] is gathered once per edge
// instead of twice and neither scores nor probabilities travel through HBM.
//
//   out[i,:] = sum_j w_ij H[j,:] / sum_j w_ij,   w_ij = exp(beta * cos(h_i, h_j) - |beta|)
//
// |cos| <= 1, so |beta| is an upper bound of every score of every row: shifting by it instead of
// by the row maximum gives the same softmax (numerator and denominator carry the same factor)
// and makes the pass single-sweep: numerator vector and denominator are plain segmented sums.
// Safe while exp(-2|beta|) is a normal fp32 number (|beta| < 43).
//
// The row norms of the cosine are recomputed from the row slices that are in registers anyway
// (a second DPP reduction in the lane group), so the pass needs no array of inverse norms and no
// random 4-byte gather per edge.
//
// Work partition, run structure and the handling of rows cut by run / wave boundaries are
// those of the edge-balanced SpMM (spmm_seg.hip): 512 edges per wave staged in LDS, groups of
// LPR lanes walk contiguous runs, complete rows are stored from registers, cut rows are summed
// in edge order in LDS and through a carry buffer.  The partial of a cut row is the pair
// (numerator vector, denominator); the division happens once all pieces are added.
#include "ftc_common.hpp"

namespace ftc {

constexpr int AG_R = SEG_R;  // edges per wave
constexpr int AG_B = 4;    // edges per batch

bool seg_shape(int dtype, int D, int *vec, int *lpr);

size_t agnn_fused_ws(int nnz, int D)
{
    int vec, lpr, dp = 0;
    if (seg_shape(FTC_F32, D, &vec, &lpr)) dp = vec * lpr;
    if (seg_shape(FTC_F16, D, &vec, &lpr) && vec * lpr > dp) dp = vec * lpr;
    if (dp == 0 || nnz == 0) return 0;
    const size_t n_ranges = (static_cast<size_t>(nnz) + AG_R - 1) / AG_R;
    return align_up(n_ranges * 2 * (dp + 4) * sizeof(float), 256) + align_up(n_ranges * 2 * sizeof(int), 256);
}

// KEEP: also write what the backward pass needs (row_z, out32); compiled out of the inference kernel.
template <class T, int VEC, int LPR, bool KEEP>
__global__ __launch_bounds__(256) void agnn_fused_kernel(int nnz, int n_ranges, const int *__restrict__ row_ptr,
                                                         const int *__restrict__ col_idx,
                                                         const int *__restrict__ edge_to_row,
                                                         const void *__restrict__ H, int ld, int D, float beta,
                                                         void *__restrict__ out, int ldo, int odt,
                                                         float *__restrict__ carry, int *__restrict__ carry_tail_row,
                                                         float *__restrict__ row_z, float *__restrict__ out32,
                                                         int ld32)
{
    constexpr int NG = 64 / LPR;
    constexpr int RUN = AG_R / NG;
    constexpr int RP = AG_R + NG;
    constexpr int DP = LPR * VEC;
    constexpr int DPZ = DP + 4;  // feature slots, then the denominator
    constexpr int IDX_WORDS = 4 * 2 * RP;
    static_assert(RUN % AG_B == 0, "runs are whole batches");
    constexpr int PART_WORDS = 4 * 2 * NG * DPZ;
    __shared__ int smem[IDX_WORDS > PART_WORDS ? IDX_WORDS : PART_WORDS];
    __shared__ int s_meta[4][3][NG];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int g = lane / LPR, sub = lane % LPR;
    int *s_col = smem + wave * 2 * RP;
    int *s_row = s_col + RP;

    const int v = xcd_chunked_block(blockIdx.x, gridDim.x) * 4 + wave;
    const bool active = v < n_ranges;
    const int base = active ? v * AG_R : 0;
    const int n_valid = active ? min(AG_R, nnz - base) : 0;
    int rows[AG_R / 64];
    if (n_valid == AG_R && rows_from_starts<AG_R>(row_ptr, edge_to_row, base, lane, rows)) {
#pragma unroll
        for (int j = 0; j < AG_R / 64; ++j) {
            const int i = j * 64 + lane;
            const int p = i + i / RUN;
            s_col[p] = __builtin_nontemporal_load(col_idx + base + i);  // streamed once: no need to keep it in L2
            s_row[p] = rows[j];
        }
    } else {
#pragma unroll
        for (int j = 0; j < AG_R / 64; ++j) {
            const int i = j * 64 + lane;
            if (i < n_valid) {
                const int p = i + i / RUN;
                s_col[p] = __builtin_nontemporal_load(col_idx + base + i);  // streamed once: no need to keep it in L2
                s_row[p] = __builtin_nontemporal_load(edge_to_row + base + i);
            }
        }
    }
    const int prev_row = (active && base > 0) ? edge_to_row[base - 1] : -1;
    const int next_row = (active && n_valid == AG_R && base + AG_R < nnz) ? edge_to_row[base + AG_R] : -1;
    // row of the first edge after the NEXT range: tells whether a row left open here ends there
    const int far_row = (active && static_cast<int64_t>(base) + 2 * AG_R < nnz) ? edge_to_row[base + 2 * AG_R] : -1;
    __syncthreads();

    const int rs = g * RUN;
    const int re = min(rs + RUN, n_valid);
    const bool has = rs < n_valid;
    const bool live = sub * VEC < D;
    const float absb = fabsf(beta);
    float acc[VEC], hacc[VEC];
#pragma unroll
    for (int j = 0; j < VEC; ++j) { acc[j] = 0.f; hacc[j] = 0.f; }
    RawVec<T, VEC> xi;  // slice of H[i,:] of the current row, as loaded
    zero_raw(xi);
    float z = 0.f, hz = 0.f, ri = 0.f;
    bool have_head = false, head_closed = false, have_tail = false;
    int head_row = -1, cur = -1;
    bool first = true;
    const int left_row = !has ? -2 : (rs == 0 ? prev_row : s_row[rs - 1 + g - 1]);

    auto direct_store = [&](int row) {
        if (live) {
            const float inv = __builtin_amdgcn_rcpf(z);  // v_rcp_f32: one ulp, one instruction
            float o[VEC];
#pragma unroll
            for (int j = 0; j < VEC; ++j) o[j] = acc[j] * inv;
            store_vec_nt<VEC>(out, static_cast<int64_t>(row) * ldo + sub * VEC, odt, o);
            if constexpr (KEEP)
                if (out32) store_vec<VEC>(out32, static_cast<int64_t>(row) * ld32 + sub * VEC, FTC_F32, o);  // unrounded copy
        }
        if constexpr (KEEP)
            if (row_z && sub == 0) row_z[row] = z;  // softmax denominator (shifted by |beta|), kept for the backward pass
    };

    // every group runs the same number of batches: the lane shuffles of the dot product need the
    // whole wave; edges beyond the group's run are masked.  (Issuing the next batch's gathers before
    // consuming the current one was tried: the extra registers cost more occupancy than the
    // overlap gains.)
    for (int b = rs; b < rs + RUN; b += AG_B) {
        int c[AG_B], r[AG_B];
        bool need[AG_B];
        RawVec<T, VEC> y[AG_B], xs[AG_B];
#pragma unroll
        for (int k = 0; k < AG_B; ++k) {
            const bool ok = b + k < re;
            const int p = ok ? b + k + g : 0;
            c[k] = ok ? s_col[p] : -1;
            r[k] = ok ? s_row[p] : -1;
        }
        int prev = cur;
#pragma unroll
        for (int k = 0; k < AG_B; ++k) {
            need[k] = r[k] >= 0 && r[k] != prev;
            if (r[k] >= 0) prev = r[k];
        }
#pragma unroll
        for (int k = 0; k < AG_B; ++k) {
            if (c[k] >= 0 && live) load_raw<T, VEC>(H, static_cast<int64_t>(c[k]) * ld + sub * VEC, y[k]);
            else zero_raw(y[k]);
            if (need[k] && live) load_raw<T, VEC>(H, static_cast<int64_t>(r[k]) * ld + sub * VEC, xs[k]);
            else zero_raw(xs[k]);
        }
#pragma unroll
        for (int k = 0; k < AG_B; ++k) {
            if (need[k]) {  // a new row starts: close the segment of the previous one
                if (cur >= 0) {
                    if (first && left_row == cur) {
#pragma unroll
                        for (int j = 0; j < VEC; ++j) hacc[j] = acc[j];
                        hz = z;
                        have_head = true; head_closed = true; head_row = cur;
                    } else {
                        direct_store(cur);
                    }
                    first = false;
                }
                cur = r[k];
#pragma unroll
                for (int j = 0; j < VEC; ++j) acc[j] = 0.f;
                z = 0.f;
                xi = xs[k];
                const float q = group_sum_dpp<LPR>(dot_raw<T, VEC>(xi, xi, 0.f));  // the group's lanes branch together
                ri = __frsqrt_rn(fmaxf(q, 1e-24f));  // = 1 / max(||h_i||, 1e-12)
            }
            const float d = group_sum_dpp<LPR>(dot_raw<T, VEC>(xi, y[k], 0.f));
            const float qj = group_sum_dpp<LPR>(dot_raw<T, VEC>(y[k], y[k], 0.f));
            if (r[k] >= 0) {
                const float rj = __frsqrt_rn(fmaxf(qj, 1e-24f));
                const float wgt = __expf(beta * ri * rj * d - absb);
                float yf[VEC];
                unpack<T, VEC>(y[k], yf);
#pragma unroll
                for (int j = 0; j < VEC; ++j) acc[j] = fmaf(wgt, yf[j], acc[j]);
                z += wgt;
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
            for (int j = 0; j < VEC; ++j) hacc[j] = acc[j];
            hz = z;
            have_head = true; head_closed = !right_open; head_row = cur;
        } else if (!right_open) {
            direct_store(cur);
        } else {
            have_tail = true;
        }
    }
    __syncthreads();  // staged indices are dead: the LDS is reused for partials

    float *part = reinterpret_cast<float *>(smem) + wave * 2 * NG * DPZ;
    if (have_head) {
#pragma unroll
        for (int j = 0; j < VEC; ++j) part[(2 * g) * DPZ + sub * VEC + j] = hacc[j];
        if (sub == 0) part[(2 * g) * DPZ + DP] = hz;
    }
    if (have_tail) {
#pragma unroll
        for (int j = 0; j < VEC; ++j) part[(2 * g + 1) * DPZ + sub * VEC + j] = acc[j];
        if (sub == 0) part[(2 * g + 1) * DPZ + DP] = z;
    }
    if (sub == 0) {
        s_meta[wave][0][g] = have_head ? head_row : -1;
        s_meta[wave][1][g] = head_closed ? 1 : 0;
        s_meta[wave][2][g] = have_tail ? cur : -1;
    }
    __syncthreads();

    if (active) {
        int tail_out = -1;
        for (int d = lane; d < DP; d += 64) {
            float run = 0.f, run_z = 0.f;
            int run_row = -1;
            bool from_outside = false;
            tail_out = -1;
            float *cv = carry + (static_cast<size_t>(v) * 2) * DPZ;
            for (int q = 0; q < NG; ++q) {
                const int hr = s_meta[wave][0][q];
                if (hr >= 0) {
                    if (run_row < 0) { run_row = hr; run = 0.f; run_z = 0.f; from_outside = true; }
                    run += part[(2 * q) * DPZ + d];
                    run_z += part[(2 * q) * DPZ + DP];
                    if (s_meta[wave][1][q]) {
                        if (from_outside) {
                            cv[d] = run;
                            if (d == 0) cv[DP] = run_z;
                        } else {
                            if (d < D) store_elem(out, static_cast<int64_t>(run_row) * ldo + d, odt, run / run_z);
                            if constexpr (KEEP) {
                                if (out32 && d < D) out32[static_cast<int64_t>(run_row) * ld32 + d] = run / run_z;
                                if (row_z && d == 0) row_z[run_row] = run_z;
                            }
                        }
                        run_row = -1;
                        from_outside = false;
                    }
                }
                const int tr = s_meta[wave][2][q];
                if (tr >= 0) {
                    run_row = tr;
                    run = part[(2 * q + 1) * DPZ + d];
                    run_z = part[(2 * q + 1) * DPZ + DP];
                    from_outside = false;
                }
            }
            if (run_row >= 0) {
                if (from_outside) {
                    cv[d] = run;
                    if (d == 0) cv[DP] = run_z;
                } else {
                    cv[DPZ + d] = run;
                    if (d == 0) cv[DPZ + DP] = run_z;
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

// G lanes (four features each) finish one cut row, 64 / G rows per wave: the kernel is a chain of two dependent
// loads per row (the range's record, then the two pieces), so it is the number of rows in flight that counts.
template <int G>
__global__ __launch_bounds__(256) void agnn_fused_fixup_kernel(int n, int n_ranges, const int *__restrict__ row_ptr,
                                                               const float *__restrict__ carry,
                                                               const int *__restrict__ carry_tail_row, int DP,
                                                               int D, void *__restrict__ out, int ldo, int odt,
                                                               float *__restrict__ row_z, float *__restrict__ out32,
                                                               int ld32)
{
    constexpr int R = 64 / G;  // ranges per wave
    const int DPZ = DP + 4;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int sub = lane % G;
    const int v_mine = (blockIdx.x * 4 + wave) * R + lane / G;
    int2 rec = make_int2(-1, 0);
    if (v_mine < n_ranges) rec = reinterpret_cast<const int2 *>(carry_tail_row)[v_mine];
    // Nearly every open row ends in the next range: numerator and denominator are the head piece of range
    // v + 1 plus the tail piece of range v.  Their addresses depend on v alone, so they are loaded together
    // with the range's record instead of after it.
    {
        const bool ok = v_mine + 1 < n_ranges && sub * 4 < DP;
        const size_t vv = ok ? static_cast<size_t>(v_mine) : 0;
        const float *hv = carry + (vv + 1) * 2 * DPZ;
        const float *tv = carry + (vv * 2 + 1) * DPZ;
        float4 h4 = make_float4(0.f, 0.f, 0.f, 0.f), t4 = h4;
        float spec_z = 1.f;
        if (ok) {
            h4 = *reinterpret_cast<const float4 *>(hv + sub * 4);
            t4 = *reinterpret_cast<const float4 *>(tv + sub * 4);
            spec_z = hv[DP] + tv[DP];
        }
        const int r = rec.x;
        if (ok && r >= 0 && rec.y && sub * 4 < D) {
            const float o[4] = {(h4.x + t4.x) / spec_z, (h4.y + t4.y) / spec_z, (h4.z + t4.z) / spec_z,
                                (h4.w + t4.w) / spec_z};
            store_vec<4>(out, static_cast<int64_t>(r) * ldo + sub * 4, odt, o);
            if (out32) store_vec<4>(out32, static_cast<int64_t>(r) * ld32 + sub * 4, FTC_F32, o);
        }
        if (ok && r >= 0 && rec.y && row_z && sub == 0) row_z[r] = spec_z;
    }
    // rows that go on beyond the next range (long rows of a power-law graph): one at a time, by the whole wave
    unsigned long long longs = __builtin_amdgcn_ballot_w64(rec.x >= 0 && !rec.y && sub == 0);
    while (longs) {
        const int src = __ffsll(static_cast<long long>(longs)) - 1;
        longs &= longs - 1;
        const int v = __shfl(v_mine, src, 64), r = __shfl(rec.x, src, 64);
        {
            const int last = (row_ptr[r + 1] - 1) / AG_R;
            // teams of `dl` lanes (one lane per feature) share the ranges of a long row round-robin,
            // four loads in flight each; team sums are added in team order (fixed by the shape)
            int dl = 1;
            while (dl < D && dl < 64) dl <<= 1;
            const int parts = 64 / dl;
            const int part = lane / dl;
            // denominator: every lane adds all pieces
            float zsum;
            {
                float z0 = 0.f, z1 = 0.f, z2 = 0.f, z3 = 0.f;
                int u = v + 1 + part;
                for (; u + 3 * parts <= last; u += 4 * parts) {
                    z0 += carry[(static_cast<size_t>(u) * 2) * DPZ + DP];
                    z1 += carry[(static_cast<size_t>(u + parts) * 2) * DPZ + DP];
                    z2 += carry[(static_cast<size_t>(u + 2 * parts) * 2) * DPZ + DP];
                    z3 += carry[(static_cast<size_t>(u + 3 * parts) * 2) * DPZ + DP];
                }
                for (; u <= last; u += parts) z0 += carry[(static_cast<size_t>(u) * 2) * DPZ + DP];
                zsum = (z0 + z1) + (z2 + z3);
                for (int off = 32; off >= dl; off >>= 1) zsum += __shfl_down(zsum, off, 64);
                zsum = __shfl(zsum, 0, 64) + carry[(static_cast<size_t>(v) * 2 + 1) * DPZ + DP];
                if (row_z && lane == 0) row_z[r] = zsum;
            }
            for (int d0 = 0; d0 < D; d0 += 64) {
                const int d = d0 + lane % dl;
                const bool dok = d < D;
                const float *base = carry + (dok ? d : 0);
                float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
                int u = v + 1 + part;
                for (; u + 3 * parts <= last; u += 4 * parts) {
                    const float a0 = base[(static_cast<size_t>(u) * 2) * DPZ];
                    const float a1 = base[(static_cast<size_t>(u + parts) * 2) * DPZ];
                    const float a2 = base[(static_cast<size_t>(u + 2 * parts) * 2) * DPZ];
                    const float a3 = base[(static_cast<size_t>(u + 3 * parts) * 2) * DPZ];
                    s0 += a0; s1 += a1; s2 += a2; s3 += a3;
                }
                for (; u <= last; u += parts) s0 += base[(static_cast<size_t>(u) * 2) * DPZ];
                float sum = (s0 + s1) + (s2 + s3);
                for (int off = 32; off >= dl; off >>= 1) sum += __shfl_down(sum, off, 64);
                if (lane < dl && dok) {
                    sum += carry[(static_cast<size_t>(v) * 2 + 1) * DPZ + d];
                    store_elem(out, static_cast<int64_t>(r) * ldo + d, odt, sum / zsum);
                    if (out32) out32[static_cast<int64_t>(r) * ld32 + d] = sum / zsum;
                }
            }
        }
    }
    const int64_t row = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (row < n && row_ptr[row] == row_ptr[row + 1]) {
        for (int d = 0; d < D; ++d) store_elem(out, row * ldo + d, odt, 0.f);
        if (out32)
            for (int d = 0; d < D; ++d) out32[row * ld32 + d] = 0.f;
        if (row_z) row_z[row] = 0.f;
    }
}

template <class T>
static void launch_agnn_t(int vec, int lpr, unsigned grid, hipStream_t s, int nnz, int n_ranges, const ftc_csr &g,
                          const int *e2r, const void *H, int ld, int D, float beta, void *out,
                          int ldo, int odt, float *carry, int *tail_row, float *row_z, float *out32, int ld32)
{
    constexpr int VM = T::VEC;
#define FTC_AG(V, L)                                                                                                  \
    if (row_z || out32)                                                                                               \
        hipLaunchKernelGGL((agnn_fused_kernel<T, V, L, true>), dim3(grid), dim3(256), 0, s, nnz, n_ranges, g.row_ptr, \
                           g.col_idx, e2r, H, ld, D, beta, out, ldo, odt, carry, tail_row, row_z, out32, ld32);       \
    else                                                                                                              \
        hipLaunchKernelGGL((agnn_fused_kernel<T, V, L, false>), dim3(grid), dim3(256), 0, s, nnz, n_ranges,           \
                           g.row_ptr, g.col_idx, e2r, H, ld, D, beta, out, ldo, odt, carry, tail_row, row_z, out32, ld32)
    if (vec == VM) {
        if (lpr == 4) { FTC_AG(VM, 4); }
        else if (lpr == 8) { FTC_AG(VM, 8); }
        else if (lpr == 16) { FTC_AG(VM, 16); }
        else { FTC_AG(VM, 32); }
    } else if (vec == VM / 2) {
        FTC_AG(VM / 2, 4);
    } else {
        FTC_AG(VM / 4, 4);
    }
#undef FTC_AG
}

// Caller has checked: window index present, seg_shape() accepts (dt, D), rows of H and out 16-byte
// aligned, workspace of agnn_fused_ws() bytes.
int32_t launch_agnn_fused(const ftc_csr &g, const ftc_windows &w, const void *H, int ld, int dt, int D,
                          float beta, void *out, int ldo, int odt, float *row_z, float *out32, int ld32, void *ws,
                          hipStream_t s)
{
    int vec = 0, lpr = 0;
    seg_shape(dt, D, &vec, &lpr);
    const int dp = vec * lpr;
    const int n_ranges = ceil_div(g.nnz, AG_R);
    float *carry = static_cast<float *>(ws);
    int *tail_row = reinterpret_cast<int *>(
        static_cast<char *>(ws) + align_up(static_cast<size_t>(n_ranges) * 2 * (dp + 4) * sizeof(float), 256));
    if (n_ranges > 0) {
        const unsigned grid = static_cast<unsigned>((n_ranges + 3) / 4);
        if (dt == FTC_F32)
            launch_agnn_t<F32>(vec, lpr, grid, s, g.nnz, n_ranges, g, w.edge_to_row, H, ld, D, beta, out, ldo,
                               odt, carry, tail_row, row_z, out32, ld32);
        else if (dt == FTC_F16)
            launch_agnn_t<F16>(vec, lpr, grid, s, g.nnz, n_ranges, g, w.edge_to_row, H, ld, D, beta, out, ldo,
                               odt, carry, tail_row, row_z, out32, ld32);
        else
            launch_agnn_t<BF16>(vec, lpr, grid, s, g.nnz, n_ranges, g, w.edge_to_row, H, ld, D, beta, out, ldo,
                                odt, carry, tail_row, row_z, out32, ld32);
        const int32_t st = launch_status("agnn_fused");
        if (st != FTC_OK) return st;
    }
    // lanes per cut row in the fix-up kernel: four features per lane
    int grp = 1;
    while (grp * 4 < dp) grp <<= 1;
    const int64_t blocks_rows = (static_cast<int64_t>(g.n) + 255) / 256;
    const int64_t per_block = 4 * (64 / grp);
    const int64_t blocks_ranges = (n_ranges + per_block - 1) / per_block;
    const unsigned grid2 = static_cast<unsigned>(blocks_rows > blocks_ranges ? blocks_rows : blocks_ranges);
#define FTC_FX(G)                                                                                                    \
    case G:                                                                                                          \
        hipLaunchKernelGGL(agnn_fused_fixup_kernel<G>, dim3(grid2), dim3(256), 0, s, g.n, n_ranges, g.row_ptr, carry, \
                           tail_row, dp, D, out, ldo, odt, row_z, out32, ld32);                                      \
        break;
    switch (grp) {
        FTC_FX(1) FTC_FX(2) FTC_FX(4) FTC_FX(8) FTC_FX(16) FTC_FX(32) FTC_FX(64)
    }
#undef FTC_FX
    return launch_status("agnn_fused fixup");
}

}  // namespace ftc
