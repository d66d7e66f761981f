// Work-balanced sparse neighbour aggregation (SpMM, Section V.A) on the vector units.
//
// The paper gives one row window to one thread block; on power-law graphs a single window can
// hold 10^5 edges while the median row has two, so here the unit of work is a fixed number of
// EDGES instead.  The window index supplies what makes that possible without searching:
// edge_to_row (`edgeToRow`) tells every edge its output row.
//
//   - A wave owns SEG_R consecutive edges.  Their (column, value, row) triples are loaded once,
//     coalesced, into LDS.
//   - The wave is cut into groups of LPR lanes; a group walks a contiguous run of the wave's
//     edges, SEG_B at a time (SEG_B independent 16-byte gathers of X rows in flight per lane),
//     and accumulates in registers while the row stays the same.
//   - A row that lies completely inside one run is stored straight from registers.  A row cut by
//     a run boundary leaves a partial sum: the pieces inside one wave are added in LDS in edge
//     order; the pieces that cross a wave boundary go to a small carry buffer and are added, again
//     in edge order, by a second tiny kernel.  No floating-point atomics: results are
//     reproducible bit for bit.
#include "ftc_common.hpp"

namespace ftc {

constexpr int SEG_B = 4;    // edges per batch (gathers in flight per lane)

static int pow2_ceil(int x)
{
    int p = 1;
    while (p < x) p *= 2;
    return p;
}

// Lane layout for a feature width: `vec` elements per lane, `lpr` lanes per row (4..32).
bool seg_shape(int dtype, int D, int *vec, int *lpr)
{
    const int vmax = dtype == FTC_F32 ? 4 : 8;
    for (int v = vmax; v >= vmax / 4 && v >= 1; v /= 2) {
        if (D % v != 0) continue;
        const int l = pow2_ceil(D / v);
        // narrower-than-16-byte lanes exist only in the 4-lane layout (small D)
        if (l >= 4 && l <= (v == vmax ? 32 : 4)) {
            *vec = v;
            *lpr = l;
            return true;
        }
    }
    return false;
}

size_t spmm_seg_ws(int nnz, int D)
{
    int vec, lpr, dp = 0;
    if (seg_shape(FTC_F32, D, &vec, &lpr)) dp = vec * lpr;
    if (seg_shape(FTC_F16, D, &vec, &lpr) && vec * lpr > dp) dp = vec * lpr;
    if (dp == 0 || nnz == 0) return 0;
    const size_t n_ranges = (static_cast<size_t>(nnz) + SEG_R - 1) / SEG_R;
    const size_t seg = align_up(n_ranges * 2 * dp * sizeof(float), 256) + align_up(n_ranges * 2 * sizeof(int), 256);
    const size_t lane = D <= 16 ? spmm_lane_ws(nnz) : 0;  // narrow rows may take the lane-per-edge kernel
    return seg > lane ? seg : lane;
}

// VALS = false: all edge values are one (vals == NULL): nothing is staged or multiplied for them, which
// also cuts the LDS footprint by a third (more workgroups per CU).
template <class T, int VEC, int LPR, bool VALS>
__global__ __launch_bounds__(256) void spmm_seg_kernel(int nnz, int n_ranges, const int *__restrict__ row_ptr,
                                                       const int *__restrict__ col_idx,
                                                       const int *__restrict__ edge_to_row,
                                                       const float *__restrict__ vals,
                                                       const void *__restrict__ X, int ldx, int D,
                                                       void *__restrict__ out, int ldo, int odt, Epi epi,
                                                       float *__restrict__ carry, int *__restrict__ carry_tail_row,
                                                       const uint8_t *__restrict__ dense)
{
    constexpr int NG = 64 / LPR;      // groups per wave
    constexpr int RUN = SEG_R / NG;   // edges per group
    constexpr int RP = SEG_R + NG;    // one pad word per run keeps the groups on different LDS banks
    constexpr int DP = LPR * VEC;     // padded feature width
    static_assert(RUN % SEG_B == 0, "runs are whole batches");
    constexpr int IDX_WORDS = 4 * (VALS ? 3 : 2) * RP;
    constexpr int PART_WORDS = 4 * 2 * NG * DP;
    __shared__ int smem[IDX_WORDS > PART_WORDS ? IDX_WORDS : PART_WORDS];
    __shared__ int s_meta[4][3][NG];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int g = lane / LPR, sub = lane % LPR;
    int *s_col = smem + wave * (VALS ? 3 : 2) * RP;
    int *s_row = s_col + RP;
    float *s_val = reinterpret_cast<float *>(s_row + RP);  // only with VALS

    const int v = xcd_chunked_block(blockIdx.x, gridDim.x) * 4 + wave;
    const bool active = v < n_ranges;
    const int base = active ? v * SEG_R : 0;
    const int n_valid = active ? min(SEG_R, nnz - base) : 0;
    int rows[SEG_R / 64];
    const bool from_starts = n_valid == SEG_R && rows_from_starts<SEG_R>(row_ptr, edge_to_row, base, lane, rows);
#pragma unroll
    for (int j = 0; j < SEG_R / 64; ++j) {
        const int i = j * 64 + lane;
        if (i < n_valid) {
            const int p = i + i / RUN;
            const int er = from_starts ? rows[j] : edge_to_row[base + i];
            // edges of windows that go to the matrix cores are skipped here (column -1)
            s_col[p] = (dense && dense[er >> 4]) ? -1 : __builtin_nontemporal_load(col_idx + base + i);  // streamed once
            s_row[p] = er;
            if constexpr (VALS) s_val[p] = __builtin_nontemporal_load(vals + base + i);
        }
    }
    const int prev_row = (active && base > 0) ? edge_to_row[base - 1] : -1;
    const int next_row = (active && n_valid == SEG_R && base + SEG_R < nnz) ? edge_to_row[base + SEG_R] : -1;
    // row of the first edge after the NEXT range: tells whether a row left open here ends there
    const int far_row = (active && static_cast<int64_t>(base) + 2 * SEG_R < nnz) ? edge_to_row[base + 2 * SEG_R] : -1;
    __syncthreads();

    const int rs = g * RUN;
    const int re = min(rs + RUN, n_valid);
    const bool has = rs < n_valid;
    const bool live = sub * VEC < D;
    float acc[VEC], hacc[VEC];
#pragma unroll
    for (int j = 0; j < VEC; ++j) { acc[j] = 0.f; hacc[j] = 0.f; }
    bool have_head = false, head_closed = false, have_tail = false;
    int head_row = -1, cur = -1;

    auto direct_store = [&](int row) {
        if (live && !(dense && dense[row >> 4])) {
            float o[VEC];
            const float f = epi.factor(row);
#pragma unroll
            for (int j = 0; j < VEC; ++j) o[j] = epi.apply(f, acc[j]);
            store_vec_nt<VEC>(out, static_cast<int64_t>(row) * ldo + sub * VEC, odt, o);
        }
    };

    if (has) {
        cur = s_row[rs + g];
        const int left_row = rs == 0 ? prev_row : s_row[rs - 1 + g - 1];
        const bool left_open = left_row == cur;
        bool first = true;
        for (int b = rs; b < re; b += SEG_B) {
            int c[SEG_B], r[SEG_B];
            float a[SEG_B];
            RawVec<T, VEC> x[SEG_B];
#pragma unroll
            for (int k = 0; k < SEG_B; ++k) {
                const bool ok = b + k < re;
                const int p = (ok ? b + k : rs) + g;
                c[k] = s_col[p];
                r[k] = ok ? s_row[p] : -1;
                a[k] = VALS ? s_val[p] : 1.f;
            }
#pragma unroll
            for (int k = 0; k < SEG_B; ++k) {
                if (r[k] >= 0 && c[k] >= 0 && live) load_raw<T, VEC>(X, static_cast<int64_t>(c[k]) * ldx + sub * VEC, x[k]);
                else zero_raw(x[k]);
            }
#pragma unroll
            for (int k = 0; k < SEG_B; ++k) {
                if (r[k] >= 0) {
                    if (r[k] != cur) {  // the segment of row `cur` ends here
                        if (first && left_open) {
#pragma unroll
                            for (int j = 0; j < VEC; ++j) hacc[j] = acc[j];
                            have_head = true; head_closed = true; head_row = cur;
                        } else {
                            direct_store(cur);
                        }
                        first = false;
                        cur = r[k];
#pragma unroll
                        for (int j = 0; j < VEC; ++j) acc[j] = 0.f;
                    }
                    float xf[VEC];
                    unpack<T, VEC>(x[k], xf);
#pragma unroll
                    for (int j = 0; j < VEC; ++j) acc[j] = VALS ? fmaf(a[k], xf[j], acc[j]) : acc[j] + xf[j];
                }
            }
        }
        // the run's last segment
        int right_row;
        if (re < n_valid) right_row = s_row[re + g + 1];
        else right_row = next_row;  // -1 when the edge list ends here
        const bool right_open = right_row == cur;
        if (first && left_open) {
#pragma unroll
            for (int j = 0; j < VEC; ++j) hacc[j] = acc[j];
            have_head = true; head_closed = !right_open; head_row = cur;
        } else if (!right_open) {
            direct_store(cur);
        } else {
            have_tail = true;
        }
    }
    __syncthreads();  // every wave is done with the staged indices: the LDS is reused for partials

    float *part = reinterpret_cast<float *>(smem) + wave * 2 * NG * DP;
    if (have_head) {
#pragma unroll
        for (int j = 0; j < VEC; ++j) part[(2 * g) * DP + sub * VEC + j] = hacc[j];
    }
    if (have_tail) {
#pragma unroll
        for (int j = 0; j < VEC; ++j) part[(2 * g + 1) * DP + sub * VEC + j] = acc[j];
    }
    if (sub == 0) {
        s_meta[wave][0][g] = have_head ? head_row : -1;
        s_meta[wave][1][g] = head_closed ? 1 : 0;
        s_meta[wave][2][g] = have_tail ? cur : -1;
    }
    __syncthreads();

    // Add the pieces of rows cut inside this wave, in edge order; one lane per feature.
    if (active) {
        int tail_out = -1;
        for (int d = lane; d < DP; d += 64) {
            float run = 0.f;
            int run_row = -1;
            bool from_outside = false;
            tail_out = -1;
            for (int q = 0; q < NG; ++q) {
                const int hr = s_meta[wave][0][q];
                if (hr >= 0) {
                    if (run_row < 0) { run_row = hr; run = 0.f; from_outside = true; }
                    run += part[(2 * q) * DP + d];
                    if (s_meta[wave][1][q]) {
                        if (from_outside) carry[(static_cast<size_t>(v) * 2) * DP + d] = run;
                        else if (d < D && !(dense && dense[run_row >> 4]))
                            store_elem(out, static_cast<int64_t>(run_row) * ldo + d, odt,
                                       epi.apply(epi.factor(run_row), run));
                        run_row = -1;
                        from_outside = false;
                    }
                }
                const int tr = s_meta[wave][2][q];
                if (tr >= 0) { run_row = tr; run = part[(2 * q + 1) * DP + d]; from_outside = false; }
            }
            if (run_row >= 0) {
                if (from_outside) {
                    carry[(static_cast<size_t>(v) * 2) * DP + d] = run;  // the row covers the whole wave
                } else {
                    carry[(static_cast<size_t>(v) * 2 + 1) * DP + d] = run;
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

// Second pass: rows cut by a wave boundary, and rows without any stored entry.  G lanes (four features
// each) finish one cut row, 64 / G rows per wave: the kernel is a chain of two dependent loads per row (the
// range's record, then the two pieces), so it is the number of rows in flight that counts.  DP is a
// multiple of 4 and the carry buffer 16-byte aligned (both by construction of the first pass).
template <int G>
__global__ __launch_bounds__(256) void spmm_seg_fixup_kernel(int n, int n_ranges, const int *__restrict__ row_ptr,
                                                             const float *__restrict__ carry,
                                                             const int *__restrict__ carry_tail_row, int DP,
                                                             int D, void *__restrict__ out, int ldo, int odt,
                                                             Epi epi, const uint8_t *__restrict__ dense, int seg_r)
{
    constexpr int R = 64 / G;  // ranges per wave
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int sub = lane % G;
    const int v_mine = (blockIdx.x * 4 + wave) * R + lane / G;
    int2 rec = make_int2(-1, 0);
    if (v_mine < n_ranges) rec = reinterpret_cast<const int2 *>(carry_tail_row)[v_mine];
    // Nearly every open row ends in the next range: out = head piece of range v + 1 + tail piece of
    // range v.  Their addresses depend on v alone, so they are loaded together with the range's record
    // instead of after it.
    for (int f0 = 0; f0 < DP; f0 += 4 * G) {
        const int f = f0 + sub * 4;
        const bool ok = v_mine + 1 < n_ranges && f < DP;
        const size_t vv = ok ? static_cast<size_t>(v_mine) : 0;
        float4 h4 = make_float4(0.f, 0.f, 0.f, 0.f), t4 = h4;
        if (ok) {
            h4 = *reinterpret_cast<const float4 *>(carry + (vv + 1) * 2 * DP + f);
            t4 = *reinterpret_cast<const float4 *>(carry + (vv * 2 + 1) * DP + f);
        }
        int r = rec.x;
        if (r >= 0 && dense && dense[r >> 4]) r = -1;
        if (f0 == 0) rec.x = r;
        if (ok && r >= 0 && rec.y) {
            const float fac = epi.factor(r);
            const float o[4] = {h4.x + t4.x, h4.y + t4.y, h4.z + t4.z, h4.w + t4.w};
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (f + i < D) store_elem(out, static_cast<int64_t>(r) * ldo + f + i, odt, epi.apply(fac, o[i]));
        }
    }
    // rows that go on beyond the next range (long rows of a power-law graph): one at a time, by the whole wave
    unsigned long long longs = __builtin_amdgcn_ballot_w64(rec.x >= 0 && !rec.y && sub == 0);
    while (longs) {
        const int src = __ffsll(static_cast<long long>(longs)) - 1;
        longs &= longs - 1;
        const int v = __shfl(v_mine, src, 64), r = __shfl(rec.x, src, 64);
        const int last = (row_ptr[r + 1] - 1) / seg_r;  // wave range holding the row's final edge
        // A hub row can span hundreds of ranges.  The 64 lanes are split into `parts` teams of
        // `dl` lanes (one lane per feature); team p adds the head pieces of ranges v+1+p,
        // v+1+p+parts, ... four at a time, then the teams' sums are added in team order.  The
        // order is fixed by the shape alone, so the result is reproducible.
        int dl = 1;
        while (dl < D && dl < 64) dl <<= 1;
        const int parts = 64 / dl;
        const int part = lane / dl;
        for (int d0 = 0; d0 < D; d0 += 64) {
            const int d = d0 + lane % dl;
            const bool dok = d < D;
            const float *base = carry + (dok ? d : 0);
            float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
            int u = v + 1 + part;
            for (; u + 3 * parts <= last; u += 4 * parts) {
                const float a0 = base[(static_cast<size_t>(u) * 2) * DP];
                const float a1 = base[(static_cast<size_t>(u + parts) * 2) * DP];
                const float a2 = base[(static_cast<size_t>(u + 2 * parts) * 2) * DP];
                const float a3 = base[(static_cast<size_t>(u + 3 * parts) * 2) * DP];
                s0 += a0; s1 += a1; s2 += a2; s3 += a3;
            }
            for (; u <= last; u += parts) s0 += base[(static_cast<size_t>(u) * 2) * DP];
            float sum = (s0 + s1) + (s2 + s3);
            for (int off = 32; off >= dl; off >>= 1) sum += __shfl_down(sum, off, 64);
            if (lane < dl && dok) {
                sum += carry[(static_cast<size_t>(v) * 2 + 1) * DP + d];
                store_elem(out, static_cast<int64_t>(r) * ldo + d, odt, epi.apply(epi.factor(r), sum));
            }
        }
    }
    const int64_t row = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (row < n && row_ptr[row] == row_ptr[row + 1] && !(dense && dense[row >> 4]))
        for (int d = 0; d < D; ++d) store_elem(out, row * ldo + d, odt, 0.f);
}

int32_t launch_seg_fixup(int n, int n_ranges, const int *row_ptr, const float *carry, const int *tail_row, int dp,
                         int D, void *out, int ldo, int odt, Epi epi, const uint8_t *dense, int seg_r, hipStream_t s,
                         const char *what)
{
    int grp = 1;
    while (grp * 4 < dp && grp < 16) grp <<= 1;  // at most 16 lanes a row: wider rows take several rounds
    const int64_t blocks_rows = (static_cast<int64_t>(n) + 255) / 256;
    const int64_t blocks_ranges = ceil_div(n_ranges, 4 * (64 / grp));
    const unsigned grid2 = static_cast<unsigned>(blocks_rows > blocks_ranges ? blocks_rows : blocks_ranges);
#define FTC_FX(G)                                                                                                  \
    case G:                                                                                                        \
        hipLaunchKernelGGL(spmm_seg_fixup_kernel<G>, dim3(grid2), dim3(256), 0, s, n, n_ranges, row_ptr, carry,    \
                           tail_row, dp, D, out, ldo, odt, epi, dense, seg_r);                                     \
        break;
    switch (grp) {
        FTC_FX(1) FTC_FX(2) FTC_FX(4) FTC_FX(8) FTC_FX(16)
    }
#undef FTC_FX
    return launch_status(what);
}

template <class T>
static void launch_seg_t(int vec, int lpr, unsigned grid, hipStream_t s, int nnz, int n_ranges,
                         const ftc_csr &g, const int *e2r, const float *vals, const void *X, int ldx, int D,
                         void *out, int ldo, int odt, Epi epi, float *carry, int *tail_row, const uint8_t *dense)
{
    constexpr int VM = T::VEC;
#define FTC_SEG(V, L)                                                                                       \
    do {                                                                                                    \
        if (vals)                                                                                           \
            hipLaunchKernelGGL((spmm_seg_kernel<T, V, L, true>), dim3(grid), dim3(256), 0, s, nnz, n_ranges, \
                               g.row_ptr, g.col_idx, e2r, vals, X, ldx, D, out, ldo, odt, epi, carry,        \
                               tail_row, dense);                                                            \
        else                                                                                                \
            hipLaunchKernelGGL((spmm_seg_kernel<T, V, L, false>), dim3(grid), dim3(256), 0, s, nnz,         \
                               n_ranges, g.row_ptr, g.col_idx, e2r, vals, X, ldx, D, out, ldo, odt, epi,    \
                               carry, tail_row, dense);                                                     \
    } while (0)
    if (vec == VM) {
        if (lpr == 4) FTC_SEG(VM, 4);
        else if (lpr == 8) FTC_SEG(VM, 8);
        else if (lpr == 16) FTC_SEG(VM, 16);
        else FTC_SEG(VM, 32);
    } else if (vec == VM / 2) {
        FTC_SEG(VM / 2, 4);
    } else {
        FTC_SEG(VM / 4, 4);
    }
#undef FTC_SEG
}

// Caller has checked: window index present, seg_shape() accepts (xdt, D), X and out rows 16-byte
// aligned, workspace of spmm_seg_ws() bytes.
int32_t launch_spmm_seg(const ftc_csr &g, const ftc_windows &w, const float *vals, const void *X, int ldx,
                        int xdt, int D, void *out, int ldo, int odt, Epi epi, void *ws, const uint8_t *dense,
                        hipStream_t s)
{
    // rows of at most 32 bytes: one or two lanes per run of edges instead of four lanes per row
    if (!dense && spmm_lane_shape(xdt, D, ldx))
        return launch_spmm_lane(g, w, vals, X, ldx, xdt, D, out, ldo, odt, epi, ws, s);
    int vec = 0, lpr = 0;
    seg_shape(xdt, D, &vec, &lpr);
    const int dp = vec * lpr;
    const int n_ranges = ceil_div(g.nnz, SEG_R);
    float *carry = static_cast<float *>(ws);
    int *tail_row = reinterpret_cast<int *>(static_cast<char *>(ws) +
                                            align_up(static_cast<size_t>(n_ranges) * 2 * dp * sizeof(float), 256));
    if (n_ranges > 0) {
        const unsigned grid = static_cast<unsigned>((n_ranges + 3) / 4);
        if (xdt == FTC_F32)
            launch_seg_t<F32>(vec, lpr, grid, s, g.nnz, n_ranges, g, w.edge_to_row, vals, X, ldx, D, out, ldo,
                              odt, epi, carry, tail_row, dense);
        else if (xdt == FTC_F16)
            launch_seg_t<F16>(vec, lpr, grid, s, g.nnz, n_ranges, g, w.edge_to_row, vals, X, ldx, D, out, ldo,
                              odt, epi, carry, tail_row, dense);
        else
            launch_seg_t<BF16>(vec, lpr, grid, s, g.nnz, n_ranges, g, w.edge_to_row, vals, X, ldx, D, out, ldo,
                               odt, epi, carry, tail_row, dense);
        const int32_t st = launch_status("spmm_seg");
        if (st != FTC_OK) return st;
    }
    return launch_seg_fixup(g.n, n_ranges, g.row_ptr, carry, tail_row, dp, D, out, ldo, odt, epi, dense, SEG_R, s,
                            "spmm_seg fixup");
}

}  // namespace ftc
