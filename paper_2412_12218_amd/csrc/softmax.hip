// Edge softmax over the stored entries of each CSR row.  Row lengths range from 1 to tens of
// thousands (power-law graphs), so a workgroup takes 256 consecutive rows and treats them in
// three classes: short rows by one lane each, medium rows by one wave each, long rows by the
// whole workgroup.  Every row's reduction order depends only on its length, so results are
// reproducible from run to run.
#include "ftc_common.hpp"

namespace ftc {

constexpr int SM_SHORT = 16;    // <= : one lane per row
constexpr int SM_MEDIUM = 2048; // <= : one wave per row; above: the workgroup

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    return v;
}

__global__ __launch_bounds__(256) void edge_softmax_kernel(int n, const int *__restrict__ row_ptr,
                                                           const float *in, float *out)
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
    if (len > 0 && len <= SM_SHORT) {
        float m = -INFINITY;
        for (int e = e0; e < e1; ++e) m = fmaxf(m, in[e]);
        float z = 0.f;
        for (int e = e0; e < e1; ++e) z += expf(in[e] - m);
        const float inv = 1.f / z;
        for (int e = e0; e < e1; ++e) out[e] = expf(in[e] - m) * inv;
    } else if (len > SM_SHORT && len <= SM_MEDIUM) {
        mid_rows[atomicAdd(&n_mid, 1)] = static_cast<int>(row);
    } else if (len > SM_MEDIUM) {
        big_rows[atomicAdd(&n_big, 1)] = static_cast<int>(row);
    }
    __syncthreads();
    const int nm = n_mid, nb = n_big;
    for (int i = wave; i < nm; i += 4) {
        const int r = mid_rows[i];
        const int a = row_ptr[r], b = row_ptr[r + 1];
        float m = -INFINITY;
        for (int e = a + lane; e < b; e += 64) m = fmaxf(m, in[e]);
        m = wave_max(m);
        float z = 0.f;
        for (int e = a + lane; e < b; e += 64) z += expf(in[e] - m);
        z = wave_sum(z);
        const float inv = 1.f / z;
        for (int e = a + lane; e < b; e += 64) out[e] = expf(in[e] - m) * inv;
    }
    for (int i = 0; i < nb; ++i) {  // nb is uniform over the workgroup
        const int r = big_rows[i];
        const int a = row_ptr[r], b = row_ptr[r + 1];
        float m = -INFINITY;
        for (int e = a + tid; e < b; e += 256) m = fmaxf(m, in[e]);
        m = wave_max(m);
        __syncthreads();
        if (lane == 0) red[wave] = m;
        __syncthreads();
        m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        float z = 0.f;
        for (int e = a + tid; e < b; e += 256) z += expf(in[e] - m);
        z = wave_sum(z);
        __syncthreads();
        if (lane == 0) red[wave] = z;
        __syncthreads();
        z = (red[0] + red[1]) + (red[2] + red[3]);
        const float inv = 1.f / z;
        for (int e = a + tid; e < b; e += 256) out[e] = expf(in[e] - m) * inv;
    }
}

int32_t launch_softmax(const ftc_csr &g, const float *in, float *out, hipStream_t s)
{
    if (g.n == 0 || g.nnz == 0) return FTC_OK;
    const unsigned grid = static_cast<unsigned>((static_cast<int64_t>(g.n) + 255) / 256);
    hipLaunchKernelGGL(edge_softmax_kernel, dim3(grid), dim3(256), 0, s, g.n, g.row_ptr, in, out);
    return launch_status("edge_softmax");
}

// ------------------------------------------------------------------------------------------------
// Edge-balanced variant for graphs with a window index (edge_to_row known for every edge).
//
//   1. local kernel: a wave takes SMS_R consecutive edges and keeps their scores and row ids in
//      registers.  The pair (running maximum m, sum of exp(s - m)) is an associative reduction, so
//      a segmented inclusive scan over the 64 lanes (segments = runs of equal row id) gives every
//      row piece its pair.  A row that lies completely inside the wave's range gets its pair into
//      a table in LDS and its probabilities are written at once from the registers: such edges
//      cross HBM twice in all (score in, probability out).  The piece entering from the left and
//      the piece leaving to the right go to a carry buffer together with their extents.
//   2. cut-row kernel: the wave that owns a range combines the pieces of the (at most two) rows cut by its
//      boundaries, in an order fixed by the row's extent, and writes the probabilities of its own pieces.
constexpr int SMS_R = 1024;
constexpr int SMS_C = SMS_R / 64;  // 64-edge chunks per wave

struct MZ {
    float m, z;
};

__device__ __forceinline__ MZ mz_combine(MZ a, MZ b)
{
    // exp of a non-positive number only; the larger maximum keeps its sum unscaled
    MZ r;
    if (a.m >= b.m) { r.m = a.m; r.z = a.z + b.z * __expf(b.m - a.m); }
    else { r.m = b.m; r.z = b.z + a.z * __expf(a.m - b.m); }
    return r;
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_i(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, CTRL, ROW_MASK, 0xf, false);
}

// Segmented inclusive scan of (m, z) over the lanes of a wave; `head` != 0 marks the first lane of a
// segment.  Data-parallel-primitive moves: shifts by 1, 2, 4, 8 inside rows of 16 lanes, then lane
// 15 of a row into the next row (rows 1 and 3) and lane 31 into rows 2 and 3.  The head flags are
// OR-ed along with the values: a lane stops taking from the left once a head lies in its span.
template <class Op>
__device__ __forceinline__ MZ wave_segmented_scan(MZ x, int head, int lane)
{
#define FTC_STEP(CTRL, ROW_MASK, VALID)                                                  \
    {                                                                                    \
        MZ y;                                                                            \
        y.m = __int_as_float(dpp_i<CTRL, ROW_MASK>(__float_as_int(x.m)));                \
        y.z = __int_as_float(dpp_i<CTRL, ROW_MASK>(__float_as_int(x.z)));                \
        const int yh = dpp_i<CTRL, ROW_MASK>(head);                                      \
        if (VALID) {                                                                     \
            if (!head) x = Op::combine(y, x);                                            \
            head |= yh;                                                                  \
        }                                                                                \
    }
    const int r16 = lane & 15;
    FTC_STEP(0x111, 0xf, r16 >= 1)
    FTC_STEP(0x112, 0xf, r16 >= 2)
    FTC_STEP(0x114, 0xf, r16 >= 4)
    FTC_STEP(0x118, 0xf, r16 >= 8)
    FTC_STEP(0x142, 0xa, (lane & 16) != 0)
    FTC_STEP(0x143, 0xc, lane >= 32)
#undef FTC_STEP
    return x;
}

__device__ __forceinline__ int wave_sum_int(int v)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    return v;
}

// One more score for a running (maximum, sum of exp) pair: one exponential.
__device__ __forceinline__ void mz_push(MZ &a, float s)
{
    if (s <= a.m) {
        a.z += __expf(s - a.m);
    } else {
        a.z = a.z * __expf(a.m - s) + 1.f;  // a.m = -inf, a.z = 0 for an empty pair: 0 * 0 + 1
        a.m = s;
    }
}

// The two row-wise edge operations that run on the range kernels below.  Both reduce a row to a
// pair and then map every edge with it:
//   forward   pair = (maximum, sum of exp) of the scores;           p  = exp(s - m) / z
//   backward  pair = (unused, sum of p * dp) of the row's entries;  ds = p * (dp - sum)
struct SoftmaxFwd {
    static constexpr bool TWO_INPUTS = false;
    __device__ static MZ identity() { return MZ{-INFINITY, 0.f}; }
    __device__ static void push(MZ &a, float s, float) { mz_push(a, s); }
    __device__ static MZ combine(MZ a, MZ b) { return mz_combine(a, b); }
    // a row's pair as its entries use it: (maximum, 1 / sum), the division done once per row piece
    __device__ static float2 final_pair(float2 t) { return make_float2(t.x, 1.f / t.y); }
    __device__ static float result(float s, float, float2 t) { return __expf(s - t.x) * t.y; }
};

struct SoftmaxBwd {
    static constexpr bool TWO_INPUTS = true;
    __device__ static MZ identity() { return MZ{0.f, 0.f}; }
    __device__ static void push(MZ &a, float p, float dp) { a.z = fmaf(p, dp, a.z); }
    __device__ static MZ combine(MZ a, MZ b) { return MZ{0.f, a.z + b.z}; }
    __device__ static float2 final_pair(float2 t) { return t; }
    __device__ static float result(float p, float dp, float2 t) { return p * (dp - t.y); }
};

// A lane owns SMS_L consecutive edges of the wave's range: it walks them once to build the pairs of
// the row pieces it holds (rows that begin and end inside the lane are final at once), ONE
// segmented scan over the lanes joins the pieces that continue from lane to lane, and a second walk
// writes the probabilities.  Rows are numbered in order of appearance (row ids may skip rows
// without entries): number 0 is the row that enters the range from the left (it may not exist),
// the others count the row beginnings; the number indexes the table of final pairs in LDS.
//
// Per range: carry[2v] = pair of the piece entering from the left, carry[2v+1] = pair of the piece
// leaving to the right; meta[2v] = {edges of the entering piece, first edge of the leaving piece
// (n_valid when none), 1 if there is a leaving piece else -1, first range of the entering piece's row},
// meta[2v+1] = {last range of the entering piece's row, last range of the leaving piece's row, -, -}: the
// second kernel finds the pieces of its cut rows without reading a row start.
constexpr int SMS_L = SMS_R / 64;

// Rows that may begin inside a range before the per-entry row ids are read instead of the row starts.
constexpr int SMS_Q = 4;  // row starts per lane

template <class Op, bool VEC>
__global__ __launch_bounds__(256) void softmax_local_kernel(int nnz, int n_ranges, const int *__restrict__ row_ptr,
                                                            const int *__restrict__ edge_to_row,
                                                            const float *in, const float *in2, float *out,
                                                            float2 *__restrict__ carry,
                                                            int4 *__restrict__ meta)
{
    __shared__ float2 table_all[4][SMS_R + 1];
    __shared__ __attribute__((aligned(16))) uint8_t marks_all[4][SMS_R];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int v = blockIdx.x * 4 + wave;
    if (v >= n_ranges) return;  // no workgroup barrier below
    float2 *table = table_all[wave];
    uint8_t *marks = marks_all[wave];
    const int base = v * SMS_R;
    const int n_valid = min(SMS_R, nnz - base);
    const int prev_row = base > 0 ? edge_to_row[base - 1] : -1;
    const int next_row = base + n_valid < nnz ? edge_to_row[base + n_valid] : -1;
    const int r_first = edge_to_row[base], r_last = edge_to_row[base + n_valid - 1];
    // extents of the two rows the range's boundaries may cut (lanes 0, 1, 2; used at the very end)
    const int ext = row_ptr[lane == 0 ? r_first : (lane == 1 ? r_first + 1 : r_last + 1)];
    const int e0 = lane * SMS_L;  // first edge of the lane inside the range
    float sc[SMS_L], sc2[Op::TWO_INPUTS ? SMS_L : 1];
    unsigned begins = 0;  // bit k: a row begins at the lane's k-th edge
    const int n_starts = r_last - r_first;  // rows r_first + 1 .. r_last begin inside the range
    if (VEC && n_valid == SMS_R && n_starts <= 64 * SMS_Q) {
        // The scores are the only per-entry stream: where the rows begin comes from the row starts (a few per
        // lane), marked in a byte per entry in LDS; every lane then reads the marks of its own entries.  (Rows
        // without entries share their start with the next row: the same mark.)
        int st[SMS_Q];
#pragma unroll
        for (int q = 0; q < SMS_Q; ++q) {
            const int t = q * 64 + lane;
            st[q] = t < n_starts ? row_ptr[r_first + 1 + t] - base : -1;
        }
#pragma unroll
        for (int q = 0; q < SMS_L / 4; ++q) {
            const float4 s4 = *reinterpret_cast<const float4 *>(in + base + e0 + 4 * q);
            sc[4 * q] = s4.x; sc[4 * q + 1] = s4.y; sc[4 * q + 2] = s4.z; sc[4 * q + 3] = s4.w;
            if constexpr (Op::TWO_INPUTS) {
                const float4 t4 = *reinterpret_cast<const float4 *>(in2 + base + e0 + 4 * q);
                sc2[4 * q] = t4.x; sc2[4 * q + 1] = t4.y; sc2[4 * q + 2] = t4.z; sc2[4 * q + 3] = t4.w;
            }
        }
        *reinterpret_cast<uint4 *>(marks + e0) = make_uint4(0u, 0u, 0u, 0u);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int q = 0; q < SMS_Q; ++q)
            if (st[q] >= 0 && st[q] < SMS_R) marks[st[q]] = 1;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const uint4 mk = *reinterpret_cast<const uint4 *>(marks + e0);
        const uint32_t mw[4] = {mk.x, mk.y, mk.z, mk.w};
#pragma unroll
        for (int k = 0; k < SMS_L; ++k) begins |= ((mw[k / 4] >> (8 * (k % 4))) & 1u) << k;
        if (lane == 0 && prev_row != r_first) begins |= 1u;  // the range's first entry begins a row
    } else {
        int rw[SMS_L];
        if (VEC && n_valid == SMS_R) {
#pragma unroll
            for (int q = 0; q < SMS_L / 4; ++q) {
                const int4 r4 = *reinterpret_cast<const int4 *>(edge_to_row + base + e0 + 4 * q);
                const float4 s4 = *reinterpret_cast<const float4 *>(in + base + e0 + 4 * q);
                rw[4 * q] = r4.x; rw[4 * q + 1] = r4.y; rw[4 * q + 2] = r4.z; rw[4 * q + 3] = r4.w;
                sc[4 * q] = s4.x; sc[4 * q + 1] = s4.y; sc[4 * q + 2] = s4.z; sc[4 * q + 3] = s4.w;
                if constexpr (Op::TWO_INPUTS) {
                    const float4 t4 = *reinterpret_cast<const float4 *>(in2 + base + e0 + 4 * q);
                    sc2[4 * q] = t4.x; sc2[4 * q + 1] = t4.y; sc2[4 * q + 2] = t4.z; sc2[4 * q + 3] = t4.w;
                }
            }
        } else {
#pragma unroll
            for (int k = 0; k < SMS_L; ++k) {
                const bool ok = e0 + k < n_valid;
                rw[k] = ok ? edge_to_row[base + e0 + k] : -2 - (e0 + k);  // padding: rows of their own
                sc[k] = ok ? in[base + e0 + k] : 0.f;
                if constexpr (Op::TWO_INPUTS) sc2[k] = ok ? in2[base + e0 + k] : 0.f;
            }
        }
        // row beginnings inside the lane; `left` is the row of the edge before the lane's first
        int left = __builtin_amdgcn_update_dpp(0, rw[SMS_L - 1], 0x138, 0xf, 0xf, false);  // wave_shr:1
        if (lane == 0) left = prev_row;
#pragma unroll
        for (int k = 0; k < SMS_L; ++k) begins |= (rw[k] != (k == 0 ? left : rw[k - 1]) ? 1u : 0u) << k;
    }
    const int nb = __popc(begins);
    const int first_num = wave_inclusive_scan(nb) - nb;  // number of the row that is open at the lane's start
    // first walk: pairs of the pieces
    MZ cur = Op::identity(), first_piece = Op::identity();
    float seg_max[Op::TWO_INPUTS ? 1 : SMS_L];  // forward: maximum of the piece every entry lies in
    if constexpr (!Op::TWO_INPUTS) {
        // Branch-free: running maxima forwards (restarting where a row begins), the piece's maximum carried
        // backwards to all its entries, ONE exponential per entry relative to that maximum, running sums.  What
        // an entry still lacks afterwards is a factor of its piece alone: exp(piece maximum - row maximum) / row sum.
        float run[SMS_L];
#pragma unroll
        for (int k = 0; k < SMS_L; ++k) run[k] = (k == 0 || (begins >> k & 1u)) ? sc[k] : fmaxf(run[k - 1], sc[k]);
        seg_max[SMS_L - 1] = run[SMS_L - 1];
#pragma unroll
        for (int k = SMS_L - 2; k >= 0; --k) seg_max[k] = (begins >> (k + 1) & 1u) ? run[k] : seg_max[k + 1];
#pragma unroll
        for (int k = 0; k < SMS_L; ++k) {
            sc[k] = __expf(sc[k] - seg_max[k]);                                   // sc now holds the exponentials
            run[k] = (k == 0 || (begins >> k & 1u)) ? sc[k] : run[k - 1] + sc[k];  // ... and run their sums inside the piece
        }
#pragma unroll
        for (int k = 0; k < SMS_L - 1; ++k) {
            if (begins >> (k + 1) & 1u) {  // a piece ends at entry k
                const int before = __popc(begins & ((2u << k) - 1u));  // row beginnings up to entry k
                if (before == 0) first_piece = MZ{seg_max[k], run[k]};  // joined with the lanes on the left below
                else table[first_num + before] = make_float2(seg_max[k], run[k]);  // a row inside the lane: final
            }
        }
        cur = MZ{seg_max[SMS_L - 1], run[SMS_L - 1]};
        if (nb == 0) first_piece = cur;
    } else {
        int seen = 0;
#pragma unroll
        for (int k = 0; k < SMS_L; ++k) {
            if (begins >> k & 1u) {
                if (seen == 0) first_piece = cur;                                  // joined with the lanes on the left below
                else table[first_num + seen] = make_float2(cur.m, cur.z);           // a row inside the lane: final
                ++seen;
                cur = Op::identity();
            }
            Op::push(cur, sc[k], sc2[Op::TWO_INPUTS ? k : 0]);
        }
        if (nb == 0) first_piece = cur;
    }
    // one segmented scan over the lanes: what flows into a lane from the left
    const MZ incl = wave_segmented_scan<Op>(cur, nb > 0 ? 1 : 0, lane);  // `cur` is the lane's last (or only) piece
    MZ from_left;
    from_left.m = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(incl.m), 0x138, 0xf, 0xf, false));
    from_left.z = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(incl.z), 0x138, 0xf, 0xf, false));
    if (lane == 0) from_left = Op::identity();
    if (nb > 0) {  // the row that was open at the lane's start ends at the lane's first beginning
        const MZ t = Op::combine(from_left, first_piece);
        if (first_num == 0) carry[2 * static_cast<size_t>(v)] = make_float2(t.m, t.z);  // entered from the left
        else table[first_num] = make_float2(t.m, t.z);
    }
    const int last_num = __shfl(first_num + nb, 63, 64);  // number of the range's last row
    const bool right_open = n_valid == SMS_R && next_row == r_last;
    if (lane == 63) {
        if (last_num == 0) carry[2 * static_cast<size_t>(v)] = make_float2(incl.m, incl.z);  // one row, open on the left
        else if (right_open) carry[2 * static_cast<size_t>(v) + 1] = make_float2(incl.m, incl.z);
        else table[last_num] = make_float2(incl.m, incl.z);
    }
    const int tail_num = (right_open && last_num != 0) ? last_num : -1;
    // LDS operations of one wave execute in order; the fences keep the compiler from moving the
    // table reads above the writes
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // second walk: probabilities of the rows that are complete inside the range
    float pr[SMS_L];
    unsigned done = 0;
    int head_cnt = 0, tail_cnt = 0, num = first_num;
    float2 t = make_float2(0.f, 1.f);
    bool have = false;
#pragma unroll
    for (int k = 0; k < SMS_L; ++k) {
        if (begins >> k & 1u) { ++num; have = false; }
        const bool ok = e0 + k < n_valid;
        const bool in_head = ok && num == 0, in_tail = ok && num == tail_num;
        head_cnt += in_head ? 1 : 0;
        tail_cnt += in_tail ? 1 : 0;
        pr[k] = 0.f;
        if (ok && !in_head && !in_tail) {
            if constexpr (!Op::TWO_INPUTS) {
                if (!have) {  // the factor of this piece of the row
                    t = Op::final_pair(table[num]);
                    t.y *= __expf(seg_max[k] - t.x);
                    have = true;
                }
                pr[k] = sc[k] * t.y;
            } else {
                if (!have) { t = Op::final_pair(table[num]); have = true; }
                pr[k] = Op::result(sc[k], sc2[Op::TWO_INPUTS ? k : 0], t);
            }
            done |= 1u << k;
        }
    }
#pragma unroll
    for (int q = 0; q < SMS_L / 4; ++q) {
        if (VEC && (done >> (4 * q) & 15u) == 15u) {
            *reinterpret_cast<float4 *>(out + base + e0 + 4 * q) = make_float4(pr[4 * q], pr[4 * q + 1], pr[4 * q + 2], pr[4 * q + 3]);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (done >> (4 * q + j) & 1u) out[base + e0 + 4 * q + j] = pr[4 * q + j];
        }
    }
    head_cnt = wave_sum_int(head_cnt);
    tail_cnt = wave_sum_int(tail_cnt);
    const int head_begin = __shfl(ext, 0, 64), head_end = __shfl(ext, 1, 64), tail_end = __shfl(ext, 2, 64);
    if (lane == 0) {
        meta[2 * static_cast<size_t>(v)] = make_int4(head_cnt, n_valid - tail_cnt, tail_num >= 0 ? 1 : -1, head_begin / SMS_R);
        meta[2 * static_cast<size_t>(v) + 1] = make_int4((head_end - 1) / SMS_R, (tail_end - 1) / SMS_R, 0, 0);
    }
}

// The pair of a row cut by range boundaries: its leaving piece in range u_first, the whole ranges in between
// and its entering piece in range u_last, combined in an order that depends on (u_first, u_last) alone.  Every
// wave that holds a piece of the row computes the pair itself and gets the same bits (a row of K ranges is read
// K times by K waves: K is 2 for nearly every cut row and a few dozen for the longest rows of a power-law graph).
template <class Op>
__device__ __forceinline__ MZ cut_row_pair(const float2 *__restrict__ carry, int u_first, int u_last, int lane)
{
    MZ acc = Op::identity();
    bool have = false;
    for (int u = u_first + lane; u <= u_last; u += 64) {
        const float2 t = carry[2 * static_cast<size_t>(u) + (u == u_first ? 1 : 0)];
        acc = have ? Op::combine(acc, MZ{t.x, t.y}) : MZ{t.x, t.y};
        have = true;
    }
    const int n_lanes = min(64, u_last - u_first + 1);  // lanes that hold something
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        MZ o;
        o.m = __shfl_down(acc.m, off, 64);
        o.z = __shfl_down(acc.z, off, 64);
        if (lane + off < n_lanes && lane < off) acc = Op::combine(acc, o);
    }
    MZ r;
    r.m = __shfl(acc.m, 0, 64);
    r.z = __shfl(acc.z, 0, 64);
    return r;
}

// Results of the pieces of cut rows: the entering piece (edges [0, head_len) of the range, row = row of the
// edge before the range) and the leaving piece (edges [tail_start, n_valid)), by the wave that owns the range.
template <class Op>
__global__ __launch_bounds__(256) void softmax_cut_kernel(int nnz, int n_ranges, const float2 *__restrict__ carry,
                                                          const int4 *__restrict__ meta, const float *in,
                                                          const float *in2, float *out)
{
    const int lane = threadIdx.x & 63;
    const int v = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (v >= n_ranges) return;
    const int base = v * SMS_R;
    const int n_valid = min(SMS_R, nnz - base);
    const int4 mt = meta[2 * static_cast<size_t>(v)], mx = meta[2 * static_cast<size_t>(v) + 1];
    if (mt.x > 0) {
        const MZ pr = cut_row_pair<Op>(carry, mt.w, mx.x, lane);
        const float2 st = Op::final_pair(make_float2(pr.m, pr.z));
        for (int i = lane; i < mt.x; i += 64)
            out[base + i] = Op::result(in[base + i], Op::TWO_INPUTS ? in2[base + i] : 0.f, st);
    }
    if (mt.z >= 0) {
        const MZ pr = cut_row_pair<Op>(carry, v, mx.y, lane);  // the row of the leaving piece begins in this range
        const float2 st = Op::final_pair(make_float2(pr.m, pr.z));
        for (int i = mt.y + lane; i < n_valid; i += 64)
            out[base + i] = Op::result(in[base + i], Op::TWO_INPUTS ? in2[base + i] : 0.f, st);
    }
}

size_t softmax_seg_ws(int n, int nnz)
{
    (void)n;
    const size_t n_ranges = (static_cast<size_t>(nnz) + SMS_R - 1) / SMS_R;
    return align_up(n_ranges * 2 * sizeof(float2), 256) + align_up(n_ranges * 2 * sizeof(int4), 256);
}

template <class Op>
static int32_t launch_ranges(const ftc_csr &g, const ftc_windows &w, const float *in, const float *in2, float *out,
                             void *ws, hipStream_t s)
{
    if (g.n == 0 || g.nnz == 0) return FTC_OK;
    const int n_ranges = ceil_div(g.nnz, SMS_R);
    char *p = static_cast<char *>(ws);
    float2 *carry = reinterpret_cast<float2 *>(p);
    p += align_up(static_cast<size_t>(n_ranges) * 2 * sizeof(float2), 256);
    int4 *meta = reinterpret_cast<int4 *>(p);
    // 16-byte loads and stores of the edge arrays when they allow it
    const bool vec = aligned16(in) && aligned16(out) && aligned16(w.edge_to_row) && (!in2 || aligned16(in2));
    if (vec)
        hipLaunchKernelGGL((softmax_local_kernel<Op, true>), dim3((n_ranges + 3) / 4), dim3(256), 0, s, g.nnz,
                           n_ranges, g.row_ptr, w.edge_to_row, in, in2, out, carry, meta);
    else
        hipLaunchKernelGGL((softmax_local_kernel<Op, false>), dim3((n_ranges + 3) / 4), dim3(256), 0, s, g.nnz,
                           n_ranges, g.row_ptr, w.edge_to_row, in, in2, out, carry, meta);
    int32_t st = launch_status("edge_softmax local");
    if (st != FTC_OK) return st;
    hipLaunchKernelGGL(softmax_cut_kernel<Op>, dim3((n_ranges + 3) / 4), dim3(256), 0, s, g.nnz, n_ranges, carry, meta,
                       in, in2, out);
    return launch_status("edge_softmax cut rows");
}

int32_t launch_softmax_seg(const ftc_csr &g, const ftc_windows &w, const float *in, float *out, void *ws,
                           hipStream_t s)
{
    return launch_ranges<SoftmaxFwd>(g, w, in, nullptr, out, ws, s);
}

// ds = p * (dp - sum over the row of p * dp), same workspace as the forward call; ds may alias dp
int32_t launch_softmax_backward_seg(const ftc_csr &g, const ftc_windows &w, const float *p, const float *dp, float *ds,
                                    void *ws, hipStream_t s)
{
    return launch_ranges<SoftmaxBwd>(g, w, p, dp, ds, ws, s);
}

// ------------------------------------------------------------------------------------------------
// Inverse row norms for the AGNN cosine: a group of LPR lanes per row.
template <class T, int LPR>
__global__ __launch_bounds__(256) void row_rnorm_kernel(int n, const void *__restrict__ H, int ld, int D,
                                                        float *__restrict__ rinv)
{
    constexpr int V = T::VEC;
    constexpr int GROUPS = 256 / LPR;
    const int sub = threadIdx.x % LPR;
    const int64_t row = static_cast<int64_t>(blockIdx.x) * GROUPS + threadIdx.x / LPR;
    float q = 0.f;
    if (row < n && sub * V < D) {
        float h[V];
        load_vec<T>(H, row * ld + sub * V, h);
#pragma unroll
        for (int k = 0; k < V; ++k) q = fmaf(h[k], h[k], q);
    }
#pragma unroll
    for (int m = LPR / 2; m >= 1; m >>= 1) q += __shfl_xor(q, m, 64);
    if (row < n && sub == 0) rinv[row] = 1.f / fmaxf(sqrtf(q), 1e-12f);
}

__global__ __launch_bounds__(256) void row_rnorm_generic_kernel(int n, const void *H, int ld, int dt, int D,
                                                                float *rinv)
{
    const int64_t row = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (row >= n) return;
    float q = 0.f;
    for (int k = 0; k < D; ++k) {
        const float h = load_elem(H, row * ld + k, dt);
        q = fmaf(h, h, q);
    }
    rinv[row] = 1.f / fmaxf(sqrtf(q), 1e-12f);
}

template <class T>
static void rnorm_t(int lpr, int n, const void *H, int ld, int D, float *rinv, hipStream_t s)
{
#define FTC_CASE(L)                                                                                    \
    case L: {                                                                                          \
        const unsigned grid = static_cast<unsigned>((static_cast<int64_t>(n) + 256 / L - 1) / (256 / L)); \
        hipLaunchKernelGGL((row_rnorm_kernel<T, L>), dim3(grid), dim3(256), 0, s, n, H, ld, D, rinv);  \
    } break;
    switch (lpr) {
        FTC_CASE(1)
        FTC_CASE(2)
        FTC_CASE(4)
        FTC_CASE(8)
        FTC_CASE(16)
        FTC_CASE(32)
    }
#undef FTC_CASE
}

int32_t launch_row_rnorm(int n, const void *H, int ld, int dt, int D, float *rinv, hipStream_t s)
{
    if (n == 0) return FTC_OK;
    const int v = dt == FTC_F32 ? 4 : 8;
    if (aligned16(H) && (static_cast<int64_t>(ld) * elem_size(dt)) % 16 == 0 && D % v == 0 && D / v <= 32) {
        int lpr = 1;
        while (lpr * v < D) lpr *= 2;
        if (dt == FTC_F32) rnorm_t<F32>(lpr, n, H, ld, D, rinv, s);
        else if (dt == FTC_F16) rnorm_t<F16>(lpr, n, H, ld, D, rinv, s);
        else rnorm_t<BF16>(lpr, n, H, ld, D, rinv, s);
    } else {
        hipLaunchKernelGGL(row_rnorm_generic_kernel, dim3((n + 255) / 256), dim3(256), 0, s, n, H, ld, dt, D,
                           rinv);
    }
    return launch_status("row_rnorm");
}

}  // namespace ftc
