// Locality reordering in preprocessing: a node permutation by degree, the relabelled CSR with
// ascending rows, and the row maps that carry features into the new numbering and results back.
// The sparse graph transformation of Section IV.A condenses the columns the rows of a window share;
// how many they share, and how often a gathered row is still in L2, depends on the numbering of the
// nodes, which the paper takes as given.
//
// Everything here is integer work with a unique result (stable sorts), built on two primitives:
//   * an exclusive scan of int32 (three kernels: block sums, scan of the sums, block scans),
//   * a stable least-significant-digit radix sort of (key, value) pairs with 8-bit digits.
// The radix pass splits the input into wave tiles of RX_TILE consecutive elements.  A histogram
// kernel counts the digits of every tile, the scan over the (digit, tile) table gives every tile
// the first output position of each of its digits, and the scatter kernel walks the tile 64
// elements at a time: lanes that hold the same digit find each other with eight ballots, take
// consecutive positions in lane order and advance the tile's position for that digit.  A wave works
// alone on its tile (no workgroup barriers); element order inside a digit is preserved.
#include "ftc_common.hpp"

namespace ftc {

// ---- exclusive scan ---------------------------------------------------------------------------
constexpr int SC_ITEMS = 16;
constexpr int SC_BLOCK = 256 * SC_ITEMS;  // elements per workgroup

__device__ __forceinline__ int block_exclusive_scan(int v, int *total)
{
    __shared__ int wave_sums[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int incl = wave_inclusive_scan(v);
    __syncthreads();  // wave_sums of a previous call are consumed
    if (lane == 63) wave_sums[wave] = incl;
    __syncthreads();
    int before = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) before += w < wave ? wave_sums[w] : 0;
    *total = wave_sums[0] + wave_sums[1] + wave_sums[2] + wave_sums[3];
    return before + incl - v;
}

__global__ __launch_bounds__(256) void scan_sums_kernel(const int *__restrict__ in, int64_t count, int *__restrict__ sums)
{
    const int64_t base = static_cast<int64_t>(blockIdx.x) * SC_BLOCK + threadIdx.x * SC_ITEMS;
    int t = 0;
#pragma unroll
    for (int k = 0; k < SC_ITEMS; ++k) t += base + k < count ? in[base + k] : 0;
    int total;
    block_exclusive_scan(t, &total);
    if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

// one workgroup: sums[i] <- sum of sums[0 .. i); sums[n_sums] <- grand total
__global__ __launch_bounds__(256) void scan_of_sums_kernel(int *sums, int n_sums)
{
    int carry = 0;
    for (int base = 0; base < n_sums; base += 256) {
        const int i = base + threadIdx.x;
        const int v = i < n_sums ? sums[i] : 0;
        int total;
        const int ex = block_exclusive_scan(v, &total);
        if (i < n_sums) sums[i] = carry + ex;
        carry += total;
    }
    if (threadIdx.x == 0) sums[n_sums] = carry;
}

// out[i] = sum of in[0 .. i); out[count] = total when `with_total`.  in == out is allowed.
__global__ __launch_bounds__(256) void scan_apply_kernel(const int *in, int64_t count, const int *__restrict__ sums,
                                                         int n_sums, int *out, int with_total)
{
    const int64_t base = static_cast<int64_t>(blockIdx.x) * SC_BLOCK + threadIdx.x * SC_ITEMS;
    int v[SC_ITEMS], t = 0;
#pragma unroll
    for (int k = 0; k < SC_ITEMS; ++k) {
        v[k] = base + k < count ? in[base + k] : 0;
        t += v[k];
    }
    int total;
    int run = sums[blockIdx.x] + block_exclusive_scan(t, &total);
#pragma unroll
    for (int k = 0; k < SC_ITEMS; ++k) {
        if (base + k < count) out[base + k] = run;
        run += v[k];
    }
    if (with_total && blockIdx.x == 0 && threadIdx.x == 0) out[count] = sums[n_sums];
}

static size_t scan_ws(int64_t count) { return align_up(((count + SC_BLOCK - 1) / SC_BLOCK + 1) * sizeof(int), 256); }

static int32_t exclusive_scan(const int *in, int64_t count, int *out, bool with_total, void *ws, hipStream_t s)
{
    if (count <= 0) return FTC_OK;
    const int n_sums = static_cast<int>((count + SC_BLOCK - 1) / SC_BLOCK);
    int *sums = static_cast<int *>(ws);
    hipLaunchKernelGGL(scan_sums_kernel, dim3(n_sums), dim3(256), 0, s, in, count, sums);
    hipLaunchKernelGGL(scan_of_sums_kernel, dim3(1), dim3(256), 0, s, sums, n_sums);
    hipLaunchKernelGGL(scan_apply_kernel, dim3(n_sums), dim3(256), 0, s, in, count, sums, n_sums, out,
                       with_total ? 1 : 0);
    return launch_status("exclusive scan");
}

// ---- stable radix sort of pairs ----------------------------------------------------------------
constexpr int RX_ROUNDS = 32;
constexpr int RX_TILE = 64 * RX_ROUNDS;  // elements per wave

__device__ __forceinline__ void wave_lds_fence()
{
    // LDS operations of one wave execute in order; the fences keep the compiler from reordering them
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__global__ __launch_bounds__(256) void radix_hist_kernel(const uint32_t *__restrict__ keys, int64_t count, int shift,
                                                         int64_t n_tiles, int *__restrict__ hist)
{
    __shared__ int cnt_all[4][256];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t tile = static_cast<int64_t>(blockIdx.x) * 4 + wave;
    if (tile >= n_tiles) return;  // no workgroup barrier below
    int *cnt = cnt_all[wave];
#pragma unroll
    for (int k = 0; k < 4; ++k) cnt[lane + 64 * k] = 0;
    wave_lds_fence();
    const int64_t base = tile * RX_TILE;
#pragma unroll 8
    for (int r = 0; r < RX_ROUNDS; ++r) {
        const int64_t i = base + r * 64 + lane;
        if (i < count) atomicAdd(&cnt[(keys[i] >> shift) & 255u], 1);
    }
    wave_lds_fence();
#pragma unroll
    for (int k = 0; k < 4; ++k) hist[(lane + 64 * k) * n_tiles + tile] = cnt[lane + 64 * k];
}

__global__ __launch_bounds__(256) void radix_scatter_kernel(const uint32_t *__restrict__ keys,
                                                            const uint32_t *__restrict__ vals, int64_t count,
                                                            int shift, int64_t n_tiles, const int *__restrict__ pos,
                                                            uint32_t *__restrict__ keys_out,
                                                            uint32_t *__restrict__ vals_out)
{
    __shared__ int next_all[4][256];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t tile = static_cast<int64_t>(blockIdx.x) * 4 + wave;
    if (tile >= n_tiles) return;  // no workgroup barrier below
    int *next = next_all[wave];
#pragma unroll
    for (int k = 0; k < 4; ++k) next[lane + 64 * k] = pos[(lane + 64 * k) * n_tiles + tile];
    wave_lds_fence();
    const int64_t base = tile * RX_TILE;
    const uint64_t below = (1ull << lane) - 1ull;
    // the whole tile is loaded before the first element is placed: 2 * RX_ROUNDS loads in flight per lane
    uint32_t key[RX_ROUNDS], val[RX_ROUNDS];
#pragma unroll
    for (int r = 0; r < RX_ROUNDS; ++r) {
        const int64_t i = base + r * 64 + lane;
        key[r] = i < count ? keys[i] : 0u;
        val[r] = i < count ? vals[i] : 0u;
    }
#pragma unroll
    for (int r = 0; r < RX_ROUNDS; ++r) {
        const bool ok = base + r * 64 + lane < count;
        const uint32_t d = (key[r] >> shift) & 255u;
        uint64_t peers = __builtin_amdgcn_ballot_w64(ok);  // lanes that hold the same digit
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const bool bit = (d >> b) & 1u;
            const uint64_t with_bit = __builtin_amdgcn_ballot_w64(bit);
            peers &= bit ? with_bit : ~with_bit;
        }
        const int rank = __popcll(peers & below);
        const int first = ok ? next[d] : 0;
        wave_lds_fence();
        if (ok && rank == 0) next[d] = first + __popcll(peers);
        wave_lds_fence();
        if (ok) {
            keys_out[first + rank] = key[r];
            vals_out[first + rank] = val[r];
        }
    }
}

static int64_t radix_tiles(int64_t count) { return (count + RX_TILE - 1) / RX_TILE; }

static size_t radix_ws(int64_t count)
{
    const int64_t table = 256 * radix_tiles(count);
    return align_up(static_cast<size_t>(table) * sizeof(int), 256) + scan_ws(table);
}

// Sorts `count` pairs by the low `bits` bits of the key, ascending and stable.  Input in (k0, v0);
// the passes alternate between (k0, v0) and (k1, v1); the values of the last pass go to `v_final`
// when it is not NULL.  *k_result / *v_result point at the sorted arrays.
static int32_t radix_sort_pairs(uint32_t *k0, uint32_t *v0, uint32_t *k1, uint32_t *v1, int64_t count, int bits,
                                uint32_t *v_final, uint32_t **k_result, uint32_t **v_result, void *ws, hipStream_t s)
{
    *k_result = k0;
    *v_result = v0;
    if (count <= 0) return FTC_OK;
    const int passes = (bits + 7) / 8 < 1 ? 1 : (bits + 7) / 8;
    const int64_t n_tiles = radix_tiles(count);
    if (256 * n_tiles > INT32_MAX) {
        set_error("radix sort: %lld elements are more than the digit table can index", static_cast<long long>(count));
        return FTC_EUNSUPPORTED;
    }
    int *table = static_cast<int *>(ws);
    void *ws_scan = static_cast<char *>(ws) + align_up(static_cast<size_t>(256 * n_tiles) * sizeof(int), 256);
    const unsigned grid = static_cast<unsigned>((n_tiles + 3) / 4);
    uint32_t *ki = k0, *vi = v0, *ko = k1, *vo = v1;
    for (int p = 0; p < passes; ++p) {
        uint32_t *v_dst = (p == passes - 1 && v_final) ? v_final : vo;
        hipLaunchKernelGGL(radix_hist_kernel, dim3(grid), dim3(256), 0, s, ki, count, 8 * p, n_tiles, table);
        const int32_t st = exclusive_scan(table, 256 * n_tiles, table, false, ws_scan, s);
        if (st != FTC_OK) return st;
        hipLaunchKernelGGL(radix_scatter_kernel, dim3(grid), dim3(256), 0, s, ki, vi, count, 8 * p, n_tiles, table, ko,
                           v_dst);
        *k_result = ko;
        *v_result = v_dst;
        uint32_t *t = ki; ki = ko; ko = t;
        t = vi; vi = vo; vo = t;
    }
    return launch_status("radix sort");
}

static int bit_length(uint32_t x)
{
    int b = 0;
    while (x) { ++b; x >>= 1; }
    return b;
}

__global__ void reorder_set_int_kernel(int *p, int v) { *p = v; }

// ---- degree statistics ---------------------------------------------------------------------------
// stats[0] = sum of squared row lengths, stats[1] = longest row (both exact integers).
__global__ __launch_bounds__(256) void degree_stats_kernel(int n, const int *__restrict__ row_ptr,
                                                           unsigned long long *__restrict__ stats)
{
    __shared__ unsigned long long red_s[4], red_m[4];
    unsigned long long sq = 0, mx = 0;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; i < n; i += static_cast<int64_t>(gridDim.x) * 256) {
        const unsigned long long d = static_cast<unsigned long long>(row_ptr[i + 1] - row_ptr[i]);
        sq += d * d;
        mx = d > mx ? d : mx;
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        sq += __shfl_xor(sq, m, 64);
        const unsigned long long o = __shfl_xor(mx, m, 64);
        mx = o > mx ? o : mx;
    }
    if ((threadIdx.x & 63) == 0) { red_s[threadIdx.x >> 6] = sq; red_m[threadIdx.x >> 6] = mx; }
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long m2 = red_m[0];
        for (int w = 1; w < 4; ++w) m2 = red_m[w] > m2 ? red_m[w] : m2;
        atomicAdd(&stats[0], red_s[0] + red_s[1] + red_s[2] + red_s[3]);
        atomicMax(&stats[1], m2);
    }
}

__global__ void clear_stats_kernel(unsigned long long *stats) { stats[0] = 0; stats[1] = 0; }

int32_t launch_degree_stats(const ftc_csr &g, int64_t *stats, hipStream_t s)
{
    unsigned long long *st = reinterpret_cast<unsigned long long *>(stats);
    hipLaunchKernelGGL(clear_stats_kernel, dim3(1), dim3(1), 0, s, st);
    if (g.n > 0) {
        const int blocks = (g.n + 255) / 256 < 1024 ? (g.n + 255) / 256 : 1024;
        hipLaunchKernelGGL(degree_stats_kernel, dim3(blocks), dim3(256), 0, s, g.n, g.row_ptr, st);
    }
    return launch_status("degree statistics");
}

// ---- degree order --------------------------------------------------------------------------------
// key = largest key - (degree or its bit length): ascending sort = descending degree; value = node id
__global__ __launch_bounds__(256) void degree_keys_kernel(int n, const int *__restrict__ row_ptr, int mode,
                                                          uint32_t *__restrict__ keys, uint32_t *__restrict__ vals)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const uint32_t deg = static_cast<uint32_t>(row_ptr[i + 1] - row_ptr[i]);
    keys[i] = mode == FTC_ORDER_DEGREE ? 0x7fffffffu - deg : 32u - static_cast<uint32_t>(32 - __clz(deg));
    vals[i] = static_cast<uint32_t>(i);
}

__global__ __launch_bounds__(256) void invert_perm_kernel(int n, const int *__restrict__ perm, int *__restrict__ inv)
{
    const int r = blockIdx.x * 256 + threadIdx.x;
    if (r < n) inv[perm[r]] = r;
}

size_t label_propagation_ws(int n, int nnz);

size_t reorder_ws(int n, int nnz)
{
    const int64_t m = n > nnz ? n : nnz;
    const size_t order = 4 * align_up(static_cast<size_t>(m) * sizeof(uint32_t), 256) + radix_ws(m) + scan_ws(static_cast<int64_t>(n) + 1);
    const size_t lpa = label_propagation_ws(n, nnz);
    return order > lpa ? order : lpa;
}

int32_t launch_degree_order(const ftc_csr &g, int mode, int *perm, int *inv, void *ws, hipStream_t s)
{
    const int n = g.n;
    if (n == 0) return FTC_OK;
    const size_t arr = align_up(static_cast<size_t>(n) * sizeof(uint32_t), 256);
    char *p = static_cast<char *>(ws);
    uint32_t *k0 = reinterpret_cast<uint32_t *>(p), *v0 = reinterpret_cast<uint32_t *>(p + arr);
    uint32_t *k1 = reinterpret_cast<uint32_t *>(p + 2 * arr), *v1 = reinterpret_cast<uint32_t *>(p + 3 * arr);
    void *ws_sort = p + 4 * arr;
    hipLaunchKernelGGL(degree_keys_kernel, dim3((n + 255) / 256), dim3(256), 0, s, n, g.row_ptr, mode, k0, v0);
    uint32_t *kr, *vr;
    const int bits = mode == FTC_ORDER_DEGREE ? 31 : 6;
    const int32_t st = radix_sort_pairs(k0, v0, k1, v1, n, bits, reinterpret_cast<uint32_t *>(perm), &kr, &vr, ws_sort, s);
    if (st != FTC_OK) return st;
    hipLaunchKernelGGL(invert_perm_kernel, dim3((n + 255) / 256), dim3(256), 0, s, n, perm, inv);
    return launch_status("degree order");
}

// ---- order by key ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void key_pairs_kernel(int n, const int *__restrict__ keys_in, uint32_t *__restrict__ keys,
                                                        uint32_t *__restrict__ vals, int *flag)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const int k = keys_in[i];
    if (k < 0) atomicOr(flag, 1);  // negative keys are not ordered: reported, treated as 0
    keys[i] = k < 0 ? 0u : static_cast<uint32_t>(k);
    vals[i] = static_cast<uint32_t>(i);
}

int32_t launch_order_by_key(int n, const int *keys_in, int *perm, int *inv, int *flag, void *ws, hipStream_t s)
{
    hipLaunchKernelGGL(reorder_set_int_kernel, dim3(1), dim3(1), 0, s, flag, 0);
    if (n == 0) return launch_status("order by key");
    const size_t arr = align_up(static_cast<size_t>(n) * sizeof(uint32_t), 256);
    char *p = static_cast<char *>(ws);
    uint32_t *k0 = reinterpret_cast<uint32_t *>(p), *v0 = reinterpret_cast<uint32_t *>(p + arr);
    uint32_t *k1 = reinterpret_cast<uint32_t *>(p + 2 * arr), *v1 = reinterpret_cast<uint32_t *>(p + 3 * arr);
    void *ws_sort = p + 4 * arr;
    hipLaunchKernelGGL(key_pairs_kernel, dim3((n + 255) / 256), dim3(256), 0, s, n, keys_in, k0, v0, flag);
    uint32_t *kr, *vr;
    const int32_t st = radix_sort_pairs(k0, v0, k1, v1, n, 31, reinterpret_cast<uint32_t *>(perm), &kr, &vr, ws_sort, s);
    if (st != FTC_OK) return st;
    hipLaunchKernelGGL(invert_perm_kernel, dim3((n + 255) / 256), dim3(256), 0, s, n, perm, inv);
    return launch_status("order by key");
}

// ---- label propagation ---------------------------------------------------------------------------
// Every round: pairs (label of the entry's column, row) sorted by label and then, stably, by row put
// equal labels of a row side by side; a run of equal (row, label) is one candidate, its length the
// number of votes.  The candidate with the most votes and, among those, the smallest label wins:
// the maximum of (votes << 32 | ~label), taken with a 64-bit atomic maximum per row (the maximum
// does not depend on the order of the updates, so the result is reproducible).
__global__ __launch_bounds__(256) void entry_rows_kernel(int n, int nnz, const int *__restrict__ row_ptr,
                                                         uint32_t *__restrict__ rows)
{
    const int64_t e = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (e >= nnz) return;
    int a = 0, b = n;  // last row with row_ptr[row] <= e
    while (b - a > 1) {
        const int mid = (a + b) >> 1;
        if (row_ptr[mid] <= e) a = mid; else b = mid;
    }
    rows[e] = static_cast<uint32_t>(a);
}

__global__ __launch_bounds__(256) void iota_kernel(int n, int *__restrict__ out)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) out[i] = i;
}

__global__ __launch_bounds__(256) void gather_labels_kernel(int n, int nnz, const int *__restrict__ col_idx,
                                                            const int *__restrict__ label,
                                                            const uint32_t *__restrict__ rows,
                                                            uint32_t *__restrict__ keys, uint32_t *__restrict__ vals)
{
    const int64_t e = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (e >= nnz) return;
    const int c = col_idx[e];
    keys[e] = (c >= 0 && c < n) ? static_cast<uint32_t>(label[c]) : 0u;  // a column out of range votes for label 0
    vals[e] = rows[e];
}

// flags[p] = 1 where a run of equal (row, label) begins; sorted_rows / sorted_labels are grouped by row
__global__ __launch_bounds__(256) void run_flags_kernel(int nnz, const uint32_t *__restrict__ sorted_rows,
                                                        const uint32_t *__restrict__ sorted_labels, int *__restrict__ flags)
{
    const int64_t p = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (p >= nnz) return;
    flags[p] = (p == 0 || sorted_rows[p] != sorted_rows[p - 1] || sorted_labels[p] != sorted_labels[p - 1]) ? 1 : 0;
}

// run_id[p] (exclusive scan of the flags) -> starts[run] = p at every run start
__global__ __launch_bounds__(256) void run_starts_kernel(int nnz, const uint32_t *__restrict__ sorted_rows,
                                                         const uint32_t *__restrict__ sorted_labels,
                                                         const int *__restrict__ run_id, int *__restrict__ starts)
{
    const int64_t p = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (p >= nnz) return;
    if (p == 0 || sorted_rows[p] != sorted_rows[p - 1] || sorted_labels[p] != sorted_labels[p - 1]) starts[run_id[p]] = static_cast<int>(p);
}

__global__ __launch_bounds__(256) void clear_u64_kernel(int n, unsigned long long *a)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) a[i] = 0ull;
}

// one thread per run; n_runs = run_id[nnz] (the scan's total)
__global__ __launch_bounds__(256) void run_votes_kernel(int nnz, const int *__restrict__ n_runs_ptr,
                                                        const int *__restrict__ starts,
                                                        const uint32_t *__restrict__ sorted_rows,
                                                        const uint32_t *__restrict__ sorted_labels,
                                                        unsigned long long *__restrict__ best)
{
    const int n_runs = *n_runs_ptr;
    for (int64_t r = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; r < n_runs; r += static_cast<int64_t>(gridDim.x) * 256) {
        const int p = starts[r];
        const int end = r + 1 < n_runs ? starts[r + 1] : nnz;
        const unsigned long long cand = (static_cast<unsigned long long>(end - p) << 32) | (0xffffffffu - sorted_labels[p]);
        atomicMax(&best[sorted_rows[p]], cand);
    }
}

__global__ __launch_bounds__(256) void take_labels_kernel(int n, const unsigned long long *__restrict__ best,
                                                          int *__restrict__ label)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const unsigned long long b = best[i];
    if (b != 0ull) label[i] = static_cast<int>(0xffffffffu - static_cast<uint32_t>(b & 0xffffffffull));
}

size_t label_propagation_ws(int n, int nnz)
{
    const int64_t m = n > nnz ? n : nnz;
    const size_t arr = align_up(static_cast<size_t>(m) * sizeof(uint32_t), 256);
    // rows, four pair buffers, run ids (+ total), starts, best votes, sort and scan scratch
    return 5 * arr + 2 * align_up((static_cast<size_t>(m) + 1) * sizeof(int), 256) +
           align_up(static_cast<size_t>(n) * sizeof(unsigned long long), 256) + radix_ws(m) + scan_ws(static_cast<int64_t>(m) + 1);
}

int32_t launch_label_propagation(const ftc_csr &g, int iters, int *labels, void *ws, hipStream_t s)
{
    const int n = g.n, nnz = g.nnz;
    if (n == 0) return FTC_OK;
    hipLaunchKernelGGL(iota_kernel, dim3((n + 255) / 256), dim3(256), 0, s, n, labels);
    if (nnz == 0 || iters <= 0) return launch_status("label propagation");
    const int64_t m = n > nnz ? n : nnz;
    const size_t arr = align_up(static_cast<size_t>(m) * sizeof(uint32_t), 256);
    const size_t arr1 = align_up((static_cast<size_t>(m) + 1) * sizeof(int), 256);
    char *p = static_cast<char *>(ws);
    uint32_t *rows = reinterpret_cast<uint32_t *>(p); p += arr;
    uint32_t *k0 = reinterpret_cast<uint32_t *>(p); p += arr;
    uint32_t *v0 = reinterpret_cast<uint32_t *>(p); p += arr;
    uint32_t *k1 = reinterpret_cast<uint32_t *>(p); p += arr;
    uint32_t *v1 = reinterpret_cast<uint32_t *>(p); p += arr;
    int *run_id = reinterpret_cast<int *>(p); p += arr1;
    int *starts = reinterpret_cast<int *>(p); p += arr1;
    unsigned long long *best = reinterpret_cast<unsigned long long *>(p);
    p += align_up(static_cast<size_t>(n) * sizeof(unsigned long long), 256);
    void *ws_sort = p; p += radix_ws(m);
    void *ws_scan = p;
    const unsigned ge = static_cast<unsigned>(ceil_div(nnz, 256)), gn = static_cast<unsigned>((n + 255) / 256);
    hipLaunchKernelGGL(entry_rows_kernel, dim3(ge), dim3(256), 0, s, n, nnz, g.row_ptr, rows);
    const int bits = bit_length(static_cast<uint32_t>(n - 1));
    for (int it = 0; it < iters; ++it) {
        hipLaunchKernelGGL(gather_labels_kernel, dim3(ge), dim3(256), 0, s, n, nnz, g.col_idx, labels, rows, k0, v0);
        uint32_t *kr, *vr;  // after the first sort: keys = labels, values = rows
        int32_t st = radix_sort_pairs(k0, v0, k1, v1, nnz, bits, nullptr, &kr, &vr, ws_sort, s);
        if (st != FTC_OK) return st;
        uint32_t *k_other = kr == k0 ? k1 : k0, *v_other = vr == v0 ? v1 : v0;
        uint32_t *rows_sorted, *labels_sorted;  // second sort: keys = rows, values = labels
        st = radix_sort_pairs(vr, kr, v_other, k_other, nnz, bits, nullptr, &rows_sorted, &labels_sorted, ws_sort, s);
        if (st != FTC_OK) return st;
        hipLaunchKernelGGL(run_flags_kernel, dim3(ge), dim3(256), 0, s, nnz, rows_sorted, labels_sorted, run_id);
        st = exclusive_scan(run_id, nnz, run_id, true, ws_scan, s);  // run_id[nnz] = number of runs
        if (st != FTC_OK) return st;
        hipLaunchKernelGGL(run_starts_kernel, dim3(ge), dim3(256), 0, s, nnz, rows_sorted, labels_sorted, run_id, starts);
        hipLaunchKernelGGL(clear_u64_kernel, dim3(gn), dim3(256), 0, s, n, best);
        hipLaunchKernelGGL(run_votes_kernel, dim3(ge < 4096u ? ge : 4096u), dim3(256), 0, s, nnz, run_id + nnz, starts,
                           rows_sorted, labels_sorted, best);
        hipLaunchKernelGGL(take_labels_kernel, dim3(gn), dim3(256), 0, s, n, best, labels);
    }
    return launch_status("label propagation");
}

// ---- relabelled graph ----------------------------------------------------------------------------
// A (perm, inv) pair that is not a permutation and its inverse sets *flag and loses the entries of
// the rows concerned; no index is followed before it is checked.
__global__ __launch_bounds__(256) void permuted_degrees_kernel(int n, const int *__restrict__ row_ptr,
                                                               const int *__restrict__ perm,
                                                               const int *__restrict__ inv, int *__restrict__ deg_out,
                                                               int *flag)
{
    const int r = blockIdx.x * 256 + threadIdx.x;
    if (r >= n) return;
    const int old = perm[r];
    const bool ok = old >= 0 && old < n && inv[old] == r;
    deg_out[r] = ok ? row_ptr[old + 1] - row_ptr[old] : 0;
    if (!ok) atomicOr(flag, 1);
}

// One thread per stored entry of the old graph: its row by binary search, its place in the new row
// (same offset inside the row), key = new column, value = new row.
__global__ __launch_bounds__(256) void relabel_kernel(int n, int nnz, const int *__restrict__ row_ptr,
                                                      const int *__restrict__ col_idx, const int *__restrict__ inv,
                                                      const int *__restrict__ perm,
                                                      const int *__restrict__ row_ptr_new,
                                                      uint32_t *__restrict__ keys, uint32_t *__restrict__ vals,
                                                      int *flag)
{
    const int64_t e = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (e >= nnz) return;
    int a = 0, b = n;  // last row with row_ptr[row] <= e
    while (b - a > 1) {
        const int mid = (a + b) >> 1;
        if (row_ptr[mid] <= e) a = mid; else b = mid;
    }
    const int r_new = inv[a];
    const int c = col_idx[e];
    const int c_new = (c >= 0 && c < n) ? inv[c] : -1;
    const bool ok = r_new >= 0 && r_new < n && perm[r_new] == a && c_new >= 0 && c_new < n;
    if (!ok) {
        atomicOr(flag, 1);
        return;
    }
    const int64_t dst = static_cast<int64_t>(row_ptr_new[r_new]) + (e - row_ptr[a]);  // < nnz: perm[r_new] == a
    keys[dst] = static_cast<uint32_t>(c_new);
    vals[dst] = static_cast<uint32_t>(r_new);
}

// keys the relabel kernel leaves unwritten (only for an invalid permutation) must still be defined
__global__ __launch_bounds__(256) void fill_u32_kernel(uint32_t *a, uint32_t *b, int64_t count)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i < count) { a[i] = 0u; b[i] = 0u; }
}

int32_t launch_permute_graph(const ftc_csr &g, const int *perm, const int *inv, int *row_ptr_out, int *col_idx_out,
                             int *flag, void *ws, hipStream_t s)
{
    const int n = g.n, nnz = g.nnz;
    if (n == 0) return FTC_OK;
    const int64_t m = n > nnz ? n : nnz;
    const size_t arr = align_up(static_cast<size_t>(m) * sizeof(uint32_t), 256);
    char *p = static_cast<char *>(ws);
    uint32_t *k0 = reinterpret_cast<uint32_t *>(p), *v0 = reinterpret_cast<uint32_t *>(p + arr);
    uint32_t *k1 = reinterpret_cast<uint32_t *>(p + 2 * arr), *v1 = reinterpret_cast<uint32_t *>(p + 3 * arr);
    void *ws_sort = p + 4 * arr;
    void *ws_scan = static_cast<char *>(ws_sort) + radix_ws(m);
    hipLaunchKernelGGL(reorder_set_int_kernel, dim3(1), dim3(1), 0, s, flag, 0);
    // new row pointers: scan of the permuted degrees (staged in k1, free until the first sorting pass)
    int *deg = reinterpret_cast<int *>(k1);
    hipLaunchKernelGGL(permuted_degrees_kernel, dim3((n + 255) / 256), dim3(256), 0, s, n, g.row_ptr, perm, inv, deg,
                       flag);
    int32_t st = exclusive_scan(deg, n, row_ptr_out, true, ws_scan, s);
    if (st != FTC_OK) return st;
    if (nnz == 0) return FTC_OK;
    hipLaunchKernelGGL(fill_u32_kernel, dim3(ceil_div(nnz, 256)), dim3(256), 0, s, k0, v0, static_cast<int64_t>(nnz));
    hipLaunchKernelGGL(relabel_kernel, dim3(ceil_div(nnz, 256)), dim3(256), 0, s, n, nnz, g.row_ptr, g.col_idx, inv, perm,
                       row_ptr_out, k0, v0, flag);
    // ascending (row, column): stable sort by column, then by row (rows are the values of the first
    // sort and the keys of the second)
    const int bits = bit_length(static_cast<uint32_t>(n - 1));
    uint32_t *kr, *vr;
    st = radix_sort_pairs(k0, v0, k1, v1, nnz, bits, nullptr, &kr, &vr, ws_sort, s);
    if (st != FTC_OK) return st;
    uint32_t *k_other = kr == k0 ? k1 : k0, *v_other = vr == v0 ? v1 : v0;
    uint32_t *kr2, *vr2;
    st = radix_sort_pairs(vr, kr, v_other, k_other, nnz, bits, reinterpret_cast<uint32_t *>(col_idx_out), &kr2, &vr2,
                          ws_sort, s);
    return st;
}

// ---- out[r] = X[map[r]] --------------------------------------------------------------------------
// 16 bytes per lane when the rows allow it, else element by element.
// A map entry outside [0, n) gives a row of zeros.
__global__ __launch_bounds__(256) void permute_rows_vec_kernel(int64_t n, int pieces, const uint4 *__restrict__ X,
                                                               int64_t ldx16, const int *__restrict__ map,
                                                               uint4 *__restrict__ out, int64_t ldo16)
{
    const int64_t t = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (t >= n * pieces) return;
    const int64_t r = t / pieces;
    const int k = static_cast<int>(t % pieces);
    const int src = map[r];
    out[r * ldo16 + k] = (src >= 0 && src < n) ? X[static_cast<int64_t>(src) * ldx16 + k] : make_uint4(0u, 0u, 0u, 0u);
}

__global__ __launch_bounds__(256) void permute_rows_kernel(int64_t n, int D, const void *__restrict__ X, int64_t ldx,
                                                           int dt, const int *__restrict__ map, void *__restrict__ out,
                                                           int64_t ldo)
{
    const int64_t t = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (t >= n * D) return;
    const int64_t r = t / D;
    const int k = static_cast<int>(t % D);
    const int m = map[r];
    const bool ok = m >= 0 && m < n;
    const int64_t src = static_cast<int64_t>(ok ? m : 0) * ldx + k;
    if (dt == FTC_F32) static_cast<float *>(out)[r * ldo + k] = ok ? static_cast<const float *>(X)[src] : 0.f;
    else static_cast<uint16_t *>(out)[r * ldo + k] = ok ? static_cast<const uint16_t *>(X)[src] : uint16_t(0);
}

int32_t launch_permute_rows(int n, const void *X, int ldx, int dt, int D, const int *map, void *out, int ldo,
                            hipStream_t s)
{
    if (n == 0) return FTC_OK;
    const int es = elem_size(dt);
    const int64_t row_bytes = static_cast<int64_t>(D) * es;
    if (row_bytes % 16 == 0 && (static_cast<int64_t>(ldx) * es) % 16 == 0 && (static_cast<int64_t>(ldo) * es) % 16 == 0 &&
        aligned16(X) && aligned16(out)) {
        const int pieces = static_cast<int>(row_bytes / 16);
        const int64_t total = static_cast<int64_t>(n) * pieces;
        hipLaunchKernelGGL(permute_rows_vec_kernel, dim3(static_cast<unsigned>((total + 255) / 256)), dim3(256), 0, s, n,
                           pieces, static_cast<const uint4 *>(X), static_cast<int64_t>(ldx) * es / 16, map,
                           static_cast<uint4 *>(out), static_cast<int64_t>(ldo) * es / 16);
    } else {
        const int64_t total = static_cast<int64_t>(n) * D;
        hipLaunchKernelGGL(permute_rows_kernel, dim3(static_cast<unsigned>((total + 255) / 256)), dim3(256), 0, s, n, D, X,
                           ldx, dt, map, out, ldo);
    }
    return launch_status("permute rows");
}

}  // namespace ftc
