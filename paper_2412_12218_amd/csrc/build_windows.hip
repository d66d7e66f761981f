// Sparse graph transformation (Section V.A) on the GPU.
//
// Every row window is independent (the paper parallelises the same step over CPU threads), so
// one workgroup condenses one window:
//   1. edge_to_row for the window's edges,
//   2. small windows (at most SMALL_CAP edges): bitonic sort of the column ids in LDS, strict
//      de-duplication by a flag scan, rank of every edge by binary search in the unique list;
//   3. large windows (hub rows of power-law graphs) are queued and condensed by a second kernel
//      with a bitmap over the n column ids kept in the workspace: set bits, prefix sum of the
//      per-word popcounts, rank = prefix + popcount of the lower bits.
// The unique lists are first written at the window's edge offset of a temporary array (a
// window never has more distinct columns than edges), then a scan over the windows gives
// win_col_ptr / block_partition / summary and a last kernel packs the lists into win_cols.
#include "ftc_common.hpp"

namespace ftc {

constexpr int SMALL_CAP = 4096;  // edges per window handled in LDS
constexpr int BIG_SLOTS_MAX = 256;  // concurrent bitmap slots for large windows (one per CU)
constexpr int BIG_THREADS = 1024;

struct WinWorkspace {
    int *uniq_count;  // [n_windows]
    int *big_list;    // [n_windows]
    int *big_count;   // [1]
    int *tmp_cols;    // [nnz]
    uint32_t *bitmaps;  // [slots][2 * words]: bits, then exclusive popcount prefix per word
    size_t words;
    int slots;
    size_t total;
};

static WinWorkspace carve(void *ws, int n, int nnz, int n_windows)
{
    WinWorkspace w;
    char *p = static_cast<char *>(ws);
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char *q = p ? p + off : nullptr;
        off += align_up(bytes, 256);
        return q;
    };
    w.uniq_count = reinterpret_cast<int *>(take(sizeof(int) * static_cast<size_t>(n_windows)));
    w.big_list = reinterpret_cast<int *>(take(sizeof(int) * static_cast<size_t>(n_windows)));
    w.big_count = reinterpret_cast<int *>(take(sizeof(int)));
    w.tmp_cols = reinterpret_cast<int *>(take(sizeof(int) * static_cast<size_t>(nnz)));
    w.words = (static_cast<size_t>(n) + 31) / 32;
    // two words of workspace per 32 columns and slot; at most 64 MiB in total, at least 8 slots
    size_t slots = w.words ? (size_t(64) << 20) / (w.words * 2 * sizeof(uint32_t)) : BIG_SLOTS_MAX;
    w.slots = static_cast<int>(slots < 8 ? 8 : (slots > BIG_SLOTS_MAX ? BIG_SLOTS_MAX : slots));
    w.bitmaps = reinterpret_cast<uint32_t *>(take(sizeof(uint32_t) * 2 * w.words * w.slots));
    w.total = off;
    return w;
}

size_t build_windows_ws(int n, int nnz, int blk_h, int blk_w)
{
    (void)blk_w;
    const int n_windows = (n + blk_h - 1) / blk_h;
    return carve(nullptr, n, nnz, n_windows).total;
}

// Exclusive scan of one int per thread over a workgroup of NT threads (NT multiple of 64).
// `tmp` holds NT / 64 + 1 ints of LDS.  Returns the exclusive prefix; *total gets the sum.
template <int NT>
__device__ __forceinline__ int block_exclusive_scan(int v, int *tmp, int *total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int incl = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int up = __shfl_up(incl, d, 64);
        if (lane >= d) incl += up;
    }
    __syncthreads();  // protects tmp against the previous use
    if (lane == 63) tmp[wave] = incl;
    __syncthreads();
    if (threadIdx.x == 0) {
        int run = 0;
        for (int k = 0; k < NT / 64; ++k) {
            const int t = tmp[k];
            tmp[k] = run;
            run += t;
        }
        tmp[NT / 64] = run;
    }
    __syncthreads();
    *total = tmp[NT / 64];
    return tmp[wave] + incl - v;
}

__global__ void win_clear_kernel(int *counter) { *counter = 0; }

__global__ __launch_bounds__(256) void win_small_kernel(int n, const int *__restrict__ row_ptr,
                                                        const int *__restrict__ col_idx, int blk_h,
                                                        int *__restrict__ edge_to_row,
                                                        int *__restrict__ edge_to_col,
                                                        int *__restrict__ uniq_count,
                                                        int *__restrict__ tmp_cols,
                                                        int *__restrict__ big_list, int *big_count)
{
    __shared__ int keys[SMALL_CAP];
    __shared__ int uniq[SMALL_CAP];
    __shared__ int rp[65];  // row_ptr of the window's rows (blk_h <= 64)
    __shared__ int scan_tmp[256 / 64 + 1];
    const int tid = threadIdx.x;
    const int w = blockIdx.x;
    const int r0 = w * blk_h;
    const int r1 = min(n, r0 + blk_h);
    const int rows = r1 - r0;
    if (tid <= rows) rp[tid] = row_ptr[r0 + tid];
    __syncthreads();
    const int e0 = rp[0], e1 = rp[rows];
    const int cnt = e1 - e0;

    // 1. row of every edge of the window
    for (int e = e0 + tid; e < e1; e += 256) {
        int lo = 0, hi = rows;  // last k with rp[k] <= e
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (rp[mid] <= e) lo = mid; else hi = mid;
        }
        edge_to_row[e] = r0 + lo;
    }
    if (cnt == 0) {
        if (tid == 0) uniq_count[w] = 0;
        return;
    }
    if (cnt > SMALL_CAP) {
        if (tid == 0) big_list[atomicAdd(big_count, 1)] = w;
        return;
    }

    // 2. sort the column ids (padded to a power of two with the largest int)
    int P = 1;
    while (P < cnt) P <<= 1;
    for (int t = tid; t < P; t += 256) keys[t] = t < cnt ? col_idx[e0 + t] : 0x7fffffff;
    __syncthreads();
    for (int k = 2; k <= P; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int t = tid; t < (P >> 1); t += 256) {
                const int i = 2 * t - (t & (j - 1));
                const int l = i + j;
                const bool up = (i & k) == 0;
                const int a = keys[i], b = keys[l];
                if ((a > b) == up) { keys[i] = b; keys[l] = a; }
            }
            __syncthreads();
        }
    }

    // 3. strict de-duplication: each thread owns a run of consecutive sorted keys
    const int per = (P + 255) / 256;
    const int b0 = tid * per, b1 = min(cnt, b0 + per);
    int mine = 0;
    for (int t = b0; t < b1; ++t) mine += (t == 0 || keys[t] != keys[t - 1]) ? 1 : 0;
    int n_uniq;
    int pos = block_exclusive_scan<256>(mine, scan_tmp, &n_uniq);
    for (int t = b0; t < b1; ++t)
        if (t == 0 || keys[t] != keys[t - 1]) uniq[pos++] = keys[t];
    __syncthreads();

    // 4. outputs: unique list at the window's edge offset, rank of every edge
    for (int t = tid; t < n_uniq; t += 256) tmp_cols[e0 + t] = uniq[t];
    for (int t = tid; t < cnt; t += 256) {
        const int c = col_idx[e0 + t];
        int lo = 0, hi = n_uniq;  // first index with uniq[idx] >= c
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (uniq[mid] < c) lo = mid + 1; else hi = mid;
        }
        edge_to_col[e0 + t] = lo;
    }
    if (tid == 0) uniq_count[w] = n_uniq;
}

__global__ __launch_bounds__(BIG_THREADS) void win_big_kernel(int n, const int *__restrict__ row_ptr,
                                                              const int *__restrict__ col_idx, int blk_h,
                                                              int *__restrict__ edge_to_col,
                                                              int *__restrict__ uniq_count,
                                                              int *__restrict__ tmp_cols,
                                                              const int *__restrict__ big_list,
                                                              const int *big_count, uint32_t *bitmaps,
                                                              int words)
{
    __shared__ int scan_tmp[BIG_THREADS / 64 + 1];
    __shared__ int carry_s;
    const int tid = threadIdx.x;
    uint32_t *bits = bitmaps + static_cast<size_t>(blockIdx.x) * 2 * words;
    int *prefix = reinterpret_cast<int *>(bits + words);
    const int nb = *big_count;
    for (int i = blockIdx.x; i < nb; i += gridDim.x) {
        const int w = big_list[i];
        const int r0 = w * blk_h;
        const int r1 = min(n, r0 + blk_h);
        const int e0 = row_ptr[r0], e1 = row_ptr[r1];
        for (int t = tid; t < words; t += BIG_THREADS) bits[t] = 0u;
        __syncthreads();
        for (int e = e0 + tid; e < e1; e += BIG_THREADS) {
            const int c = col_idx[e];
            atomicOr(&bits[c >> 5], 1u << (c & 31));
        }
        if (tid == 0) carry_s = 0;
        __threadfence();  // the atomics above are performed in L2: drop stale L1 lines of the bitmap
        __syncthreads();
        // exclusive prefix of the per-word popcounts, BIG_THREADS words per round
        for (int base = 0; base < words; base += BIG_THREADS) {
            const int t = base + tid;
            const int pc = t < words ? __popc(bits[t]) : 0;
            int round_total;
            const int ex = block_exclusive_scan<BIG_THREADS>(pc, scan_tmp, &round_total);
            const int carry = carry_s;
            if (t < words) prefix[t] = carry + ex;
            __syncthreads();
            if (tid == 0) carry_s = carry + round_total;
            __syncthreads();
        }
        const int n_uniq = carry_s;
        for (int e = e0 + tid; e < e1; e += BIG_THREADS) {
            const int c = col_idx[e];
            const uint32_t below = bits[c >> 5] & ((1u << (c & 31)) - 1u);
            edge_to_col[e] = prefix[c >> 5] + __popc(below);
        }
        for (int t = tid; t < words; t += BIG_THREADS) {
            uint32_t b = bits[t];
            int k = prefix[t];
            while (b) {
                const int bit = __ffs(b) - 1;
                tmp_cols[e0 + k++] = t * 32 + bit;
                b &= b - 1;
            }
        }
        if (tid == 0) uniq_count[w] = n_uniq;
        __syncthreads();  // bitmap slot is reused by the next queued window
    }
}

// Single workgroup: exclusive scan of the per-window unique counts.
__global__ __launch_bounds__(1024) void win_scan_kernel(int n_windows, int blk_w,
                                                        const int *__restrict__ uniq_count,
                                                        int *__restrict__ win_col_ptr,
                                                        int *__restrict__ block_partition,
                                                        int64_t *__restrict__ summary)
{
    __shared__ int scan_tmp[1024 / 64 + 1];
    __shared__ long long blocks_s[16];
    const int tid = threadIdx.x;
    int carry = 0;
    long long my_blocks = 0;
    for (int base = 0; base < n_windows; base += 1024) {
        const int t = base + tid;
        const int u = t < n_windows ? uniq_count[t] : 0;
        int round_total;
        const int ex = block_exclusive_scan<1024>(u, scan_tmp, &round_total);
        if (t < n_windows) {
            win_col_ptr[t] = carry + ex;
            const int blocks = (u + blk_w - 1) / blk_w;
            block_partition[t] = blocks;
            my_blocks += blocks;
        }
        carry += round_total;
    }
    // sum of blocks over the workgroup
    long long v = my_blocks;
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    __syncthreads();
    if ((tid & 63) == 0) blocks_s[tid >> 6] = v;
    __syncthreads();
    if (tid == 0) {
        long long total_blocks = 0;
        for (int k = 0; k < 16; ++k) total_blocks += blocks_s[k];
        win_col_ptr[n_windows] = carry;
        summary[0] = carry;
        summary[1] = total_blocks;
    }
}

__global__ __launch_bounds__(256) void win_pack_kernel(int n, const int *__restrict__ row_ptr, int blk_h,
                                                       const int *__restrict__ win_col_ptr,
                                                       const int *__restrict__ tmp_cols,
                                                       int *__restrict__ win_cols)
{
    const int w = blockIdx.x;
    const int src = row_ptr[min(n, w * blk_h)];
    const int dst = win_col_ptr[w];
    const int cnt = win_col_ptr[w + 1] - dst;
    for (int t = threadIdx.x; t < cnt; t += 256) win_cols[dst + t] = tmp_cols[src + t];
}

int32_t launch_build_windows(const ftc_csr &g, ftc_windows &w, void *ws, size_t ws_bytes, hipStream_t s)
{
    (void)ws_bytes;
    const WinWorkspace k = carve(ws, g.n, g.nnz, w.n_windows);
    if (w.n_windows == 0) {  // n == 0: only the empty prefix and the summary are written
        hipLaunchKernelGGL(win_scan_kernel, dim3(1), dim3(1024), 0, s, 0, w.blk_w, k.uniq_count, w.win_col_ptr,
                           w.block_partition, w.summary);
        return launch_status("build_windows scan");
    }
    hipLaunchKernelGGL(win_clear_kernel, dim3(1), dim3(1), 0, s, k.big_count);
    hipLaunchKernelGGL(win_small_kernel, dim3(w.n_windows), dim3(256), 0, s, g.n, g.row_ptr, g.col_idx,
                       w.blk_h, w.edge_to_row, w.edge_to_col, k.uniq_count, k.tmp_cols, k.big_list,
                       k.big_count);
    int32_t st = launch_status("build_windows small");
    if (st != FTC_OK) return st;
    hipLaunchKernelGGL(win_big_kernel, dim3(k.slots), dim3(BIG_THREADS), 0, s, g.n, g.row_ptr, g.col_idx,
                       w.blk_h, w.edge_to_col, k.uniq_count, k.tmp_cols, k.big_list, k.big_count, k.bitmaps,
                       static_cast<int>(k.words));
    st = launch_status("build_windows big");
    if (st != FTC_OK) return st;
    hipLaunchKernelGGL(win_scan_kernel, dim3(1), dim3(1024), 0, s, w.n_windows, w.blk_w, k.uniq_count,
                       w.win_col_ptr, w.block_partition, w.summary);
    st = launch_status("build_windows scan");
    if (st != FTC_OK) return st;
    hipLaunchKernelGGL(win_pack_kernel, dim3(w.n_windows), dim3(256), 0, s, g.n, g.row_ptr, w.blk_h,
                       w.win_col_ptr, k.tmp_cols, w.win_cols);
    return launch_status("build_windows pack");
}

}  // namespace ftc
