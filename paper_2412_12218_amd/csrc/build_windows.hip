// Sparse graph transformation (Section V.A) on the GPU.
//
// Every row window is independent (the paper parallelises the same step over CPU threads), so
// one wave or one workgroup condenses one window; which one depends on the window's edge count:
//   1. up to WAVE_CAP edges (almost every window): one wave sorts the column ids in registers
//      with a bitonic network (lane shuffles, no barriers), de-duplicates with a flag scan and
//      finds every edge's rank by binary search in the unique list parked in LDS;
//   2. larger windows (hub rows of power-law graphs) are queued and condensed by a 1024-thread
//      workgroup with a bitmap of 2^20 column ids held in LDS (128 KiB of the CU's 160 KiB):
//      set bits, prefix sums of popcounts per group of 8 words, rank = group prefix + popcounts
//      up to the column's bit.  Graphs with more than 2^20 nodes take several passes over
//      successive column ranges; a pass whose range holds none of the window's columns costs
//      only the scan of the window's edges.
// Both also write edge_to_row for their window's edges.
// The unique lists are first written at the window's edge offset of a temporary array (a
// window never has more distinct columns than edges), then a scan over the windows gives
// win_col_ptr / block_partition / summary and a last kernel packs the lists into win_cols.
#include "ftc_common.hpp"

namespace ftc {

constexpr int WAVE_CAP = 1024;       // edges per window sorted by a single wave in registers
constexpr int BIG_THREADS = 1024;    // workgroup of the bitmap kernel
constexpr int RANGE_LOG2 = 20;       // column ids per bitmap pass
constexpr int RANGE_WORDS = (1 << RANGE_LOG2) / 32;
constexpr int GROUP_WORDS = 8;       // bitmap words per prefix entry
constexpr int N_GROUPS = RANGE_WORDS / GROUP_WORDS;
constexpr int BIG_GRID = 256;        // persistent workgroups, one per CU
constexpr int TOUCH_WORDS = RANGE_WORDS / 32;  // one bit per bitmap word: which words hold any bit
constexpr size_t BIG_LDS_BYTES = sizeof(uint32_t) * (RANGE_WORDS + N_GROUPS + TOUCH_WORDS);
static_assert(TOUCH_WORDS == BIG_THREADS, "one coarse word per thread");

struct WinWorkspace {
    int *uniq_count;  // [n_windows]
    int *big_list;    // [n_windows]
    int *big_count;   // [2]
    int *tmp_cols;    // [nnz]
    size_t total;
};

static WinWorkspace carve(void *ws, int n, int nnz, int n_windows)
{
    (void)n;
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
    w.big_count = reinterpret_cast<int *>(take(2 * sizeof(int)));  // queue length, next entry to hand out
    w.tmp_cols = reinterpret_cast<int *>(take(sizeof(int) * static_cast<size_t>(nnz)));
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

__global__ void win_clear_kernel(int *counters) { counters[0] = 0; counters[1] = 0; }

// ---- windows of at most WAVE_CAP edges: one wave, keys in registers --------------------------------
// Element i of the padded key array lives in lane i / E, register i % E.
template <int E>
__device__ __forceinline__ void wave_bitonic_sort(int (&key)[E], int lane)
{
    constexpr int P = 64 * E;
#pragma unroll
    for (int kk = 2; kk <= P; kk <<= 1) {
#pragma unroll
        for (int j = kk >> 1; j > 0; j >>= 1) {
            if (j >= E) {  // partner element sits in another lane, same register
                const int lm = j / E;
                const bool lower = (lane & lm) == 0;
#pragma unroll
                for (int k = 0; k < E; ++k) {
                    const int other = __shfl_xor(key[k], lm, 64);
                    const bool up = ((lane * E + k) & kk) == 0;
                    const int mn = min(key[k], other), mx = max(key[k], other);
                    key[k] = (lower == up) ? mn : mx;
                }
            } else {       // partner element sits in the same lane
#pragma unroll
                for (int k = 0; k < E; ++k) {
                    if ((k & j) == 0) {
                        const bool up = ((lane * E + k) & kk) == 0;
                        const int a = key[k], b = key[k | j];
                        const int mn = min(a, b), mx = max(a, b);
                        key[k] = up ? mn : mx;
                        key[k | j] = up ? mx : mn;
                    }
                }
            }
        }
    }
}

template <int E>
__device__ __forceinline__ void condense_window_wave(int w, int r0, int rows, const int *rp, int cnt,
                                                     const int *__restrict__ col_idx,
                                                     int *__restrict__ edge_to_row,
                                                     int *__restrict__ edge_to_col,
                                                     int *__restrict__ uniq_count, int *__restrict__ tmp_cols,
                                                     int *uniq_lds)
{
    const int lane = threadIdx.x;
    const int e0 = rp[0];
    int key[E], orig[E];
#pragma unroll
    for (int k = 0; k < E; ++k) {
        const int i = lane * E + k;
        orig[k] = i < cnt ? col_idx[e0 + i] : 0x7fffffff;
        key[k] = orig[k];
    }
    wave_bitonic_sort<E>(key, lane);
    // strict de-duplication of the sorted sequence
    const int prev_last = __shfl_up(key[E - 1], 1, 64);
    bool flag[E];
    int mine = 0;
#pragma unroll
    for (int k = 0; k < E; ++k) {
        const int i = lane * E + k;
        const int before = k == 0 ? prev_last : key[k - 1];
        flag[k] = i < cnt && (i == 0 || key[k] != before);
        mine += flag[k] ? 1 : 0;
    }
    int incl = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int up = __shfl_up(incl, d, 64);
        if (lane >= d) incl += up;
    }
    const int n_uniq = __shfl(incl, 63, 64);
    int pos = incl - mine;
#pragma unroll
    for (int k = 0; k < E; ++k) {
        if (flag[k]) {
            uniq_lds[pos] = key[k];
            tmp_cols[e0 + pos] = key[k];
            ++pos;
        }
    }
    __syncthreads();  // single-wave workgroup: makes the unique list visible to all lanes
#pragma unroll
    for (int k = 0; k < E; ++k) {
        const int i = lane * E + k;
        if (i < cnt) {
            int lo = 0, hi = n_uniq;  // first index with uniq[idx] >= column
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (uniq_lds[mid] < orig[k]) lo = mid + 1; else hi = mid;
            }
            edge_to_col[e0 + i] = lo;
            int a = 0, b = rows;  // last row index with rp[a] <= edge
            while (b - a > 1) {
                const int mid = (a + b) >> 1;
                if (rp[mid] <= e0 + i) a = mid; else b = mid;
            }
            edge_to_row[e0 + i] = r0 + a;
        }
    }
    if (lane == 0) uniq_count[w] = n_uniq;
}

__global__ __launch_bounds__(64) void win_wave_kernel(int n, const int *__restrict__ row_ptr,
                                                      const int *__restrict__ col_idx, int blk_h,
                                                      int *__restrict__ edge_to_row,
                                                      int *__restrict__ edge_to_col,
                                                      int *__restrict__ uniq_count, int *__restrict__ tmp_cols,
                                                      int *__restrict__ big_list, int *big_count)
{
    __shared__ int uniq_lds[WAVE_CAP];
    __shared__ int rp[65];
    const int w = blockIdx.x;
    const int r0 = w * blk_h;
    const int rows = min(n, r0 + blk_h) - r0;
    for (int t = threadIdx.x; t <= rows; t += 64) rp[t] = row_ptr[r0 + t];
    __syncthreads();
    const int cnt = rp[rows] - rp[0];
    if (cnt > WAVE_CAP) {  // queued for the bitmap kernel
        if (threadIdx.x == 0) big_list[atomicAdd(big_count, 1)] = w;
        return;
    }
    if (cnt == 0) {
        if (threadIdx.x == 0) uniq_count[w] = 0;
        return;
    }
#define FTC_WAVE(E) condense_window_wave<E>(w, r0, rows, rp, cnt, col_idx, edge_to_row, edge_to_col, uniq_count, tmp_cols, uniq_lds)
    if (cnt <= 64) FTC_WAVE(1);
    else if (cnt <= 128) FTC_WAVE(2);
    else if (cnt <= 256) FTC_WAVE(4);
    else if (cnt <= 512) FTC_WAVE(8);
    else FTC_WAVE(16);
#undef FTC_WAVE
}


// ---- queued windows: bitmap of 2^20 column ids in LDS ----------------------------------------------
__global__ __launch_bounds__(BIG_THREADS) void win_bitmap_kernel(int n, const int *__restrict__ row_ptr,
                                                                 const int *__restrict__ col_idx, int blk_h,
                                                                 int *__restrict__ edge_to_row,
                                                                 int *__restrict__ edge_to_col,
                                                                 int *__restrict__ uniq_count,
                                                                 int *__restrict__ tmp_cols,
                                                                 const int *__restrict__ big_list,
                                                                 int *big_count)
{
    extern __shared__ uint32_t lds[];
    uint32_t *bits = lds;                                      // [RANGE_WORDS], all zero between passes
    int *grp = reinterpret_cast<int *>(lds + RANGE_WORDS);     // [N_GROUPS] popcount sums, then prefixes
    uint32_t *touched = lds + RANGE_WORDS + N_GROUPS;          // [TOUCH_WORDS] non-empty bitmap words
    __shared__ int scan_tmp[BIG_THREADS / 64 + 1];
    __shared__ int rp[65];
    __shared__ int any_s;
    __shared__ int next_s;
    const int tid = threadIdx.x;
    for (int t = tid; t < RANGE_WORDS; t += BIG_THREADS) bits[t] = 0u;
    for (int t = tid; t < N_GROUPS; t += BIG_THREADS) grp[t] = 0;
    touched[tid] = 0u;
    const int nb = *big_count;
    const int n_pass = static_cast<int>((static_cast<int64_t>(n) + (1 << RANGE_LOG2) - 1) >> RANGE_LOG2);
    // Workgroups pull queued windows one at a time (window sizes differ by two orders of magnitude);
    // every workgroup leaves as soon as the queue is empty.
    for (;;) {
        __syncthreads();  // previous window (or the initial clearing) is done with the LDS
        if (tid == 0) next_s = atomicAdd(&big_count[1], 1);
        __syncthreads();
        const int i = next_s;
        if (i >= nb) break;
        const int w = big_list[i];
        const int r0 = w * blk_h;
        const int rows = min(n, r0 + blk_h) - r0;
        if (tid <= rows) rp[tid] = row_ptr[r0 + tid];
        __syncthreads();
        const int e0 = rp[0], e1 = rp[rows];
        // The window's column ids are handled in chunks of KREG * 1024 edges held in registers
        // (KREG independent loads in flight per thread).  A window that fits one chunk reads its
        // column ids from memory once; longer ones re-read them in the ranking phase.
        constexpr int KREG = 8;
        constexpr int CHUNK = KREG * BIG_THREADS;
        const int n_chunks = (e1 - e0 + CHUNK - 1) / CHUNK;
        int creg[KREG];
        auto load_chunk = [&](int ch) {
#pragma unroll
            for (int q = 0; q < KREG; ++q) {
                const int e = e0 + ch * CHUNK + tid + q * BIG_THREADS;
                creg[q] = e < e1 ? col_idx[e] : -1;
            }
        };
        if (n_chunks == 1) load_chunk(0);
        const bool track = n_chunks <= 2;  // longer windows touch most words: visit them all instead
        for (int e = e0 + tid; e < e1; e += BIG_THREADS) {
            int a = 0, b = rows;  // last row index with rp[a] <= e
            while (b - a > 1) {
                const int mid = (a + b) >> 1;
                if (rp[mid] <= e) a = mid; else b = mid;
            }
            edge_to_row[e] = r0 + a;
        }
        int base_rank = 0;
        for (int pass = 0; pass < n_pass; ++pass) {
            const int lo = pass << RANGE_LOG2;
            if (tid == 0) any_s = 0;
            __syncthreads();
            bool any = false;
            for (int ch = 0; ch < n_chunks; ++ch) {
                if (n_chunks > 1) load_chunk(ch);
#pragma unroll
                for (int q = 0; q < KREG; ++q) {
                    const unsigned c = static_cast<unsigned>(creg[q] - lo);
                    if (creg[q] >= 0 && c < (1u << RANGE_LOG2)) {
                        atomicOr(&bits[c >> 5], 1u << (c & 31));
                        if (track) atomicOr(&touched[c >> 10], 1u << ((c >> 5) & 31));
                        any = true;
                    }
                }
            }
            if (any) any_s = 1;
            if (!track) touched[tid] = 0xffffffffu;
            __syncthreads();
            if (!any_s) {  // uniform: none of the window's columns lies in this range
                touched[tid] = 0u;
                continue;
            }
            // popcount sums per group of GROUP_WORDS words; only words that hold a bit are visited
            // (thread t owns bitmap words 32 t .. 32 t + 31 through its coarse word)
            const uint32_t my_touched = touched[tid];
            for (uint32_t m = my_touched; m; m &= m - 1) {
                const int t = tid * 32 + (__ffs(m) - 1);
                const int pc = __popc(bits[t]);
                if (pc) atomicAdd(&grp[t / GROUP_WORDS], pc);
            }
            __syncthreads();
            // exclusive prefix over the groups: every thread owns N_GROUPS / BIG_THREADS consecutive groups
            constexpr int PER = N_GROUPS / BIG_THREADS;
            int sums[PER];
            int mine = 0;
#pragma unroll
            for (int q = 0; q < PER; ++q) { sums[q] = grp[tid * PER + q]; mine += sums[q]; }
            int pass_total;
            int run = block_exclusive_scan<BIG_THREADS>(mine, scan_tmp, &pass_total);
#pragma unroll
            for (int q = 0; q < PER; ++q) { grp[tid * PER + q] = run; run += sums[q]; }
            __syncthreads();
            // rank of every edge whose column lies in this range
            auto rank_of = [&](unsigned c) {
                const int word = c >> 5, g0 = word / GROUP_WORDS;
                int r = grp[g0];
                for (int t = g0 * GROUP_WORDS; t < word; ++t) r += __popc(bits[t]);
                return base_rank + r + __popc(bits[word] & ((1u << (c & 31)) - 1u));
            };
            for (int ch = 0; ch < n_chunks; ++ch) {
                if (n_chunks > 1) load_chunk(ch);
#pragma unroll
                for (int q = 0; q < KREG; ++q) {
                    const unsigned c = static_cast<unsigned>(creg[q] - lo);
                    if (creg[q] >= 0 && c < (1u << RANGE_LOG2))
                        edge_to_col[e0 + ch * CHUNK + tid + q * BIG_THREADS] = rank_of(c);
                }
            }
            // the unique columns of this range, ascending
            for (uint32_t m = my_touched; m; m &= m - 1) {
                const int t = tid * 32 + (__ffs(m) - 1);
                uint32_t b = bits[t];
                if (!b) continue;
                const int g0 = t / GROUP_WORDS;
                int k = base_rank + grp[g0];
                for (int q = g0 * GROUP_WORDS; q < t; ++q) k += __popc(bits[q]);
                while (b) {
                    const int bit = __ffs(b) - 1;
                    tmp_cols[e0 + k++] = lo + t * 32 + bit;
                    b &= b - 1;
                }
            }
            __syncthreads();
            // leave the LDS all zero for the next pass / window
            for (uint32_t m = my_touched; m; m &= m - 1) bits[tid * 32 + (__ffs(m) - 1)] = 0u;
            for (int t = tid; t < N_GROUPS; t += BIG_THREADS) grp[t] = 0;
            touched[tid] = 0u;
            base_rank += pass_total;
        }
        if (tid == 0) uniq_count[w] = base_rank;
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

// Packs the unique lists: one thread per slot of the temporary array.  Slot e belongs to the window
// of edge e (edge_to_row); it holds a list entry when its offset inside the window is below the
// window's unique count.
__global__ __launch_bounds__(256) void win_pack_kernel(int nnz, const int *__restrict__ row_ptr, int blk_h,
                                                       const int *__restrict__ edge_to_row,
                                                       const int *__restrict__ win_col_ptr,
                                                       const int *__restrict__ tmp_cols,
                                                       int *__restrict__ win_cols)
{
    const int64_t e = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (e >= nnz) return;
    const int w = edge_to_row[e] / blk_h;
    const int k = static_cast<int>(e) - row_ptr[w * blk_h];
    const int dst = win_col_ptr[w];
    if (k < win_col_ptr[w + 1] - dst) win_cols[dst + k] = tmp_cols[e];
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
    hipLaunchKernelGGL(win_wave_kernel, dim3(w.n_windows), dim3(64), 0, s, g.n, g.row_ptr, g.col_idx, w.blk_h,
                       w.edge_to_row, w.edge_to_col, k.uniq_count, k.tmp_cols, k.big_list, k.big_count);
    int32_t st = launch_status("build_windows wave");
    if (st != FTC_OK) return st;
    // 144 KiB of dynamic LDS: above the default limit, so the attribute is raised first
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(win_bitmap_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize,
                            static_cast<int>(BIG_LDS_BYTES)) != hipSuccess) {
        (void)hipGetLastError();
        set_error("build_windows: cannot reserve %zu bytes of LDS", BIG_LDS_BYTES);
        return FTC_EHIP;
    }
    hipLaunchKernelGGL(win_bitmap_kernel, dim3(BIG_GRID), dim3(BIG_THREADS), BIG_LDS_BYTES, s, g.n, g.row_ptr,
                       g.col_idx, w.blk_h, w.edge_to_row, w.edge_to_col, k.uniq_count, k.tmp_cols, k.big_list,
                       k.big_count);
    st = launch_status("build_windows bitmap");
    if (st != FTC_OK) return st;
    hipLaunchKernelGGL(win_scan_kernel, dim3(1), dim3(1024), 0, s, w.n_windows, w.blk_w, k.uniq_count,
                       w.win_col_ptr, w.block_partition, w.summary);
    st = launch_status("build_windows scan");
    if (st != FTC_OK) return st;
    if (g.nnz == 0) return FTC_OK;
    hipLaunchKernelGGL(win_pack_kernel, dim3((g.nnz + 255) / 256), dim3(256), 0, s, g.nnz, g.row_ptr, w.blk_h,
                       w.edge_to_row, w.win_col_ptr, k.tmp_cols, w.win_cols);
    return launch_status("build_windows pack");
}

}  // namespace ftc
