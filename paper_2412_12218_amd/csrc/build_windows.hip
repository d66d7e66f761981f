// Sparse graph transformation (Section V.A) on the GPU.
//
// Every row window is independent (the paper parallelises the same step over CPU threads).  How
// a window is condensed depends on its edge count, because power-law graphs have windows of a
// few edges next to windows of 10^5:
//   1. up to WAVE_CAP edges: one wave sorts the column ids in registers with a bitonic network
//      (lane shuffles, no barriers), de-duplicates with a flag scan and finds every edge's rank by
//      binary search in the unique list parked in LDS;
//   2. up to MID_CAP edges, in three size classes: one, two or four waves per window with a two-level
//      bitmap in LDS (a coarse bitmap names the 32-column words the window touches, the fine bitmap
//      holds one word per touched word): set bits, prefix sums of the popcounts, rank = prefix of the
//      word + bits below the column's own.  The waves keep their column ids in registers; a CU works
//      on as many windows at once as their bitmaps fit into its LDS;
//   3. above MID_CAP edges on graphs of up to DIRECT_MAX_RANGES ranges of 2^20 columns: one workgroup
//      of 1024 threads with the whole bitmap of a range in LDS (no coarse level); windows of 10^5
//      edges are queued in parts, each of which builds the bitmap and ranks its share of the edges;
//   3b. on larger graphs instead: the two-level bitmap with sixteen waves up to B4_CAP edges, a
//      workgroup of 1024 threads up to the hub threshold, and hub windows (more edges than the
//      threshold, at most HUB_SLOTS_MAX of them by the choice of the threshold) edge-parallel over
//      the whole GPU with one bitmap of n bits per hub in global memory: set bits (atomics), one
//      workgroup per hub turns popcounts into prefixes, then every edge reads its rank.
// All of them also write edge_to_row for their window's edges.
// The unique lists are first written at the window's edge offset of a temporary array (a
// window never has more distinct columns than edges), then a scan over the windows (chunk sums, then
// chunk scans) gives win_col_ptr / block_partition / summary and a last kernel packs the lists into
// win_cols.  The kernels of the size classes are independent: with side streams from the caller they
// run side by side.
#include "ftc_common.hpp"


namespace ftc {

constexpr int WAVE_CAP = 256;       // edges per window sorted by a single wave in registers
constexpr int B1_CAP = 1024;        // edges per window of the three size classes of the wave-level bitmap kernel
constexpr int B2_CAP = 2048;
constexpr int MID_CAP = 4096;
constexpr int B4_CAP = 16384;       // ... and of the same kernel with sixteen waves per window
constexpr int DIRECT_MAX_RANGES = 4; // graphs of up to this many 2^20-column ranges: every window above MID_CAP edges takes
                                     // the direct-bitmap kernel (a workgroup per window, one bit per column of a range)
constexpr int HUB_MIN_EDGES = 16384;
constexpr int HUB_SLOTS_MAX = 1024; // hub windows handled at once (one thread each in the planning kernel)
constexpr int HUB_CHUNK = 4096;     // edges per work item of the edge-parallel hub kernels
constexpr int HUB_GROUP = 8;        // bitmap words per stored prefix (one 32-byte load)
constexpr int HUB_GRID = 2048;      // workgroups of the edge-parallel hub kernels (grid-stride over chunks)

// Parts a window of `cnt` edges is queued in for the direct kernel: every part builds the window's whole bitmap
// and ranks DIRECT_PART_EDGES of its edges or fewer, so that the few windows of 10^5 edges of a power-law graph do not
// keep one workgroup busy long after every other one has finished (one workgroup took 0.31 ms for the R-MAT
// benchmark graph's largest window, 256 000 edges; building the bitmap is the cheaper half of the work, 0.18 ns per
// edge against 0.40 ns for ranking and writing).  cnt / DIRECT_PART_EDGES + 1 <= cnt / (MID_CAP + 1) above
// DIRECT_SPLIT_MIN: the queue's capacity of nnz / (MID_CAP + 1) + 1 entries holds.
constexpr int DIRECT_SPLIT_MIN = 32768, DIRECT_PART_EDGES = 16384, DIRECT_PARTS_MAX = 16;
__host__ __device__ inline int direct_parts(int cnt)
{
    if (cnt <= DIRECT_SPLIT_MIN) return 1;
    const int p = (cnt + DIRECT_PART_EDGES - 1) / DIRECT_PART_EDGES;
    return p < DIRECT_PARTS_MAX ? p : DIRECT_PARTS_MAX;
}

enum { C_B1 = 0, C_B2 = 1, C_B3 = 2, C_B4 = 3, C_LARGE = 4, C_HUB = 5, C_DIRECT = 6, C_CHUNKS = 7, C_LARGE_NEXT = 8,
       C_DIRECT_NEXT = 9, C_WORDS = 16 };

// A window is a hub when it has more edges than this.  The three terms keep (a) small windows in
// LDS, (b) a hub's bitmap (n / 8 bytes) below four bytes per edge of the hub, (c) the number of
// hubs at or below HUB_SLOTS_MAX.
static int hub_threshold(int n, int nnz)
{
    int t = HUB_MIN_EDGES;
    if ((n + 31) / 32 > t) t = (n + 31) / 32;
    const int by_slots = static_cast<int>((static_cast<int64_t>(nnz) + HUB_SLOTS_MAX - 1) / HUB_SLOTS_MAX);
    return by_slots > t ? by_slots : t;
}
static int hub_slots(int n, int nnz)
{
    const int s = nnz / hub_threshold(n, nnz);  // more than this many windows above the threshold cannot exist
    return s < 1 ? 1 : s;
}
static int hub_words_per_slot(int n) { return ((n + 31) / 32 + HUB_GROUP - 1) / HUB_GROUP * HUB_GROUP; }

constexpr int PACK_PER_WAVE = 1024;  // entries of win_cols that one wave of the pack kernel copies
constexpr int SCAN_CHUNK = 1024;     // windows per workgroup of the two-level scan
constexpr int SCAN_CHUNKS_MAX = 4096;  // beyond that many chunks the single-workgroup scan runs

struct WinWorkspace {
    int *uniq_count;      // [n_windows]
    int4 *list_b[4];      // [cap_b[i]]   windows of WAVE_CAP+1 .. B1_CAP, .. B2_CAP, .. MID_CAP, .. B4_CAP edges:
                          //              {window, first edge, edges, -}
    int4 *list_direct;    // [cap_direct] windows above MID_CAP edges on graphs of few column ranges (then list_b[3],
                          //              list_large and list_hub stay empty): {window, first edge, edges, part | parts << 8}
    int *list_large;      // [cap_large]  windows of B4_CAP+1 .. threshold edges
    int *list_hub;        // [slots]
    int *counters;        // [C_WORDS]
    int *hub_chunk_ptr;   // [slots + 1]  first work item of every hub
    int *chunk_table;     // [nnz / HUB_CHUNK + slots + 1]  hub slot of every work item
    uint32_t *hub_bits;   // [slots * words_per_slot]
    int *hub_grp;         // [slots * words_per_slot / HUB_GROUP]
    int *tmp_cols;        // [nnz]
    int *pack_win;        // [nnz / PACK_PER_WAVE + 2]  window of every PACK_PER_WAVE-th entry of win_cols
    int *chunk_uniq;      // [ceil(n_windows / SCAN_CHUNK)]  unique columns of every chunk of windows
    long long *chunk_blocks;  // the same for the tile counts
    int cap_b[4], cap_direct, cap_large, slots, wps;
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
    const int lower[4] = {WAVE_CAP, B1_CAP, B2_CAP, MID_CAP};
    for (int i = 0; i < 4; ++i) w.cap_b[i] = nnz / (lower[i] + 1) + 1 < n_windows ? nnz / (lower[i] + 1) + 1 : n_windows;
    {
        const int64_t by_parts = static_cast<int64_t>(n_windows) * DIRECT_PARTS_MAX;
        w.cap_direct = nnz / (MID_CAP + 1) + 1 < by_parts ? nnz / (MID_CAP + 1) + 1 : static_cast<int>(by_parts);
    }
    w.cap_large = nnz / (B4_CAP + 1) + 1 < n_windows ? nnz / (B4_CAP + 1) + 1 : n_windows;
    w.slots = hub_slots(n, nnz);
    w.wps = hub_words_per_slot(n);
    w.uniq_count = reinterpret_cast<int *>(take(sizeof(int) * static_cast<size_t>(n_windows)));
    for (int i = 0; i < 4; ++i) w.list_b[i] = reinterpret_cast<int4 *>(take(sizeof(int4) * static_cast<size_t>(w.cap_b[i])));
    w.list_direct = reinterpret_cast<int4 *>(take(sizeof(int4) * static_cast<size_t>(w.cap_direct)));
    w.list_large = reinterpret_cast<int *>(take(sizeof(int) * static_cast<size_t>(w.cap_large)));
    w.list_hub = reinterpret_cast<int *>(take(sizeof(int) * static_cast<size_t>(w.slots)));
    w.counters = reinterpret_cast<int *>(take(sizeof(int) * C_WORDS));
    w.hub_chunk_ptr = reinterpret_cast<int *>(take(sizeof(int) * static_cast<size_t>(w.slots + 1)));
    w.chunk_table = reinterpret_cast<int *>(take(sizeof(int) * static_cast<size_t>(nnz / HUB_CHUNK + w.slots + 1)));
    w.hub_bits = reinterpret_cast<uint32_t *>(take(sizeof(uint32_t) * static_cast<size_t>(w.slots) * w.wps));
    w.hub_grp = reinterpret_cast<int *>(take(sizeof(int) * static_cast<size_t>(w.slots) * (w.wps / HUB_GROUP)));
    w.tmp_cols = reinterpret_cast<int *>(take(sizeof(int) * static_cast<size_t>(nnz)));
    w.pack_win = reinterpret_cast<int *>(take(sizeof(int) * (static_cast<size_t>(nnz) / PACK_PER_WAVE + 2)));
    {
        const size_t chunks = (static_cast<size_t>(n_windows) + SCAN_CHUNK - 1) / SCAN_CHUNK;
        w.chunk_uniq = reinterpret_cast<int *>(take(sizeof(int) * chunks));
        w.chunk_blocks = reinterpret_cast<long long *>(take(sizeof(long long) * chunks));
    }
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

__global__ void win_clear_kernel(int *counters)
{
    if (threadIdx.x < C_WORDS) counters[threadIdx.x] = 0;
}

// Exclusive scan of one int per thread with a single barrier; `wave_tot` holds NT / 64 ints of LDS
// and must not be written again before every thread has passed another barrier.
template <int NT>
__device__ __forceinline__ int block_scan_one_barrier(int v, int *wave_tot, int *total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int incl = wave_inclusive_scan(v);
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    int off = 0, tot = 0;
#pragma unroll
    for (int k = 0; k < NT / 64; ++k) {
        const int t = wave_tot[k];
        off += k < wave ? t : 0;
        tot += t;
    }
    *total = tot;
    return off + incl - v;
}

// Index of the row that holds edge e: last a in [0, rows) with rp[a] <= e.
__device__ __forceinline__ int row_of_edge(const int *rp, int rows, int e)
{
    int a = 0, b = rows;
    while (b - a > 1) {
        const int mid = (a + b) >> 1;
        if (rp[mid] <= e) a = mid; else b = mid;
    }
    return a;
}

// ---- classification: queues of the windows that are too large for a single wave -------------------
// One thread per window.  Queue positions come from one atomic per size class and workgroup (the
// entries of a workgroup are numbered in LDS first): thousands of atomics on one address would
// serialise.
__global__ __launch_bounds__(1024) void win_classify_kernel(int n, int n_windows, const int *__restrict__ row_ptr,
                                                            int blk_h, int hub_thr, int4 *__restrict__ list_b1,
                                                            int4 *__restrict__ list_b2, int4 *__restrict__ list_b3,
                                                            int4 *__restrict__ list_b4, int *__restrict__ list_large,
                                                            int *__restrict__ list_hub, int4 *__restrict__ list_direct,
                                                            int direct, int *counters)
{
    __shared__ int cnt_s[7], base_s[7];
    if (threadIdx.x < 7) cnt_s[threadIdx.x] = 0;
    __syncthreads();
    const int w = blockIdx.x * 1024 + threadIdx.x;
    int cls = -1, pos = 0, e0 = 0, cnt = 0;
    if (w < n_windows) {
        const int r0 = w * blk_h;
        e0 = row_ptr[r0];
        cnt = row_ptr[min(n, r0 + blk_h)] - e0;
        if (cnt > WAVE_CAP)
            cls = cnt <= B1_CAP ? 0
                                : (cnt <= B2_CAP ? 1 : (cnt <= MID_CAP ? 2 : (direct ? 6 : (cnt <= hub_thr ? (cnt <= B4_CAP ? 3 : 4) : 5))));
    }
    // a window above DIRECT_SPLIT_MIN edges is queued once per part (see win_direct_kernel)
    const int parts = cls == 6 ? direct_parts(cnt) : 1;
    if (cls >= 0) pos = atomicAdd(&cnt_s[cls], parts);
    __syncthreads();
    if (threadIdx.x < 7 && cnt_s[threadIdx.x] > 0)
        base_s[threadIdx.x] = atomicAdd(&counters[threadIdx.x], cnt_s[threadIdx.x]);  // C_B1 .. C_DIRECT
    __syncthreads();
    // the bitmap kernels get the window's first edge and edge count with its id: one dependent load less per window
    if (cls == 0) list_b1[base_s[0] + pos] = make_int4(w, e0, cnt, 0);
    else if (cls == 1) list_b2[base_s[1] + pos] = make_int4(w, e0, cnt, 0);
    else if (cls == 2) list_b3[base_s[2] + pos] = make_int4(w, e0, cnt, 0);
    else if (cls == 3) list_b4[base_s[3] + pos] = make_int4(w, e0, cnt, 0);
    else if (cls == 4) list_large[base_s[4] + pos] = w;
    else if (cls == 5) list_hub[base_s[5] + pos] = w;
    else if (cls == 6)
        for (int part = 0; part < parts; ++part) list_direct[base_s[6] + pos + part] = make_int4(w, e0, cnt, part | (parts << 8));
}

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
    // Register k of lane l starts with the column of edge k * 64 + l, so that loads and the stores
    // below touch consecutive addresses in consecutive lanes (the sort takes its input in any order).
    int key[E], orig[E];
#pragma unroll
    for (int k = 0; k < E; ++k) {
        const int i = k * 64 + lane;
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
    const int incl = wave_inclusive_scan(mine);
    const int n_uniq = __shfl(incl, 63, 64);
    int pos = incl - mine;
#pragma unroll
    for (int k = 0; k < E; ++k) {
        if (flag[k]) uniq_lds[pos++] = key[k];
    }
    __syncthreads();  // single-wave workgroup: makes the unique list visible to all lanes
    for (int i = lane; i < n_uniq; i += 64) tmp_cols[e0 + i] = uniq_lds[i];
#pragma unroll
    for (int k = 0; k < E; ++k) {
        const int i = k * 64 + lane;
        if (i < cnt) {
            int lo = 0, hi = n_uniq;  // first index with uniq[idx] >= column
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (uniq_lds[mid] < orig[k]) lo = mid + 1; else hi = mid;
            }
            // the per-edge arrays are written once and read by no kernel of the build: the non-temporal hint keeps
            // them from pushing the unique lists (which the pack kernel reads back) out of the caches
            __builtin_nontemporal_store(lo, edge_to_col + e0 + i);
            int a = 0, b = rows;  // last row index with rp[a] <= edge
            while (b - a > 1) {
                const int mid = (a + b) >> 1;
                if (rp[mid] <= e0 + i) a = mid; else b = mid;
            }
            __builtin_nontemporal_store(r0 + a, edge_to_row + e0 + i);
        }
    }
    if (lane == 0) uniq_count[w] = n_uniq;
}

__global__ __launch_bounds__(64) void win_wave_kernel(int n, const int *__restrict__ row_ptr,
                                                      const int *__restrict__ col_idx, int blk_h,
                                                      int *__restrict__ edge_to_row,
                                                      int *__restrict__ edge_to_col,
                                                      int *__restrict__ uniq_count, int *__restrict__ tmp_cols)
{
    __shared__ int uniq_lds[WAVE_CAP];
    __shared__ int rp[65];
    const int w = blockIdx.x;
    const int r0 = w * blk_h;
    const int rows = min(n, r0 + blk_h) - r0;
    for (int t = threadIdx.x; t <= rows; t += 64) rp[t] = row_ptr[r0 + t];
    __syncthreads();
    const int cnt = rp[rows] - rp[0];
    if (cnt > WAVE_CAP) return;  // queued by the classification kernel for the bitmap kernels
    if (cnt == 0) {
        if (threadIdx.x == 0) uniq_count[w] = 0;
        return;
    }
#define FTC_WAVE(E) condense_window_wave<E>(w, r0, rows, rp, cnt, col_idx, edge_to_row, edge_to_col, uniq_count, tmp_cols, uniq_lds)
    if (cnt <= 64) FTC_WAVE(1);
    else if (cnt <= 128) FTC_WAVE(2);
    else FTC_WAVE(4);
#undef FTC_WAVE
}


// ---- windows of WAVE_CAP + 1 .. MID_CAP edges: one wave, two-level bitmap in LDS -------------------
// LDS operations of one wave execute in order; the fences keep the compiler from moving LDS reads
// above the writes of other lanes they depend on.
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

constexpr int WB_RANGE_LOG2 = 20;                     // column ids per pass over the coarse bitmap
constexpr int WB_CW = (1 << WB_RANGE_LOG2) / 1024;    // its words: one bit per 32-column word of the range

// One wave condenses one window of at most F edges; the window's column ids (F / 64 per lane) and the
// slots they fall into stay in registers.  Per range of 2^20 column ids:
//   A. coarse bitmap: which 32-column words does the window touch (at most one per edge, so at most F);
//   B. prefix sums of its popcounts number the touched words in ascending order (their "slots");
//   C. fine bitmap, one word per slot: set bits, prefix sums of the popcounts, rank of an edge =
//      prefix of its slot + bits below its own; every edge also stores its column id at its rank in
//      the unique list (edges with the same column store the same value to the same place).
// Lanes own 16-byte pieces of the bitmaps, piece p = lane + 64 q: the LDS accesses of a step touch 64
// consecutive pieces (no bank conflicts) and a step's prefix is one scan over the lanes.
// A persistent grid of single-wave workgroups that walks the queue with a stride of the grid size: a
// ticket counter (one atomic per window on a single address) would serialise tens of thousands of
// waves, 12 ns each, and the windows of a queue differ in size by at most a factor of four.
template <int F, int NW>
__global__ __launch_bounds__(64 * NW) void win_bitmap_wave_kernel(int n, int nnz, const int *__restrict__ row_ptr,
                                                                  const int *__restrict__ col_idx, int blk_h,
                                                                  int *__restrict__ edge_to_row,
                                                                  int *__restrict__ edge_to_col,
                                                                  int *__restrict__ uniq_count,
                                                                  int *__restrict__ tmp_cols,
                                                                  const int4 *__restrict__ list,
                                                                  const int *__restrict__ count)
{
    constexpr int NT = 64 * NW;
    constexpr int EPL = F / NT;              // edges per lane
    constexpr int NWC = NW < 4 ? NW : 4;     // waves that scan the coarse bitmap (it has 256 pieces)
    constexpr int CPW = WB_CW / 4 / NWC;     // its pieces per scanning wave ...
    constexpr int CP = CPW / 64;             // ... and per lane
    constexpr int FPW = F / 4 / NW;          // pieces of the fine bitmap per wave ...
    constexpr int FP = FPW / 64;             // ... and per lane
    static_assert(CP >= 1 && FP >= 1, "every lane owns at least one piece of each bitmap");
    constexpr bool AHEAD = EPL <= 32;        // registers for the next window's column ids as well
    __shared__ __attribute__((aligned(16))) uint32_t coarse[WB_CW];
    __shared__ __attribute__((aligned(16))) uint16_t cpre[WB_CW];   // slots before each coarse word, inside its wave's share
    __shared__ __attribute__((aligned(16))) uint32_t fine[F];
    __shared__ __attribute__((aligned(16))) uint16_t fpre[F];       // unique columns before each slot, inside its wave's share
    __shared__ int rp[65];
    __shared__ int wtot_c[2][NWC], wtot_f[2][NW];                   // per-wave totals of the two scans (double-buffered)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n_items = *count;
    const int stride = static_cast<int>(gridDim.x);
    // With one wave LDS operations execute in order and only the compiler has to be held back; with several
    // waves the phases are separated by workgroup barriers.
    auto sync = [&]() {
        if constexpr (NW == 1) wave_lds_sync();
        else __syncthreads();
    };
    if (wave < NWC) {
#pragma unroll
        for (int q = 0; q < CP; ++q)
            *reinterpret_cast<uint4 *>(&coarse[(wave * CPW + lane + 64 * q) * 4]) = make_uint4(0u, 0u, 0u, 0u);
    }
#pragma unroll
    for (int q = 0; q < FP; ++q)
        *reinterpret_cast<uint4 *>(&fine[(wave * FPW + lane + 64 * q) * 4]) = make_uint4(0u, 0u, 0u, 0u);
    const int n_ranges = static_cast<int>((static_cast<int64_t>(n) + (1 << WB_RANGE_LOG2) - 1) >> WB_RANGE_LOG2);
    // Every load that names the next windows is issued a window (the queue entry: two windows) ahead, so
    // that a window's own work starts with its column ids already in registers.
    int item = static_cast<int>(blockIdx.x);
    if (item >= n_items) return;
    int4 ent = list[item];
    int4 ent1 = list[min(item + stride, n_items - 1)];  // beyond the queue: the last entry once more, never used
    // Unconditional loads from clamped addresses, so that they are issued back to back (a branch around each
    // load makes the compiler wait for the previous one); which of them belong to the window is decided at use.
    auto load_cols = [&](const int4 &en, int (&c)[EPL]) {
#pragma unroll
        for (int k = 0; k < EPL; ++k) c[k] = col_idx[min(en.y + k * NT + tid, nnz - 1)];
    };
    // row starts of a window (for edge_to_row): thread r holds the start of row r, thread 0 also the 65th value
    // of a window of 64 rows; loaded a window ahead like the column ids
    auto load_starts = [&](const int4 &en, int &a, int &b) {
        const int r0 = en.x * blk_h;
        const int rows = min(n, r0 + blk_h) - r0;
        a = row_ptr[min(r0 + (tid & 63), n)];  // beyond the window's rows: never used
        b = row_ptr[min(r0 + 64, n)];
    };
    int col[EPL], col_ahead[AHEAD ? EPL : 1];
    int st_a = 0, st_b = 0, st_a_ahead = 0, st_b_ahead = 0;
    load_cols(ent, col);
    load_starts(ent, st_a, st_b);
    int parity = 0;
    for (; item < n_items; item += stride) {  // uniform
        const int w = ent.x, e0 = ent.y, cnt = min(ent.z, F);
        const int r0 = w * blk_h;
        const int rows = min(n, r0 + blk_h) - r0;
        sync();  // the previous window is done with rp; the clearing of the bitmaps is complete
        if (tid < 64) rp[tid] = st_a;
        if (tid == 0) rp[64] = st_b;
        __builtin_amdgcn_sched_barrier(0);  // the loads for the windows ahead are issued after this, not waited for here
        const int4 ent2 = list[min(item + 2 * stride, n_items - 1)];
        if (item + stride < n_items) {  // uniform
            if constexpr (AHEAD) load_cols(ent1, col_ahead);
            load_starts(ent1, st_a_ahead, st_b_ahead);
        }
        int base = 0;  // unique columns found so far
        for (int range = 0; range < n_ranges; ++range) {
            const int lo = range << WB_RANGE_LOG2;
            if (NW > 1 && range > 0) __syncthreads();  // the clearing after the previous range is complete
            // A. coarse bits
            bool any = false;
#pragma unroll
            for (int k = 0; k < EPL; ++k) {
                int ck = k * NT + tid < cnt ? col[k] : -1;
                asm volatile("" : "+v"(ck));  // what is derived from a column id is recomputed in every phase, not kept in registers
                const unsigned c = static_cast<unsigned>(ck - lo);
                if (ck >= 0 && c < (1u << WB_RANGE_LOG2)) {
                    atomicOr(&coarse[c >> 10], 1u << ((c >> 5) & 31));
                    any = true;
                }
                if ((k & 7) == 7) __builtin_amdgcn_sched_barrier(0);  // eight edges at a time: bounds the registers in flight
            }
            bool some;
            if constexpr (NW == 1) {
                wave_lds_sync();
                some = __builtin_amdgcn_ballot_w64(any) != 0ull;
            } else {
                some = __syncthreads_or(any ? 1 : 0) != 0;
            }
            if (!some) continue;  // none of the window's columns lies in this range (uniform)
            // B. number the touched words: every wave scans its share, the shares are joined through the wave totals
            int carry = 0;
            if (wave < NWC) {  // uniform over the wave
#pragma unroll
                for (int q = 0; q < CP; ++q) {
                    const int p = wave * CPW + lane + 64 * q;
                    const uint4 v = *reinterpret_cast<const uint4 *>(&coarse[p * 4]);
                    const int c0 = __popc(v.x), c1 = c0 + __popc(v.y), c2 = c1 + __popc(v.z), mine = c2 + __popc(v.w);
                    const int incl = wave_inclusive_scan(mine);
                    const unsigned run = static_cast<unsigned>(carry + incl - mine);
                    *reinterpret_cast<uint2 *>(&cpre[p * 4]) = make_uint2(run | ((run + c0) << 16), (run + c1) | ((run + c2) << 16));
                    carry += __shfl(incl, 63, 64);
                }
                if (lane == 0) wtot_c[parity][wave] = carry;
            }
            sync();
            int coff[NWC], n_slots = 0;  // slots before each scanning wave's share; at most one slot per edge in all
#pragma unroll
            for (int k = 0; k < NWC; ++k) {  // the same numbers in every lane: kept in scalar registers
                coff[k] = n_slots;
                n_slots += __builtin_amdgcn_readfirstlane(wtot_c[parity][k]);
            }
            // C. fine bits
            auto slot_of = [&](unsigned c) {
                const int cw = c >> 10;
                int off = 0;
#pragma unroll
                for (int k = 1; k < NWC; ++k) off = (cw >> 2) >= k * CPW ? coff[k] : off;
                return off + static_cast<int>(cpre[cw]) + __popc(coarse[cw] & ((1u << ((c >> 5) & 31)) - 1u));
            };
#pragma unroll
            for (int k = 0; k < EPL; ++k) {
                int ck = k * NT + tid < cnt ? col[k] : -1;
                asm volatile("" : "+v"(ck));
                const unsigned c = static_cast<unsigned>(ck - lo);
                if (ck >= 0 && c < (1u << WB_RANGE_LOG2)) atomicOr(&fine[slot_of(c)], 1u << (c & 31));
                if ((k & 7) == 7) __builtin_amdgcn_sched_barrier(0);
            }
            sync();
            carry = 0;
#pragma unroll
            for (int q = 0; q < FP; ++q) {
                if ((wave * FPW + 64 * q) * 4 < n_slots) {  // uniform over the wave
                    const int p = wave * FPW + lane + 64 * q;
                    const uint4 v = *reinterpret_cast<const uint4 *>(&fine[p * 4]);
                    const int c0 = __popc(v.x), c1 = c0 + __popc(v.y), c2 = c1 + __popc(v.z), mine = c2 + __popc(v.w);
                    const int incl = wave_inclusive_scan(mine);
                    const unsigned run = static_cast<unsigned>(carry + incl - mine);
                    *reinterpret_cast<uint2 *>(&fpre[p * 4]) = make_uint2(run | ((run + c0) << 16), (run + c1) | ((run + c2) << 16));
                    carry += __shfl(incl, 63, 64);
                }
            }
            if (lane == 0) wtot_f[parity][wave] = carry;
            sync();
            int foff[NW], range_total = 0;
#pragma unroll
            for (int k = 0; k < NW; ++k) {
                foff[k] = range_total;
                range_total += __builtin_amdgcn_readfirstlane(wtot_f[parity][k]);
            }
            parity ^= 1;
#pragma unroll
            for (int k = 0; k < EPL; ++k) {
                int ck = k * NT + tid < cnt ? col[k] : -1;
                asm volatile("" : "+v"(ck));
                const unsigned c = static_cast<unsigned>(ck - lo);
                if (ck >= 0 && c < (1u << WB_RANGE_LOG2)) {
                    const int sl = slot_of(c);
                    int off = 0;
#pragma unroll
                    for (int j = 1; j < NW; ++j) off = (sl >> 2) >= j * FPW ? foff[j] : off;
                    const int rank = base + off + static_cast<int>(fpre[sl]) + __popc(fine[sl] & ((1u << (c & 31)) - 1u));
                    __builtin_nontemporal_store(rank, edge_to_col + e0 + k * NT + tid);
                    tmp_cols[e0 + rank] = ck;
                }
                if ((k & 7) == 7) __builtin_amdgcn_sched_barrier(0);
            }
            base += range_total;
            sync();  // every lane is done reading the bitmaps
#pragma unroll
            for (int q = 0; q < FP; ++q)
                if ((wave * FPW + 64 * q) * 4 < n_slots)
                    *reinterpret_cast<uint4 *>(&fine[(wave * FPW + lane + 64 * q) * 4]) = make_uint4(0u, 0u, 0u, 0u);
            if (wave < NWC) {
#pragma unroll
                for (int q = 0; q < CP; ++q)
                    *reinterpret_cast<uint4 *>(&coarse[(wave * CPW + lane + 64 * q) * 4]) = make_uint4(0u, 0u, 0u, 0u);
            }
        }
        if (tid == 0) uniq_count[w] = base;
        sync();
        for (int r = wave; r < rows; r += NW) {
            const int b = min(rp[r + 1], e0 + cnt);
            for (int e = max(rp[r], e0) + lane; e < b; e += 64) __builtin_nontemporal_store(r0 + r, edge_to_row + e);
        }
        ent = ent1;
        ent1 = ent2;
        st_a = st_a_ahead;
        st_b = st_b_ahead;
        if constexpr (AHEAD) {
#pragma unroll
            for (int k = 0; k < EPL; ++k) col[k] = col_ahead[k];
        } else {
            if (item + stride < n_items) load_cols(ent, col);
        }
    }
}

// ---- windows above MID_CAP edges: one workgroup, one bit per column of a 2^20-column range in LDS -----------
// With this many edges the window touches a good part of the 32768 bitmap words of a range anyway, so the bitmap
// is kept whole (128 KiB of the CU's 160) and the coarse level drops out: set bits, prefix sums of the popcounts
// per 16-byte piece (each of the 16 waves scans a sixteenth, joined through the wave totals), rank of an edge =
// prefix of its piece + bits below its own, unique list written by the edges at their rank.  A window can have
// any number of edges (its column ids are read again in the second phase, from L2), so this one kernel takes
// what the two-level workgroup kernel and the edge-parallel hub kernels take on graphs of many column ranges,
// where a pass over all edges per range would cost too much.  Queue entries come from a ticket counter (a few
// hundred to a few thousand, very different in size); a window above DIRECT_SPLIT_MIN edges has several entries,
// one per part of its edges (see direct_parts): every part builds the whole bitmap and ranks its own edges, the
// unique list is the same whichever part writes an entry of it.
constexpr int DB_WORDS = (1 << WB_RANGE_LOG2) / 32;  // bitmap words per range
constexpr int DB_PIECES = DB_WORDS / 4;
__global__ __launch_bounds__(1024) void win_direct_kernel(int n, const int *__restrict__ row_ptr,
                                                          const int *__restrict__ col_idx, int blk_h,
                                                          int *__restrict__ edge_to_row, int *__restrict__ edge_to_col,
                                                          int *__restrict__ uniq_count, int *__restrict__ tmp_cols,
                                                          const int4 *__restrict__ list, const int *__restrict__ count,
                                                          int *next_ticket)
{
    constexpr int NT = 1024, NW = 16;
    constexpr int PW = DB_PIECES / NW;  // pieces per wave: 512
    constexpr int PL = PW / 64;         // ... and per lane: 8
    constexpr int EB = 8;               // edges per thread and batch
    __shared__ __attribute__((aligned(16))) uint32_t bits[DB_WORDS];
    __shared__ uint16_t pre[DB_PIECES];  // unique columns before each piece, inside its wave's share (below 65536)
    __shared__ int wtot[NW], woff[NW + 1];  // unique columns of every wave's share, and before it
    __shared__ int rp[65];
    __shared__ int next_s;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n_items = *count;
#pragma unroll
    for (int q = 0; q < PL; ++q) *reinterpret_cast<uint4 *>(&bits[(wave * PW + lane + 64 * q) * 4]) = make_uint4(0u, 0u, 0u, 0u);
    const int n_ranges = static_cast<int>((static_cast<int64_t>(n) + (1 << WB_RANGE_LOG2) - 1) >> WB_RANGE_LOG2);
    for (int item = blockIdx.x; item < n_items;) {  // uniform
        int ticket = 0;
        if (tid == 0) ticket = atomicAdd(next_ticket, 1) + static_cast<int>(gridDim.x);
        const int4 ent = list[item];
        const int w = ent.x, e0 = ent.y, cnt = ent.z;
        // the part of the window's edges this workgroup ranks (whole multiples of the workgroup, so that the parts'
        // loads stay aligned); the bitmap is built from all of the window's edges by every part
        const int parts = max(1, ent.w >> 8), part = ent.w & 255;
        const int per_part = ((cnt + parts - 1) / parts + NT - 1) / NT * NT;
        const int i_lo = min(cnt, part * per_part), i_hi = min(cnt, i_lo + per_part);
        const int r0 = w * blk_h;
        const int rows = min(n, r0 + blk_h) - r0;
        __syncthreads();  // the previous window is done with rp; the clearing of the bitmap is complete
        if (tid <= rows) rp[tid] = row_ptr[r0 + tid];
        // f(column or -1, index of the edge inside the window) for the edges lo .. hi - 1, EB loads in flight per thread
        // (the loads are unconditional, from an index clamped into the window: a load inside a branch is waited for at once)
        auto for_edges = [&](int lo, int hi, auto f) {
            for (int ib = lo + tid; ib < hi; ib += NT * EB) {
                int c8[EB];
#pragma unroll
                for (int j = 0; j < EB; ++j) c8[j] = col_idx[e0 + min(ib + j * NT, cnt - 1)];
#pragma unroll
                for (int j = 0; j < EB; ++j) f(ib + j * NT < hi ? c8[j] : -1, ib + j * NT);
            }
        };
        int base = 0;
        for (int range = 0; range < n_ranges; ++range) {
            const int lo = range << WB_RANGE_LOG2;
            if (range > 0) __syncthreads();  // the clearing after the previous range is complete
            bool any = false;
            for_edges(0, cnt, [&](int col, int) {
                const unsigned c = static_cast<unsigned>(col - lo);
                if (col >= 0 && c < (1u << WB_RANGE_LOG2)) {
                    // the popular columns of a large window are hit thousands of times and atomics on one address
                    // serialise: the word is read first and the atomic skipped when the bit is there (bits are only set)
                    uint32_t *p = &bits[c >> 5];
                    const uint32_t m = 1u << (c & 31);
                    if ((__hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) & m) == 0u) atomicOr(p, m);
                    any = true;
                }
            });
            if (!__syncthreads_or(any ? 1 : 0)) continue;  // none of the window's columns lies in this range
            int carry = 0;
#pragma unroll
            for (int q = 0; q < PL; ++q) {
                const int p = wave * PW + lane + 64 * q;
                const uint4 v = *reinterpret_cast<const uint4 *>(&bits[p * 4]);
                const int mine = __popc(v.x) + __popc(v.y) + __popc(v.z) + __popc(v.w);
                const int incl = wave_inclusive_scan(mine);
                pre[p] = static_cast<uint16_t>(carry + incl - mine);
                carry += __shfl(incl, 63, 64);
            }
            if (lane == 0) wtot[wave] = carry;
            __syncthreads();
            if (wave == 0) {
                const int t = lane < NW ? wtot[lane] : 0;
                const int incl = wave_inclusive_scan(t);
                if (lane < NW) woff[lane] = incl - t;
                if (lane == NW - 1) woff[NW] = incl;
            }
            __syncthreads();
            const int range_total = woff[NW];
            for_edges(i_lo, i_hi, [&](int col, int i) {
                const unsigned c = static_cast<unsigned>(col - lo);
                if (col >= 0 && c < (1u << WB_RANGE_LOG2)) {
                    const int piece = c >> 7, j = (c >> 5) & 3;
                    const uint4 v = *reinterpret_cast<const uint4 *>(&bits[piece * 4]);
                    const uint32_t own = j == 0 ? v.x : (j == 1 ? v.y : (j == 2 ? v.z : v.w));
                    const int rank = base + woff[piece / PW] + static_cast<int>(pre[piece]) + __popc(own & ((1u << (c & 31)) - 1u)) +
                                     (j > 0 ? __popc(v.x) : 0) + (j > 1 ? __popc(v.y) : 0) + (j > 2 ? __popc(v.z) : 0);
                    __builtin_nontemporal_store(rank, edge_to_col + e0 + i);
                    tmp_cols[e0 + rank] = col;
                }
            });
            base += range_total;
            __syncthreads();  // every thread is done reading the bitmap
#pragma unroll
            for (int q = 0; q < PL; ++q)
                *reinterpret_cast<uint4 *>(&bits[(wave * PW + lane + 64 * q) * 4]) = make_uint4(0u, 0u, 0u, 0u);
        }
        if (tid == 0) {
            if (part == 0) uniq_count[w] = base;
            next_s = ticket;
        }
        __syncthreads();  // rp (written before the first barrier of the window) and next_s
        for (int r = wave; r < rows; r += NW) {
            const int b = min(rp[r + 1], e0 + i_hi);
            for (int e = max(rp[r], e0 + i_lo) + lane; e < b; e += 64) __builtin_nontemporal_store(r0 + r, edge_to_row + e);
        }
        item = next_s;
    }
}

// ---- queued windows below the hub threshold: two-level bitmap in LDS ------------------------------
// A window of c edges touches at most c of the n / 32 bitmap words of the column space, so the
// bitmap is kept compact.  Per range of 2^CRANGE_LOG2 column ids:
//   A. a coarse bitmap with one bit per 32-column word says which words the window touches;
//   B. prefix sums of its popcounts number the touched words in ascending order ("slots");
//   C. the fine bitmap holds one 32-bit word per slot (FINE_SLOTS slots at a time): set bits,
//      prefix sums of the popcounts, rank of an edge = prefix of its slot + bits below its own;
//      the unique list comes out of the same pass, ascending.
// The cost depends on the window's edge count, not on n; nothing is walked once per column range
// except the window's own column ids.
constexpr int CRANGE_LOG2 = 20;
constexpr int CW = (1 << CRANGE_LOG2) / 1024;  // coarse words per range

// A thread owns a run of consecutive LDS words and moves it with 16-byte accesses.  With a
// thread-to-thread stride of 8 or 16 words those would fall on a few banks only, so such arrays get
// a stride whose count of 16-byte pieces is odd.
constexpr int lds_stride_words(int words_per_thread)
{
    return words_per_thread >= 4 && (words_per_thread / 4) % 2 == 0 ? words_per_thread + 4 : words_per_thread;
}

// NT threads condense one window at a time.  RankT holds a rank inside one pass over the fine
// bitmap (16 bits when the window has fewer than 2^16 edges).
template <int NT, int FINE_SLOTS, class RankT, int MIN_WG_PER_CU>
__global__ __launch_bounds__(NT, MIN_WG_PER_CU) void win_compact_kernel(
    int n, const int *__restrict__ row_ptr, const int *__restrict__ col_idx, int blk_h,
    int *__restrict__ edge_to_row, int *__restrict__ edge_to_col, int *__restrict__ uniq_count,
    int *__restrict__ tmp_cols, const int *__restrict__ list, const int *__restrict__ count, int *next_ticket)
{
    constexpr int CPT = CW / NT;                       // coarse words owned by a thread
    constexpr int FPT = FINE_SLOTS / NT;               // fine words owned by a thread
    constexpr int RANKS_PER_WORD = 4 / sizeof(RankT);  // ranks packed into one 32-bit LDS word
    constexpr int RW = FPT / RANKS_PER_WORD;           // 32-bit words of ranks owned by a thread
    static_assert(CPT >= 1 && FPT >= 4 && FPT % 4 == 0 && RW >= 4 && RW % 4 == 0, "16-byte pieces");
    constexpr int SF = lds_stride_words(FPT);
    constexpr int SR = lds_stride_words(RW);
    __shared__ __attribute__((aligned(16))) uint32_t coarse[CW];        // zero between ranges
    __shared__ __attribute__((aligned(16))) uint32_t cpre[CW];          // touched words before each coarse word
    __shared__ __attribute__((aligned(16))) uint32_t fine[NT * SF];     // zero between passes
    __shared__ __attribute__((aligned(16))) uint32_t fpre[NT * SR];     // unique columns of the pass before each slot
    __shared__ uint16_t slot_word[FINE_SLOTS];                          // bitmap word (inside the range) of each slot
    __shared__ int wave_tot[NT / 64];
    __shared__ int rp[65];
    __shared__ int next_s;
    const int tid = threadIdx.x;
    const int n_items = *count;
    auto fpos = [](int slot) { return (slot / FPT) * SF + (slot % FPT); };
    auto rpos = [](int slot) { return (slot / FPT) * (SR * RANKS_PER_WORD) + (slot % FPT); };
    for (int k = 0; k < CPT; ++k) coarse[tid * CPT + k] = 0u;
#pragma unroll
    for (int k = 0; k < FPT; k += 4) *reinterpret_cast<uint4 *>(&fine[tid * SF + k]) = make_uint4(0u, 0u, 0u, 0u);
    // A persistent grid: one workgroup per possible queue entry would start tens of thousands of
    // workgroups that only find the queue shorter than the bound.  The first item is the
    // workgroup's own index, later ones come from a ticket counter whose atomic is issued before
    // the current window is condensed, so that its latency is hidden.
    for (int item = blockIdx.x; item < n_items;) {  // uniform
        int ticket = 0;
        if (tid == 0) ticket = atomicAdd(next_ticket, 1) + static_cast<int>(gridDim.x);
        const int w = list[item];
        const int r0 = w * blk_h;
        const int rows = min(n, r0 + blk_h) - r0;
        __syncthreads();  // the previous window is done with rp; the initial clearing is complete
        if (tid <= rows) rp[tid] = row_ptr[r0 + tid];
        __syncthreads();
        const int e0 = rp[0], e1 = rp[rows];
        for (int e = e0 + tid; e < e1; e += NT) __builtin_nontemporal_store(r0 + row_of_edge(rp, rows, e), edge_to_row + e);
        // f(column, edge) for every edge of the window.  The column ids are read again in every
        // phase (they come from L2 after the first time): keeping them in registers between the
        // phases was measured slower, because it halves the number of workgroups a CU can hold.
        auto for_edges = [&](auto f) {
            for (int eb = e0 + tid; eb < e1; eb += NT * 8) {
                int c8[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int e = eb + j * NT;
                    c8[j] = e < e1 ? col_idx[e] : -1;
                }
#pragma unroll
                for (int j = 0; j < 8; ++j) f(c8[j], eb + j * NT);
            }
        };
        const int n_ranges = static_cast<int>((static_cast<int64_t>(n) + (1 << CRANGE_LOG2) - 1) >> CRANGE_LOG2);
        int base = 0;  // unique columns found so far
        for (int range = 0; range < n_ranges; ++range) {
            const int lo = range << CRANGE_LOG2;
            // A. which bitmap words of this range does the window touch
            bool any = false;
            for_edges([&](int col, int) {
                const unsigned c = static_cast<unsigned>(col - lo);
                if (col >= 0 && c < (1u << CRANGE_LOG2)) {
                    atomicOr(&coarse[c >> 10], 1u << ((c >> 5) & 31));
                    any = true;
                }
            });
            if (!__syncthreads_or(any ? 1 : 0)) continue;  // none of the window's columns lies in this range
            // B. number the touched words
            uint32_t cwv[CPT];
            int mine = 0;
#pragma unroll
            for (int k = 0; k < CPT; ++k) {
                cwv[k] = coarse[tid * CPT + k];
                mine += __popc(cwv[k]);
            }
            int n_slots;
            const int first_slot = block_scan_one_barrier<NT>(mine, wave_tot, &n_slots);
            {
                int run = first_slot;
#pragma unroll
                for (int k = 0; k < CPT; ++k) {
                    cpre[tid * CPT + k] = run;
                    run += __popc(cwv[k]);
                }
            }
            // slot of a column of this range (its bitmap word is touched by construction)
            auto slot_of = [&](unsigned c) {
                const int cw = c >> 10;
                return static_cast<int>(cpre[cw]) + __popc(coarse[cw] & ((1u << ((c >> 5) & 31)) - 1u));
            };
            // C. fine bitmap, FINE_SLOTS slots per pass
            for (int s0 = 0; s0 < n_slots; s0 += FINE_SLOTS) {  // uniform
                {   // bitmap word of every slot of this pass, from the owners of the coarse words
                    int run = first_slot;
#pragma unroll
                    for (int k = 0; k < CPT; ++k) {
                        for (uint32_t m = cwv[k]; m; m &= m - 1) {
                            const unsigned rel = static_cast<unsigned>(run - s0);
                            if (rel < static_cast<unsigned>(FINE_SLOTS))
                                slot_word[rel] = static_cast<uint16_t>((tid * CPT + k) * 32 + (__ffs(m) - 1));
                            ++run;
                        }
                    }
                }
                __syncthreads();  // cpre (first pass) and slot_word are complete
                for_edges([&](int col, int) {
                    const unsigned c = static_cast<unsigned>(col - lo);
                    if (col >= 0 && c < (1u << CRANGE_LOG2)) {
                        const unsigned rel = static_cast<unsigned>(slot_of(c) - s0);
                        if (rel < static_cast<unsigned>(FINE_SLOTS)) atomicOr(&fine[fpos(rel)], 1u << (c & 31));
                    }
                });
                __syncthreads();
                uint32_t fw[FPT];
#pragma unroll
                for (int k = 0; k < FPT; k += 4) {
                    const uint4 v = *reinterpret_cast<const uint4 *>(&fine[tid * SF + k]);
                    fw[k] = v.x; fw[k + 1] = v.y; fw[k + 2] = v.z; fw[k + 3] = v.w;
                }
                int cnt_mine = 0;
#pragma unroll
                for (int k = 0; k < FPT; ++k) cnt_mine += __popc(fw[k]);
                int pass_total;
                int run = block_scan_one_barrier<NT>(cnt_mine, wave_tot, &pass_total);
                uint32_t rw[RW];
#pragma unroll
                for (int k = 0; k < RW; ++k) rw[k] = 0u;
#pragma unroll
                for (int k = 0; k < FPT; ++k) {
                    rw[k / RANKS_PER_WORD] |= static_cast<uint32_t>(run) << (8 * sizeof(RankT) * (k % RANKS_PER_WORD));
                    if (fw[k]) {
                        const int col0 = lo + static_cast<int>(slot_word[tid * FPT + k]) * 32;
                        for (uint32_t m = fw[k]; m; m &= m - 1) tmp_cols[e0 + base + run++] = col0 + (__ffs(m) - 1);
                    }
                }
#pragma unroll
                for (int k = 0; k < RW; k += 4)
                    *reinterpret_cast<uint4 *>(&fpre[tid * SR + k]) = make_uint4(rw[k], rw[k + 1], rw[k + 2], rw[k + 3]);
                __syncthreads();
                const RankT *fpre_e = reinterpret_cast<const RankT *>(fpre);
                for_edges([&](int col, int e) {
                    const unsigned c = static_cast<unsigned>(col - lo);
                    if (col >= 0 && c < (1u << CRANGE_LOG2)) {
                        const unsigned rel = static_cast<unsigned>(slot_of(c) - s0);
                        if (rel < static_cast<unsigned>(FINE_SLOTS))
                            edge_to_col[e] = base + static_cast<int>(fpre_e[rpos(rel)]) +
                                             __popc(fine[fpos(rel)] & ((1u << (c & 31)) - 1u));
                    }
                });
                base += pass_total;
                __syncthreads();  // every thread is done reading fine, fpre, slot_word
#pragma unroll
                for (int k = 0; k < FPT; k += 4)
                    if (fw[k] | fw[k + 1] | fw[k + 2] | fw[k + 3])
                        *reinterpret_cast<uint4 *>(&fine[tid * SF + k]) = make_uint4(0u, 0u, 0u, 0u);
            }
            // the coarse words were last read in the ranking, before the barrier above
#pragma unroll
            for (int k = 0; k < CPT; ++k)
                if (cwv[k]) coarse[tid * CPT + k] = 0u;
            __syncthreads();
        }
        if (tid == 0) {
            uniq_count[w] = base;
            next_s = ticket;
        }
        __syncthreads();
        item = next_s;
    }
}

// ---- hub windows: one bitmap of n bits per hub in global memory, edge-parallel ---------------------
// Single workgroup: work items (HUB_CHUNK edges of one hub) and the table that maps an item to its hub.
__global__ __launch_bounds__(1024) void hub_plan_kernel(int n, const int *__restrict__ row_ptr, int blk_h,
                                                        const int *__restrict__ list_hub, int *counters,
                                                        int *__restrict__ hub_chunk_ptr,
                                                        int *__restrict__ chunk_table)
{
    __shared__ int scan_tmp[1024 / 64 + 1];
    __shared__ int s_ptr[HUB_SLOTS_MAX + 1];
    const int tid = threadIdx.x;
    const int nh = counters[C_HUB];
    int chunks = 0;
    if (tid < nh) {
        const int r0 = list_hub[tid] * blk_h;
        const int cnt = row_ptr[min(n, r0 + blk_h)] - row_ptr[r0];
        chunks = (cnt + HUB_CHUNK - 1) / HUB_CHUNK;
    }
    int total;
    const int ex = block_exclusive_scan<1024>(chunks, scan_tmp, &total);
    s_ptr[tid] = ex;
    if (tid == 0) {
        s_ptr[HUB_SLOTS_MAX] = total;
        counters[C_CHUNKS] = total;
        hub_chunk_ptr[nh] = total;
    }
    if (tid < nh) hub_chunk_ptr[tid] = ex;
    __syncthreads();
    for (int h = 0; h < nh; ++h) {
        const int p = s_ptr[h], q = s_ptr[h + 1];  // s_ptr[nh] == total also when nh < HUB_SLOTS_MAX
        for (int t = p + tid; t < q; t += 1024) chunk_table[t] = h;
    }
}

__global__ __launch_bounds__(256) void hub_clear_kernel(const int *__restrict__ counters, uint32_t *hub_bits,
                                                        int wps)
{
    const int64_t total = static_cast<int64_t>(counters[C_HUB]) * (wps / 4);  // 16-byte pieces of the used slots
    uint4 *p = reinterpret_cast<uint4 *>(hub_bits);
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; i < total;
         i += static_cast<int64_t>(gridDim.x) * 256)
        p[i] = make_uint4(0u, 0u, 0u, 0u);
}

// RANK = false: edge_to_row and the bitmap bits of every hub edge.  RANK = true: edge_to_col from the
// finished bitmaps and the group prefixes.
template <bool RANK>
__global__ __launch_bounds__(256) void hub_edges_kernel(int n, const int *__restrict__ row_ptr,
                                                        const int *__restrict__ col_idx, int blk_h,
                                                        const int *__restrict__ list_hub,
                                                        const int *__restrict__ counters,
                                                        const int *__restrict__ hub_chunk_ptr,
                                                        const int *__restrict__ chunk_table,
                                                        uint32_t *hub_bits, const int *__restrict__ hub_grp,
                                                        int wps, int *__restrict__ edge_to_row,
                                                        int *__restrict__ edge_to_col,
                                                        int *__restrict__ tmp_cols)
{
    __shared__ int rp[65];
    constexpr int PER = HUB_CHUNK / 256;
    const int tid = threadIdx.x;
    const int total = counters[C_CHUNKS];
    if constexpr (RANK) {
        // Unique lists of all hubs.  A work item is a tile of 256 bitmap words of one hub: ranks
        // inside the tile from a workgroup scan, column ids parked in LDS at their rank, then copied
        // out with consecutive lanes writing consecutive entries.  (Writing them straight from the
        // thread that owns the word costs a store instruction one cycle per lane, and the low
        // columns of a hub are dense.)
        __shared__ int stage[256 * 32];
        __shared__ int wave_tot[2][4];
        const int tiles = (wps + 255) / 256;
        const int items = counters[C_HUB] * tiles;
        int parity = 0;
        for (int it = blockIdx.x; it < items; it += gridDim.x) {  // uniform trip count per workgroup
            const int slot = it / tiles, word = (it % tiles) * 256 + tid;
            const uint32_t v = word < wps ? hub_bits[static_cast<size_t>(slot) * wps + word] : 0u;
            int tile_total;
            int off = block_scan_one_barrier<256>(__popc(v), wave_tot[parity], &tile_total);
            parity ^= 1;
            if (tile_total == 0) continue;  // uniform
            for (uint32_t m = v; m; m &= m - 1) stage[off++] = word * 32 + (__ffs(m) - 1);
            __syncthreads();
            // the tile starts at a group boundary (256 is a multiple of HUB_GROUP)
            const int dst = row_ptr[list_hub[slot] * blk_h] +
                            hub_grp[static_cast<size_t>(slot) * (wps / HUB_GROUP) + (it % tiles) * (256 / HUB_GROUP)];
            for (int i = tid; i < tile_total; i += 256) tmp_cols[dst + i] = stage[i];
            __syncthreads();  // stage is free again
        }
    }
    for (int c = blockIdx.x; c < total; c += gridDim.x) {  // uniform trip count per workgroup
        const int slot = chunk_table[c];
        const int r0 = list_hub[slot] * blk_h;
        const int rows = min(n, r0 + blk_h) - r0;
        __syncthreads();  // the previous item is done with rp
        if (tid <= rows) rp[tid] = row_ptr[r0 + tid];
        __syncthreads();
        const int e0 = rp[0] + (c - hub_chunk_ptr[slot]) * HUB_CHUNK;
        const int e1 = min(rp[rows], e0 + HUB_CHUNK);
        uint32_t *bm = hub_bits + static_cast<size_t>(slot) * wps;
        int col[PER];
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const int e = e0 + tid + q * 256;
            col[q] = e < e1 ? col_idx[e] : -1;
        }
        if constexpr (!RANK) {
            const int lane = tid & 63;
#pragma unroll
            for (int q = 0; q < PER; ++q) {
                const int e = e0 + tid + q * 256;
                if (col[q] >= 0) __builtin_nontemporal_store(r0 + row_of_edge(rp, rows, e), edge_to_row + e);
                // Consecutive lanes hold consecutive edges, and inside a (sorted) row consecutive
                // edges of a hub often fall into the same bitmap word: their bits are OR-ed along
                // the lanes (a scan over runs of equal words) and only the last lane of a run goes
                // to memory.  Atomics on one address serialise, and the popular columns of a hub are
                // hit thousands of times; for the same reason the word is read first (from L2,
                // where the atomics execute) and the atomic is skipped when nothing is missing.
                // Bits are only ever set, so a set bit that is read is never wrong.
                const int word = col[q] >= 0 ? col[q] >> 5 : -1 - lane;  // invalid lanes match nobody
                uint32_t bits = col[q] >= 0 ? 1u << (col[q] & 31) : 0u;
#pragma unroll
                for (int d = 1; d < 64; d <<= 1) {
                    const int ow = __shfl_up(word, d, 64);
                    const uint32_t ob = __shfl_up(bits, d, 64);
                    if (lane >= d && ow == word) bits |= ob;
                }
                const int nw = __shfl_down(word, 1, 64);
                if (col[q] >= 0 && (lane == 63 || nw != word)) {
                    uint32_t *p = &bm[word];
                    if ((__hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & bits) != bits) atomicOr(p, bits);
                }
            }
        } else {
            const int *gp = hub_grp + static_cast<size_t>(slot) * (wps / HUB_GROUP);
#pragma unroll
            for (int q = 0; q < PER; ++q) {
                if (col[q] >= 0) {
                    const int word = col[q] >> 5, g = word / HUB_GROUP, j = word % HUB_GROUP;
                    const uint4 a = *reinterpret_cast<const uint4 *>(bm + g * HUB_GROUP);
                    const uint4 b = *reinterpret_cast<const uint4 *>(bm + g * HUB_GROUP + 4);
                    const uint32_t wv[HUB_GROUP] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
                    const uint32_t below = (1u << (col[q] & 31)) - 1u;
                    int r = gp[g];
#pragma unroll
                    for (int k = 0; k < HUB_GROUP; ++k) r += __popc(wv[k] & (k < j ? 0xffffffffu : (k == j ? below : 0u)));
                    __builtin_nontemporal_store(r, edge_to_col + e0 + tid + q * 256);
                }
            }
        }
    }
}

// One workgroup per hub: prefix of the popcounts per group of HUB_GROUP words, and the unique count.
// (The unique lists are written by the ranking kernel, spread over the whole GPU: scattered 4-byte
// stores cost a CU one cycle per lane, and a hub can have 10^5 distinct columns.)
__global__ __launch_bounds__(1024) void hub_scan_kernel(const int *__restrict__ list_hub,
                                                        const int *__restrict__ counters,
                                                        const uint32_t *__restrict__ hub_bits,
                                                        int *__restrict__ hub_grp, int wps,
                                                        int *__restrict__ uniq_count)
{
    __shared__ int wave_tot[2][1024 / 64];
    const int slot = blockIdx.x;
    if (slot >= counters[C_HUB]) return;  // uniform
    const int tid = threadIdx.x;
    const int w = list_hub[slot];
    const int n_groups = wps / HUB_GROUP;
    const uint32_t *bm = hub_bits + static_cast<size_t>(slot) * wps;
    int *gp = hub_grp + static_cast<size_t>(slot) * n_groups;
    int carry = 0, parity = 0;
    for (int g0 = 0; g0 < n_groups; g0 += 1024) {  // uniform trip count
        const int g = g0 + tid;
        uint32_t wv[HUB_GROUP] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
        if (g < n_groups) {
            const uint4 a = *reinterpret_cast<const uint4 *>(bm + g * HUB_GROUP);
            const uint4 b = *reinterpret_cast<const uint4 *>(bm + g * HUB_GROUP + 4);
            wv[0] = a.x; wv[1] = a.y; wv[2] = a.z; wv[3] = a.w;
            wv[4] = b.x; wv[5] = b.y; wv[6] = b.z; wv[7] = b.w;
        }
        int mine = 0;
#pragma unroll
        for (int k = 0; k < HUB_GROUP; ++k) mine += __popc(wv[k]);
        int tile_total;
        // two buffers: a fast thread may start the next scan while a slow one still reads this one's
        // totals; the scan after that is separated from this one by the next scan's barrier
        int run = carry + block_scan_one_barrier<1024>(mine, wave_tot[parity], &tile_total);
        parity ^= 1;
        if (g < n_groups) gp[g] = run;
        carry += tile_total;
    }
    if (tid == 0) uniq_count[w] = carry;
}

// Single workgroup: exclusive scan of the per-window unique counts.  A round covers 4096 windows
// (every thread takes four consecutive ones); the loads of SCAN_ROUNDS rounds are issued together so
// that a pass over 65536 windows pays the memory latency once.
constexpr int SCAN_ROUNDS = 16;
__global__ __launch_bounds__(1024) void win_scan_kernel(int n_windows, int blk_w,
                                                        const int *__restrict__ uniq_count,
                                                        int *__restrict__ win_col_ptr,
                                                        int *__restrict__ block_partition,
                                                        int64_t *__restrict__ summary)
{
    __shared__ int wave_tot[2][1024 / 64];
    __shared__ long long blocks_s[16];
    const int tid = threadIdx.x;
    const int shift = (blk_w & (blk_w - 1)) == 0 ? __ffs(blk_w) - 1 : -1;  // blk_w a power of two: no division
    auto blocks_of = [&](int u) { return shift >= 0 ? (u + blk_w - 1) >> shift : (u + blk_w - 1) / blk_w; };
    const bool vec_ok = ((reinterpret_cast<uintptr_t>(win_col_ptr) | reinterpret_cast<uintptr_t>(block_partition)) & 15u) == 0;
    int carry = 0, parity = 0;
    long long my_blocks = 0;
    for (int super0 = 0; super0 < n_windows; super0 += 4096 * SCAN_ROUNDS) {  // uniform trip count
        int u[SCAN_ROUNDS][4];
#pragma unroll
        for (int r = 0; r < SCAN_ROUNDS; ++r) {
            const int first = super0 + r * 4096 + tid * 4;
            if (first + 3 < n_windows) {  // uniq_count lives in the workspace: 256-byte aligned
                const int4 v = *reinterpret_cast<const int4 *>(uniq_count + first);
                u[r][0] = v.x; u[r][1] = v.y; u[r][2] = v.z; u[r][3] = v.w;
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) u[r][j] = first + j < n_windows ? uniq_count[first + j] : 0;
            }
        }
#pragma unroll
        for (int r = 0; r < SCAN_ROUNDS; ++r) {
            const int first = super0 + r * 4096 + tid * 4;
            if (super0 + r * 4096 < n_windows) {  // uniform
            int round_total;
            int run = carry + block_scan_one_barrier<1024>(u[r][0] + u[r][1] + u[r][2] + u[r][3],
                                                           wave_tot[parity], &round_total);
            parity ^= 1;
            if (vec_ok && first + 3 < n_windows) {
                // one 16-byte store per array: scalar stores with a lane stride of 16 bytes cost the
                // single CU this kernel runs on four times as many memory instructions
                const int p1 = run + u[r][0], p2 = p1 + u[r][1], p3 = p2 + u[r][2];
                const int4 b = make_int4(blocks_of(u[r][0]), blocks_of(u[r][1]), blocks_of(u[r][2]), blocks_of(u[r][3]));
                *reinterpret_cast<int4 *>(win_col_ptr + first) = make_int4(run, p1, p2, p3);
                *reinterpret_cast<int4 *>(block_partition + first) = b;
                my_blocks += static_cast<long long>(b.x) + b.y + b.z + b.w;
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (first + j < n_windows) {
                        win_col_ptr[first + j] = run;
                        const int blocks = blocks_of(u[r][j]);
                        block_partition[first + j] = blocks;
                        my_blocks += blocks;
                        run += u[r][j];
                    }
                }
            }
            carry += round_total;
            }
        }
    }
    // sum of blocks over the workgroup
    long long v = my_blocks;
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
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

// ---- the same scan on many workgroups ------------------------------------------------------------------
// A single workgroup needs 23 us for 65536 windows, all of it latency.  Two small kernels instead: every
// workgroup adds up the unique counts (and tile counts) of its SCAN_CHUNK windows; then every workgroup adds
// the sums of the chunks before its own (at most SCAN_CHUNKS_MAX of them), scans its own windows and writes
// win_col_ptr, block_partition and, for every run of PACK_PER_WAVE entries of win_cols that begins inside
// one of its lists, the window that holds the run's first entry (what win_pack_plan_kernel writes after
// the single-workgroup scan).  Integer sums: the result does not depend on the order.
__device__ __forceinline__ int tiles_of(int u, int blk_w, int shift)
{
    return shift >= 0 ? (u + blk_w - 1) >> shift : (u + blk_w - 1) / blk_w;
}

__device__ __forceinline__ void load_counts4(const int *__restrict__ uniq_count, int first, int n_windows, int (&u)[4])
{
    if (first + 3 < n_windows) {  // uniq_count lives in the workspace: 256-byte aligned
        const int4 v = *reinterpret_cast<const int4 *>(uniq_count + first);
        u[0] = v.x; u[1] = v.y; u[2] = v.z; u[3] = v.w;
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) u[j] = first + j < n_windows ? uniq_count[first + j] : 0;
    }
}

__global__ __launch_bounds__(256) void win_chunk_sums_kernel(int n_windows, int blk_w, const int *__restrict__ uniq_count,
                                                             int *__restrict__ chunk_uniq,
                                                             long long *__restrict__ chunk_blocks)
{
    __shared__ int su[4];
    __shared__ long long sb[4];
    const int tid = threadIdx.x;
    const int shift = (blk_w & (blk_w - 1)) == 0 ? __ffs(blk_w) - 1 : -1;
    int u[4];
    load_counts4(uniq_count, blockIdx.x * SCAN_CHUNK + tid * 4, n_windows, u);
    int a = u[0] + u[1] + u[2] + u[3];
    long long b = static_cast<long long>(tiles_of(u[0], blk_w, shift)) + tiles_of(u[1], blk_w, shift) +
                  tiles_of(u[2], blk_w, shift) + tiles_of(u[3], blk_w, shift);
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        a += __shfl_xor(a, m, 64);
        b += __shfl_xor(b, m, 64);
    }
    if ((tid & 63) == 0) { su[tid >> 6] = a; sb[tid >> 6] = b; }
    __syncthreads();
    if (tid == 0) {
        chunk_uniq[blockIdx.x] = su[0] + su[1] + su[2] + su[3];
        chunk_blocks[blockIdx.x] = sb[0] + sb[1] + sb[2] + sb[3];
    }
}

__global__ __launch_bounds__(256) void win_chunk_scan_kernel(int n_windows, int blk_w, const int *__restrict__ uniq_count,
                                                             const int *__restrict__ chunk_uniq,
                                                             const long long *__restrict__ chunk_blocks,
                                                             int *__restrict__ win_col_ptr,
                                                             int *__restrict__ block_partition,
                                                             int64_t *__restrict__ summary, int *__restrict__ pack_win)
{
    __shared__ int su[4];
    __shared__ long long sb[4];
    __shared__ int wave_tot[4];
    const int tid = threadIdx.x;
    const int shift = (blk_w & (blk_w - 1)) == 0 ? __ffs(blk_w) - 1 : -1;
    const bool vec_ok = ((reinterpret_cast<uintptr_t>(win_col_ptr) | reinterpret_cast<uintptr_t>(block_partition)) & 15u) == 0;
    const int first = blockIdx.x * SCAN_CHUNK + tid * 4;
    int u[4];
    load_counts4(uniq_count, first, n_windows, u);
    // sums of the chunks before this one (and, in the last workgroup, of all chunks: the summary)
    const bool last = blockIdx.x == gridDim.x - 1;
    int a = 0;
    long long b = 0;
    for (int c = tid; c < static_cast<int>(blockIdx.x); c += 256) {
        a += chunk_uniq[c];
        if (last) b += chunk_blocks[c];
    }
    if (last && tid == 0) b += chunk_blocks[blockIdx.x];
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        a += __shfl_xor(a, m, 64);
        b += __shfl_xor(b, m, 64);
    }
    if ((tid & 63) == 0) { su[tid >> 6] = a; sb[tid >> 6] = b; }
    __syncthreads();
    const int carry = su[0] + su[1] + su[2] + su[3];
    int chunk_total;
    const int run = carry + block_scan_one_barrier<256>(u[0] + u[1] + u[2] + u[3], wave_tot, &chunk_total);
    const int p[5] = {run, run + u[0], run + u[0] + u[1], run + u[0] + u[1] + u[2], run + u[0] + u[1] + u[2] + u[3]};
    if (vec_ok && first + 3 < n_windows) {
        *reinterpret_cast<int4 *>(win_col_ptr + first) = make_int4(p[0], p[1], p[2], p[3]);
        *reinterpret_cast<int4 *>(block_partition + first) =
            make_int4(tiles_of(u[0], blk_w, shift), tiles_of(u[1], blk_w, shift), tiles_of(u[2], blk_w, shift),
                      tiles_of(u[3], blk_w, shift));
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (first + j < n_windows) {
                win_col_ptr[first + j] = p[j];
                block_partition[first + j] = tiles_of(u[j], blk_w, shift);
            }
        }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if (first + j < n_windows) {
            // runs of the pack kernel that begin inside this window's list
            for (long long c = (p[j] + static_cast<long long>(PACK_PER_WAVE) - 1) / PACK_PER_WAVE; c * PACK_PER_WAVE < p[j + 1]; ++c)
                pack_win[c] = first + j;
            if (first + j == n_windows - 1) {
                pack_win[(p[j + 1] + static_cast<long long>(PACK_PER_WAVE) - 1) / PACK_PER_WAVE] = first + j;
                win_col_ptr[n_windows] = p[j + 1];
                summary[0] = p[j + 1];
            }
        }
    }
    if (last && tid == 0) summary[1] = sb[0] + sb[1] + sb[2] + sb[3];
}

// The pack kernel's work units are runs of PACK_PER_WAVE entries of win_cols.  Every window names
// itself to the runs that begin inside its list (none for most windows; at most n / PACK_PER_WAVE + 1
// for one window, since a list has at most n entries); the entry after the last run holds the last
// window, so that a run always finds the window of its successor's first entry.
__global__ __launch_bounds__(256) void win_pack_plan_kernel(int n_windows, const int *__restrict__ win_col_ptr,
                                                            int *__restrict__ pack_win)
{
    const int w = blockIdx.x * 256 + threadIdx.x;
    if (w >= n_windows) return;
    const int b = win_col_ptr[w], e = win_col_ptr[w + 1];
    for (int c = static_cast<int>((b + static_cast<long long>(PACK_PER_WAVE) - 1) / PACK_PER_WAVE);
         c * static_cast<long long>(PACK_PER_WAVE) < e; ++c)
        pack_win[c] = w;
    if (w == n_windows - 1) pack_win[(e + static_cast<long long>(PACK_PER_WAVE) - 1) / PACK_PER_WAVE] = w;
}

// Packs the unique lists.  Window w's list lies at the start of its slot range of the temporary array
// (the slot of an edge is its index) and goes to win_cols[win_col_ptr[w] ...].  The work is balanced
// over the OUTPUT: a wave copies PACK_PER_WAVE consecutive entries of win_cols, so only list entries
// are read (13 % of the slots on the R-MAT workload hold none) and no per-edge array is needed to
// name the window.  The plan kernel has left the window of every run's first entry in pack_win (a
// search over win_col_ptr here, 64 or 256 scattered probes per wave and round, cost more memory
// requests than the copy itself); the list starts and slot starts of the run's windows are fetched
// one per lane, every entry picks its window from those registers, then all reads of the temporary
// array are issued together.
// More than 256 windows in a wave's run (lists of under four entries on average): binary search per entry.
constexpr int PACK_WPL = 4;  // windows per lane held in registers

__global__ __launch_bounds__(256) void win_pack_kernel(int n_windows, const int *__restrict__ row_ptr, int blk_h,
                                                       const int *__restrict__ win_col_ptr,
                                                       const int *__restrict__ pack_win,
                                                       const int *__restrict__ tmp_cols,
                                                       int *__restrict__ win_cols)
{
    constexpr int STEPS = PACK_PER_WAVE / 64;
    const int lane = threadIdx.x & 63;
    const int64_t run = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    const int total = win_col_ptr[n_windows];
    if (run * PACK_PER_WAVE >= total) return;  // the whole wave (the grid is sized for the capacity of win_cols)
    const int o_first = static_cast<int>(run) * PACK_PER_WAVE;
    const int n_here = total - o_first < PACK_PER_WAVE ? total - o_first : PACK_PER_WAVE;  // entries of this run
    // pack_win[run + 1] is the window of the next run's first entry, or the last window
    const int w_lo = pack_win[run], w_hi = pack_win[run + 1], n_win = w_hi - w_lo + 1;
    int src[STEPS];
    if (n_win <= 64 * PACK_WPL) {
        int begin_l[PACK_WPL], first_l[PACK_WPL];  // of window w_lo + 64 q + lane
#pragma unroll
        for (int q = 0; q < PACK_WPL; ++q) {
            const bool in = q * 64 + lane < n_win;
            begin_l[q] = in ? win_col_ptr[w_lo + q * 64 + lane] : INT32_MAX;
            first_l[q] = in ? row_ptr[(w_lo + q * 64 + lane) * blk_h] : 0;
        }
        int begin[STEPS], first[STEPS];
#pragma unroll
        for (int j = 0; j < STEPS; ++j) { begin[j] = 0; first[j] = 0; }
#pragma unroll
        for (int q = 0; q < PACK_WPL; ++q) {
            const int n_q = n_win - q * 64 < 64 ? n_win - q * 64 : 64;
            for (int t = 0; t < n_q; ++t) {  // list starts are non-decreasing: the last window that starts at or before the entry
                const int bt = __builtin_amdgcn_readlane(begin_l[q], t), ft = __builtin_amdgcn_readlane(first_l[q], t);
#pragma unroll
                for (int j = 0; j < STEPS; ++j) {
                    if (j * 64 + lane >= bt - o_first) { begin[j] = bt; first[j] = ft; }  // entry o_first + 64 j + lane
                }
            }
        }
#pragma unroll
        for (int j = 0; j < STEPS; ++j) {
            const int rel = j * 64 + lane;
            src[j] = rel < n_here ? first[j] + (o_first - begin[j]) + rel : -1;
        }
    } else {
        int w = w_lo;
        int w_begin = win_col_ptr[w], w_end = win_col_ptr[w + 1], first = row_ptr[w * blk_h];
#pragma unroll
        for (int j = 0; j < STEPS; ++j) {
            src[j] = -1;
            if (j * 64 + lane < n_here) {
                const int o = o_first + j * 64 + lane;
                if (o >= w_end) {  // the entry's window lies in (w, w_hi]
                    int a = w + 1 < w_hi ? w + 1 : w_hi, b = w_hi;
                    while (a < b) {
                        const int m = (a + b + 1) >> 1;
                        if (win_col_ptr[m] <= o) a = m;
                        else b = m - 1;
                    }
                    w = a;
                    w_begin = win_col_ptr[w];
                    w_end = win_col_ptr[w + 1];
                    first = row_ptr[w * blk_h];
                }
                src[j] = first + (o - w_begin);
            }
        }
    }
    int val[STEPS];
#pragma unroll
    for (int j = 0; j < STEPS; ++j) val[j] = src[j] >= 0 ? __builtin_nontemporal_load(tmp_cols + src[j]) : 0;  // read once
#pragma unroll
    for (int j = 0; j < STEPS; ++j)
        if (src[j] >= 0) __builtin_nontemporal_store(val[j], win_cols + o_first + j * 64 + lane);
}

// The classes of windows are condensed by different kernels, none of which depends on another and each of
// which fills only part of the GPU.  With three side streams and four events from the caller they run side
// by side after the classification: the caller's stream forks into the side streams with an event and
// joins them again before the scan.  Nothing here waits on the host and the library keeps no state.
int32_t launch_build_windows(const ftc_csr &g, ftc_windows &w, void *ws, size_t ws_bytes, const ftc_side_streams *side_in,
                             hipStream_t s)
{
    (void)ws_bytes;
    const WinWorkspace k = carve(ws, g.n, g.nnz, w.n_windows);
    if (w.n_windows == 0) {  // n == 0: only the empty prefix and the summary are written
        hipLaunchKernelGGL(win_scan_kernel, dim3(1), dim3(1024), 0, s, 0, w.blk_w, k.uniq_count, w.win_col_ptr,
                           w.block_partition, w.summary);
        return launch_status("build_windows scan");
    }
    const int hub_thr = hub_threshold(g.n, g.nnz);
    const bool direct = (static_cast<int64_t>(g.n) + (1 << WB_RANGE_LOG2) - 1) >> WB_RANGE_LOG2 <= DIRECT_MAX_RANGES;
    const bool queued = g.nnz > WAVE_CAP;  // otherwise no window can be queued
    int32_t st = FTC_OK;
    hipStream_t s_mid = s, s_large = s, s_hub = s;
    const ftc_side_streams *side = nullptr;
    // compute units of the current device: the persistent grids are multiples of it
    int n_cu = 256, dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        n_cu < 1) {
        (void)hipGetLastError();
        n_cu = 256;
    }
    if (queued) {
        hipLaunchKernelGGL(win_clear_kernel, dim3(1), dim3(64), 0, s, k.counters);
        hipLaunchKernelGGL(win_classify_kernel, dim3((w.n_windows + 1023) / 1024), dim3(1024), 0, s, g.n,
                           w.n_windows, g.row_ptr, w.blk_h, hub_thr, k.list_b[0], k.list_b[1], k.list_b[2], k.list_b[3],
                           k.list_large, k.list_hub, k.list_direct, direct ? 1 : 0, k.counters);
        st = launch_status("build_windows classify");
        if (st != FTC_OK) return st;
        side = side_in;
        if (side) {
            hipEvent_t fork = static_cast<hipEvent_t>(side->fork);
            bool good = hipEventRecord(fork, s) == hipSuccess;
            for (int i = 0; i < 3 && good; ++i)
                good = hipStreamWaitEvent(static_cast<hipStream_t>(side->stream[i]), fork, 0) == hipSuccess;
            if (!good) {
                // a side stream that did not take the dependency must not be used; the ones that did only
                // wait for work that is already queued on s
                (void)hipGetLastError();
                set_error("build_windows: cannot fork into the side streams");
                return FTC_EHIP;
            }
            s_mid = static_cast<hipStream_t>(side->stream[0]);
            s_large = static_cast<hipStream_t>(side->stream[1]);
            s_hub = static_cast<hipStream_t>(side->stream[2]);
        }
    }
    // The one-workgroup bitmap kernel is the longest chain of the build.  With side streams it stays on the caller's
    // stream and is launched first (a dependency between streams costs about 20 us before the dependent kernel
    // starts, and again at the join if the side stream is the last to finish); the wave kernel takes its place on the
    // side stream.
    hipStream_t s_wave = s;
    if (queued && g.nnz > MID_CAP && direct) {
        hipLaunchKernelGGL(win_direct_kernel, dim3(k.cap_direct < n_cu ? k.cap_direct : n_cu), dim3(1024), 0, s, g.n,
                           g.row_ptr, g.col_idx, w.blk_h, w.edge_to_row, w.edge_to_col, k.uniq_count, k.tmp_cols,
                           k.list_direct, k.counters + C_DIRECT, k.counters + C_DIRECT_NEXT);
        st = launch_status("build_windows direct bitmap (above 4096 edges)");
        if (st != FTC_OK && !side) return st;
        s_wave = s_large;
    }
    if (st == FTC_OK) {
        hipLaunchKernelGGL(win_wave_kernel, dim3(w.n_windows), dim3(64), 0, s_wave, g.n, g.row_ptr, g.col_idx, w.blk_h,
                           w.edge_to_row, w.edge_to_col, k.uniq_count, k.tmp_cols);
        st = launch_status("build_windows wave");
    }
    if (queued) {
        // persistent grids: as many workgroups as fit on the chip at once (five 256-thread or one
        // 1024-thread workgroup per CU), never more than the queue can hold
#define FTC_RANGE(NT, SLOTS, RANK, PER_CU, CAP, LIST, COUNTER, NEXT, STREAM)                                  \
    hipLaunchKernelGGL((win_compact_kernel<NT, SLOTS, RANK, PER_CU>),                                         \
                       dim3(CAP < PER_CU * n_cu ? CAP : PER_CU * n_cu), dim3(NT), 0, STREAM, g.n, g.row_ptr,  \
                       g.col_idx, w.blk_h, w.edge_to_row, w.edge_to_col, k.uniq_count, k.tmp_cols, LIST,      \
                       k.counters + COUNTER, k.counters + NEXT)
        // bitmap kernels, largest windows first; as many workgroups per CU as their LDS allows
#define FTC_WB(F, NW, PER_CU, I, COUNTER, STREAM)                                                                    \
    hipLaunchKernelGGL((win_bitmap_wave_kernel<F, NW>), dim3(k.cap_b[I] < PER_CU * n_cu ? k.cap_b[I] : PER_CU * n_cu), \
                       dim3(64 * NW), 0, STREAM, g.n, g.nnz, g.row_ptr, g.col_idx, w.blk_h, w.edge_to_row, w.edge_to_col, \
                       k.uniq_count, k.tmp_cols, k.list_b[I], k.counters + COUNTER)
        if (st == FTC_OK && g.nnz > MID_CAP && !direct) {
            FTC_WB(16384, 16, 1, 3, C_B4, s_large);
            st = launch_status("build_windows bitmap (4097 .. 16384 edges)");
        }
        if (st == FTC_OK && g.nnz > B2_CAP) {
            FTC_WB(4096, 4, 5, 2, C_B3, s_mid);
            st = launch_status("build_windows bitmap (2049 .. 4096 edges)");
        }
        if (st == FTC_OK && g.nnz > B1_CAP) {
            FTC_WB(2048, 2, 8, 1, C_B2, direct ? s_hub : s_mid);  // the hub stream is free when the direct kernel takes the hubs
            st = launch_status("build_windows bitmap (1025 .. 2048 edges)");
        }
        if (st == FTC_OK) {
            // last on the caller's stream when that stream also runs the one-workgroup kernel: the stream that
            // finishes last should be the caller's, whose wait for the side streams then costs nothing
            FTC_WB(1024, 1, 13, 0, C_B1, (direct && g.nnz > MID_CAP) ? s : s_mid);
            st = launch_status("build_windows bitmap (257 .. 1024 edges)");
        }
#undef FTC_WB
        if (st == FTC_OK && g.nnz > B4_CAP && hub_thr > B4_CAP && !direct) {
            FTC_RANGE(1024, 8192, uint32_t, 1, k.cap_large, k.list_large, C_LARGE, C_LARGE_NEXT, s_large);
            st = launch_status("build_windows compact (large)");
        }
#undef FTC_RANGE
        if (st == FTC_OK && g.nnz > hub_thr && !direct) {
            hipLaunchKernelGGL(hub_plan_kernel, dim3(1), dim3(1024), 0, s_hub, g.n, g.row_ptr, w.blk_h, k.list_hub,
                               k.counters, k.hub_chunk_ptr, k.chunk_table);
            hipLaunchKernelGGL(hub_clear_kernel, dim3(512), dim3(256), 0, s_hub, k.counters, k.hub_bits, k.wps);
            hipLaunchKernelGGL((hub_edges_kernel<false>), dim3(HUB_GRID), dim3(256), 0, s_hub, g.n, g.row_ptr,
                               g.col_idx, w.blk_h, k.list_hub, k.counters, k.hub_chunk_ptr, k.chunk_table, k.hub_bits,
                               k.hub_grp, k.wps, w.edge_to_row, w.edge_to_col, k.tmp_cols);
            hipLaunchKernelGGL(hub_scan_kernel, dim3(k.slots), dim3(1024), 0, s_hub, k.list_hub, k.counters,
                               k.hub_bits, k.hub_grp, k.wps, k.uniq_count);
            hipLaunchKernelGGL((hub_edges_kernel<true>), dim3(HUB_GRID), dim3(256), 0, s_hub, g.n, g.row_ptr,
                               g.col_idx, w.blk_h, k.list_hub, k.counters, k.hub_chunk_ptr, k.chunk_table, k.hub_bits,
                               k.hub_grp, k.wps, w.edge_to_row, w.edge_to_col, k.tmp_cols);
            st = launch_status("build_windows hubs");
        }
        if (side) {
            // join: also after a failed launch, so that no side stream is left ahead of the caller's
            for (int i = 0; i < 3; ++i) {
                if (hipEventRecord(static_cast<hipEvent_t>(side->join[i]), static_cast<hipStream_t>(side->stream[i])) !=
                        hipSuccess ||
                    hipStreamWaitEvent(s, static_cast<hipEvent_t>(side->join[i]), 0) != hipSuccess) {
                    (void)hipGetLastError();
                    if (st == FTC_OK) {
                        set_error("build_windows: cannot join the side streams");
                        st = FTC_EHIP;
                    }
                }
            }
        }
    }
    if (st != FTC_OK) return st;
    const int chunks = ceil_div(w.n_windows, SCAN_CHUNK);
    if (chunks > 1 && chunks <= SCAN_CHUNKS_MAX && g.nnz > 0) {
        hipLaunchKernelGGL(win_chunk_sums_kernel, dim3(chunks), dim3(256), 0, s, w.n_windows, w.blk_w, k.uniq_count,
                           k.chunk_uniq, k.chunk_blocks);
        hipLaunchKernelGGL(win_chunk_scan_kernel, dim3(chunks), dim3(256), 0, s, w.n_windows, w.blk_w, k.uniq_count,
                           k.chunk_uniq, k.chunk_blocks, w.win_col_ptr, w.block_partition, w.summary, k.pack_win);
        st = launch_status("build_windows scan (chunks)");
        if (st != FTC_OK) return st;
    } else {
        hipLaunchKernelGGL(win_scan_kernel, dim3(1), dim3(1024), 0, s, w.n_windows, w.blk_w, k.uniq_count,
                           w.win_col_ptr, w.block_partition, w.summary);
        st = launch_status("build_windows scan");
        if (st != FTC_OK) return st;
        if (g.nnz == 0) return FTC_OK;
        hipLaunchKernelGGL(win_pack_plan_kernel, dim3((w.n_windows + 255) / 256), dim3(256), 0, s, w.n_windows, w.win_col_ptr,
                           k.pack_win);
    }
    hipLaunchKernelGGL(win_pack_kernel, dim3(ceil_div(g.nnz, 4 * PACK_PER_WAVE)), dim3(256), 0, s,
                       w.n_windows, g.row_ptr, w.blk_h, w.win_col_ptr, k.pack_win, k.tmp_cols, w.win_cols);
    return launch_status("build_windows pack");
}

}  // namespace ftc
