// Sparse Graph Translation on the GPU (Algorithm 1 and section 4.1 of the paper) and the
// execution plan derived from it.
//
// The paper notes that row windows are independent, so each window is translated by one
// workgroup.  Size classes by the number of stored entries, all producing the same canonical result
// (ascending unique column list, rank of every edge's column in it):
//   up to 1024 entries   (five classes: 64, 128, 256, 512, 1024) a bitonic sorting network held in
//                        registers, 64 to 256 threads; the keys carry the entry's position, so ranks are
//                        scattered straight to edge_to_col
//   above               a bitmap over the column space -- in LDS when it fits (up to about 1.12 M
//                        columns), else in device scratch (then a class of up to 4096 entries is still
//                        sorted): set a bit per edge, prefix-popcount the words, rank = prefix + popcount
//                        below.  Hub windows of power-law graphs land here; the cost is
//                        O(n_cols / 32 + nnz_w) per window, and in LDS a window of more than kHubEntries
//                        entries is shared by up to kHubMaxParts workgroups.
// Every window writes its unique list at its own edge offset of col_to_row (the list is never longer than
// the window's edge range) and it stays there: the kernels that use it find it through row_ptr, and only
// the export packs the lists back to back.
//
// Host side: one stream synchronisation per build (see sgt_build_impl) and three arena allocations;
// everything else is enqueued back to back.
#include "common.h"

#include <limits.h>

#include <algorithm>
#include <mutex>

namespace tcg {

namespace {

__device__ __forceinline__ int wave_inclusive_scan(int v)
{
    const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        int t = __shfl_up(v, off, kWave);
        if (lane >= off) v += t;
    }
    return v;
}

// Exclusive prefix over one int per thread of the block.  tmp: LDS, blockDim.x / 64 + 1 ints.
// Every thread of the block must call it.  *total receives the block-wide sum.
__device__ __forceinline__ int block_exclusive_scan(int v, int *tmp, int *total)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wid = threadIdx.x >> 6;
    const int nw = (blockDim.x + kWave - 1) >> 6;
    int incl = wave_inclusive_scan(v);
    if (lane == kWave - 1) tmp[wid] = incl;
    __syncthreads();
    if (wid == 0) {
        int t = lane < nw ? tmp[lane] : 0;
        int s = wave_inclusive_scan(t);
        if (lane < nw) tmp[lane] = s - t;
        if (lane == nw - 1) tmp[nw] = s;
    }
    __syncthreads();
    int res = tmp[wid] + incl - v;
    *total = tmp[nw];
    __syncthreads();
    return res;
}

// ---- device-wide exclusive scan ------------------------------------------------------------------
// Three steps: per-block sums of 4096-element blocks, a single-workgroup scan of those sums, and a
// per-block rescan with the block's offset.  Inputs of up to 4096 elements take the single-workgroup
// kernel alone.

constexpr int kScanThreads = 256;
constexpr int kScanItems = 16;
constexpr int kScanBlock = kScanThreads * kScanItems;

__global__ __launch_bounds__(1024) void scan_single_kernel(const int32_t *in, int32_t *out, int64_t n)
{
    __shared__ int tmp[1024 / kWave + 1];
    int carry = 0;
    for (int64_t base = 0; base < n; base += 1024 * 4) {
        int64_t i0 = base + (int64_t)threadIdx.x * 4;
        int v[4];
        int sum = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            v[k] = (i0 + k < n) ? in[i0 + k] : 0;
            sum += v[k];
        }
        int total;
        int run = carry + block_exclusive_scan(sum, tmp, &total);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (i0 + k < n) out[i0 + k] = run;
            run += v[k];
        }
        carry += total;
    }
    if (threadIdx.x == 0) out[n] = carry;
}

__global__ __launch_bounds__(kScanThreads) void scan_block_sum_kernel(const int32_t *in, int64_t n,
                                                                      int32_t *block_sums)
{
    __shared__ int tmp[kScanThreads / kWave + 1];
    const int64_t i0 = (int64_t)blockIdx.x * kScanBlock + (int64_t)threadIdx.x * kScanItems;
    int sum = 0;
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) sum += (i0 + k < n) ? in[i0 + k] : 0;
    int total;
    (void)block_exclusive_scan(sum, tmp, &total);
    if (threadIdx.x == 0) block_sums[blockIdx.x] = total;
}

__global__ __launch_bounds__(kScanThreads) void scan_apply_kernel(const int32_t *in, int32_t *out, int64_t n,
                                                                  const int32_t *block_offs, int64_t n_blocks)
{
    __shared__ int tmp[kScanThreads / kWave + 1];
    const int64_t i0 = (int64_t)blockIdx.x * kScanBlock + (int64_t)threadIdx.x * kScanItems;
    int v[kScanItems];
    int sum = 0;
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) {
        v[k] = (i0 + k < n) ? in[i0 + k] : 0;
        sum += v[k];
    }
    int total;
    int run = block_offs[blockIdx.x] + block_exclusive_scan(sum, tmp, &total);
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) {
        if (i0 + k < n) out[i0 + k] = run;
        run += v[k];
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) out[n] = block_offs[n_blocks];
}

// ---- CSR validation ------------------------------------------------------------------------------
// flag bit 0 = row_ptr ends wrong, bit 1 = not monotone, bit 2 = column out of range.
__global__ void validate_csr_kernel(int32_t n_rows, int64_t nnz, const int32_t *rp, int *flag)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    int bad = 0;
    if (i == 0 && (rp[0] != 0 || (int64_t)rp[n_rows] != nnz)) bad |= 1;
    for (int64_t r = i; r < n_rows; r += stride)
        if (rp[r] > rp[r + 1] || rp[r] < 0) bad |= 2;
    if (bad) atomicOr(flag, bad);
}

__global__ void validate_cols_kernel(int32_t n_cols, int64_t nnz, const int32_t *ci, int *flag)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    int bad = 0;
    for (int64_t e = i; e < nnz; e += stride)
        if (ci[e] < 0 || ci[e] >= n_cols) bad = 4;
    if (bad) atomicOr(flag, bad);
}

__device__ __forceinline__ void window_edge_range(const int32_t *rp, int32_t n_rows, int32_t win_h,
                                                  int64_t w, int32_t *lo, int32_t *hi)
{
    int64_t r0 = w * win_h;
    int64_t r1 = r0 + win_h;
    if (r1 > n_rows) r1 = n_rows;
    *lo = rp[r0];
    *hi = rp[r1];
}

// ---- size classes and the per-build block of small results ---------------------------------------
// A window's class follows its number of stored entries: seven classes of the register sorting network
// (<= 64, 128, ..., 4096 entries) and the bitmap class above.
constexpr int kClsLarge = 7, kClasses = 8;
constexpr int kSortCap = 4096;            // largest window that is sorted
constexpr int kLdsBitmapFrom = 1024;      // ... when the bitmap class works in LDS
constexpr int kHubEntries = 16384;        // LDS bitmap class: a window with more entries is listed in several parts,
constexpr int kHubMaxParts = 8;
constexpr int kSlotSharers = 8;                     // workgroups per row block in seg_fill_kernel's first phase (large graphs)
constexpr int64_t kForkMinEntries = 1 << 20;       // a translation of fewer entries runs on one stream           // one per kHubEntries entries up to this many (see the kernel)

__device__ __forceinline__ int window_class(int32_t cnt, int32_t sort_cap)
{
    if (cnt > sort_cap) return kClsLarge;
    if (cnt <= 64) return 0;
    if (cnt <= 128) return 1;
    if (cnt <= 256) return 2;
    if (cnt <= 512) return 3;
    if (cnt <= 1024) return 4;
    if (cnt <= 2048) return 5;
    return 6;
}

// Everything the host needs from a build sits in one device block that is copied once, at the end.
struct BuildInfo {
    int32_t cls_count[8];                       // windows per size class
    int32_t ticket;                             // work counter of the bitmap-class kernel
    int32_t n_seg, n_long, n_slots;             // gather plan sizes
    int32_t sort_tail;                          // single-segment rows ordered by length class
    int32_t flag;                               // CSR validation
    int32_t total_unique;
    int32_t n_gchunks;                          // kGiantChunk-entry pieces of the rows beyond kGiantRow entries
    int32_t lane_tab[kLaneTabStride * kXcds];   // see plan_segment()
    unsigned long long counters[8];             // choose_path_kernel totals
};

// ---- gather plan, step 1: per-row-block counts; window classification ----------------------------
// Rows are handled in blocks of kRowBlock (four rounds of 256 threads; row = block * kRowBlock + round * 256
// + thread).  Every row is cut into segments of at most kSegLen entries.  Per block: the number of split
// rows (more than one segment), the number of their segments, and the number of single-segment rows in
// each length class.  The same launch appends every non-empty window to the list of its size class
// (order inside a list is irrelevant: a window's result depends on the window only).
constexpr int kRowBlock = 1024;
constexpr int kTailClasses = 8;
constexpr int kPlanSums = 2 + kTailClasses;

// Length classes of single-segment rows follow the number of gather iterations a row needs (longest
// first), so that the lane groups of a wavefront get rows of similar length.
__device__ __forceinline__ int length_class(int32_t deg)
{
    return deg > 96 ? 0 : deg > 64 ? 1 : deg > 48 ? 2 : deg > 32 ? 3 : deg > 24 ? 4 : deg > 16 ? 5 : deg > 8 ? 6 : 7;
}

__global__ __launch_bounds__(256) void prep_kernel(int32_t n_rows, int32_t win_h, int64_t n_win,
                                                   const int32_t *__restrict__ rp, int64_t nb_rows,
                                                   int32_t *__restrict__ block_sums, int32_t *__restrict__ lists,
                                                   int32_t *cls_count, int32_t *__restrict__ win_unique, int32_t sort_cap,
                                                   int32_t *__restrict__ large_part, int32_t hub_entries, int32_t slot_len)
{
    const int lane = threadIdx.x & (kWave - 1);
    if ((int64_t)blockIdx.x < nb_rows) {
        __shared__ int s_sum[kPlanSums];
        if (threadIdx.x < kPlanSums) s_sum[threadIdx.x] = 0;
        __syncthreads();
        int n_long = 0, n_slot = 0;
#pragma unroll
        for (int round = 0; round < kRowBlock / 256; ++round) {
            const int64_t r = (int64_t)blockIdx.x * kRowBlock + round * 256 + threadIdx.x;
            int cls = -1;
            if (r < n_rows) {
                const int32_t deg = rp[r + 1] - rp[r];
                if (deg > kSegLen) {
                    ++n_long;
                    n_slot += (deg + slot_len - 1) / slot_len;
                } else {
                    cls = length_class(deg);
                }
            }
#pragma unroll
            for (int c = 0; c < kTailClasses; ++c) {
                const unsigned long long mask = __ballot(cls == c);
                if (lane == 0 && mask) atomicAdd(&s_sum[2 + c], __popcll(mask));
            }
        }
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
            n_long += __shfl_xor(n_long, off, kWave);
            n_slot += __shfl_xor(n_slot, off, kWave);
        }
        if (lane == 0 && n_long) {
            atomicAdd(&s_sum[0], n_long);
            atomicAdd(&s_sum[1], n_slot);
        }
        __syncthreads();
        if (threadIdx.x < kPlanSums) block_sums[(int64_t)threadIdx.x * nb_rows + blockIdx.x] = s_sum[threadIdx.x];
        return;
    }
    const int64_t w = ((int64_t)blockIdx.x - nb_rows) * 256 + threadIdx.x;
    int cls = -1;
    int32_t cnt = 0;
    if (w < n_win) {
        int32_t lo, hi;
        window_edge_range(rp, n_rows, win_h, w, &lo, &hi);
        cnt = hi - lo;
        if (cnt == 0) win_unique[w] = 0;
        else cls = window_class(cnt, sort_cap);
    }
    // The bitmap class is small and its list has one item per part of a window (large_part: part number, and the
    // number of parts from bit 8 up): its windows draw their places themselves.
    if (cls == kClsLarge) {
        const int parts = cnt > hub_entries ? min(kHubMaxParts, (cnt + hub_entries - 1) / hub_entries) : 1;
        const int at = atomicAdd(&cls_count[kClsLarge], parts);
        for (int j = 0; j < parts; ++j) {
            lists[(int64_t)kClsLarge * n_win + at + j] = (int32_t)w;
            large_part[at + j] = j | (parts << 8);
        }
        cls = -1;
    }
    // One atomic per workgroup and class instead of one per window: the wavefronts count their windows of
    // every class with ballots, one thread per class draws the workgroup's range of the list (all classes in
    // one round trip), and every window takes its place inside it.
    __shared__ int s_wave_cnt[256 / kWave][kClasses];
    __shared__ int s_base[kClasses];
    const int wave = threadIdx.x >> 6;
    int rank_in_wave = 0;
#pragma unroll
    for (int c = 0; c < kClsLarge; ++c) {
        const unsigned long long mask = __ballot(cls == c);
        if (lane == 0) s_wave_cnt[wave][c] = __popcll(mask);
        if (cls == c) rank_in_wave = __popcll(mask & ((1ull << lane) - 1ull));
    }
    __syncthreads();
    if (threadIdx.x < kClsLarge) {
        int t = 0;
#pragma unroll
        for (int w2 = 0; w2 < 256 / kWave; ++w2) t += s_wave_cnt[w2][threadIdx.x];
        s_base[threadIdx.x] = t ? atomicAdd(&cls_count[threadIdx.x], t) : 0;
    }
    __syncthreads();
    if (cls >= 0) {
        int p = s_base[cls] + rank_in_wave;
        for (int w2 = 0; w2 < wave; ++w2) p += s_wave_cnt[w2][cls];
        lists[(int64_t)cls * n_win + p] = (int32_t)w;
    }
}

// ---- ordinary windows: sorting network in registers ---------------------------------------------
// One workgroup of THREADS threads per window of at most N = THREADS * KPT entries; the workgroups walk
// their class list with a grid stride (the list's length is only known on the device).  Every entry
// becomes one key (column << pos_bits) | position-in-window, so the sorted keys carry the edge each
// column came from: no lookup by binary search afterwards, the rank is scattered straight to
// edge_to_col.  Thread t holds the KPT network slots t * KPT .. t * KPT + KPT - 1 in registers.  A
// compare-exchange at distance j stays inside a thread for j < KPT, is a lane exchange inside the
// wavefront for j < 64 * KPT, and only goes through LDS (one round trip) beyond that -- three of the 55
// stages of a 1024-entry window.  K is uint32_t when column and position fit 31 bits, uint64_t otherwise.
template <typename K>
__device__ __forceinline__ K lane_xor(K v, int mask)
{
    if constexpr (sizeof(K) == 4) {
        return (K)__shfl_xor((int)v, mask, kWave);
    } else {
        const int lo = __shfl_xor((int)(uint32_t)v, mask, kWave);
        const int hi = __shfl_xor((int)(uint32_t)(v >> 32), mask, kWave);
        return ((K)(uint32_t)hi << 32) | (uint32_t)lo;
    }
}

template <typename K>
__device__ __forceinline__ K lane_up1(K v)
{
    if constexpr (sizeof(K) == 4) {
        return (K)__shfl_up((int)v, 1, kWave);
    } else {
        const int lo = __shfl_up((int)(uint32_t)v, 1, kWave);
        const int hi = __shfl_up((int)(uint32_t)(v >> 32), 1, kWave);
        return ((K)(uint32_t)hi << 32) | (uint32_t)lo;
    }
}

template <int THREADS, int KPT, typename K>
__device__ __forceinline__ void sort_windows(
    int64_t first, int64_t stride, int32_t n_rows, int32_t win_h, const int32_t *__restrict__ win_list,
    const int32_t *__restrict__ list_len, const int32_t *__restrict__ rp, const int32_t *__restrict__ ci,
    int32_t *__restrict__ edge_to_col, int32_t *__restrict__ col_to_row, int32_t *__restrict__ win_unique)
{
    constexpr int N = THREADS * KPT;
    constexpr int WAVES = THREADS / kWave;
    __shared__ K s_x[WAVES > 1 ? N : 1];
    __shared__ K s_last[WAVES];
    __shared__ int s_tmp[WAVES + 1];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
    const int32_t n_items = *list_len;
    int pos_bits = 0;
    while ((1 << pos_bits) < N) ++pos_bits;
    const K pos_mask = ((K)1 << pos_bits) - 1;

    for (int64_t item = first; item < n_items; item += stride) {
        const int64_t w = win_list[item];
        int32_t lo, hi;
        window_edge_range(rp, n_rows, win_h, w, &lo, &hi);
        const int cnt = hi - lo;          // 1 <= cnt <= N by classification

        // Coalesced loads: entry r * THREADS + t goes to slot t * KPT + r (any assignment will do, the
        // key remembers where the entry came from); empty slots get the largest key and sort last.
        K key[KPT];
#pragma unroll
        for (int r = 0; r < KPT; ++r) {
            const int e = r * THREADS + tid;
            key[r] = e < cnt ? (((K)(uint32_t)ci[lo + e] << pos_bits) | (K)e) : ~(K)0;
        }

#pragma unroll
        for (int k = 2; k <= N; k <<= 1) {
#pragma unroll
            for (int j = k >> 1; j > 0; j >>= 1) {
                if (j < KPT) {
#pragma unroll
                    for (int a = 0; a < KPT; ++a) {
                        if (a & j) continue;
                        const int b = a | j;
                        const bool asc = ((tid * KPT + a) & k) == 0;
                        const K x = key[a], y = key[b];
                        const bool sw = (x > y) == asc;
                        key[a] = sw ? y : x;
                        key[b] = sw ? x : y;
                    }
                } else if (j < KPT * kWave) {
                    const int lm = j / KPT;
                    const bool lower = (lane & lm) == 0;
#pragma unroll
                    for (int r = 0; r < KPT; ++r) {
                        const K other = lane_xor(key[r], lm);
                        const bool asc = ((tid * KPT + r) & k) == 0;
                        const K mn = key[r] < other ? key[r] : other;
                        const K mx = key[r] < other ? other : key[r];
                        key[r] = (lower == asc) ? mn : mx;
                    }
                } else {
                    const int pt = tid ^ (j / KPT);
                    const bool lower = (tid & (j / KPT)) == 0;
#pragma unroll
                    for (int r = 0; r < KPT; ++r) s_x[r * THREADS + tid] = key[r];
                    __syncthreads();
#pragma unroll
                    for (int r = 0; r < KPT; ++r) {
                        const K other = s_x[r * THREADS + pt];
                        const bool asc = ((tid * KPT + r) & k) == 0;
                        const K mn = key[r] < other ? key[r] : other;
                        const K mx = key[r] < other ? other : key[r];
                        key[r] = (lower == asc) ? mn : mx;
                    }
                    __syncthreads();
                }
            }
        }

        // Slot i now holds the i-th smallest key; slots cnt .. N-1 hold the filler.  A slot is the head
        // of a run of equal columns when the slot before it has another column.
        K prev = lane_up1(key[KPT - 1]);
        if (WAVES > 1) {
            if (lane == kWave - 1) s_last[wave] = key[KPT - 1];
            __syncthreads();
            if (lane == 0 && wave > 0) prev = s_last[wave - 1];
        }
        bool head[KPT];
        int local = 0;
#pragma unroll
        for (int r = 0; r < KPT; ++r) {
            const int i = tid * KPT + r;
            const K before = r == 0 ? prev : key[r - 1];
            head[r] = i < cnt && (i == 0 || (key[r] >> pos_bits) != (before >> pos_bits));
            local += head[r] ? 1 : 0;
        }
        int run, total;
        if (WAVES > 1) {
            run = block_exclusive_scan(local, s_tmp, &total);
        } else {
            const int incl = wave_inclusive_scan(local);
            run = incl - local;
            total = __shfl(incl, kWave - 1, kWave);
        }
#pragma unroll
        for (int r = 0; r < KPT; ++r) {
            const int i = tid * KPT + r;
            if (head[r]) {
                col_to_row[lo + run] = (int32_t)(key[r] >> pos_bits);
                ++run;
            }
            if (i < cnt) edge_to_col[lo + (int32_t)(key[r] & pos_mask)] = run - 1;
        }
        if (tid == 0) win_unique[w] = total;
    }
}

template <int THREADS, int KPT, typename K>
__global__ __launch_bounds__(THREADS) void sgt_window_sort_kernel(
    int32_t n_rows, int32_t win_h, const int32_t *__restrict__ win_list, const int32_t *__restrict__ list_len,
    const int32_t *__restrict__ rp, const int32_t *__restrict__ ci, int32_t *__restrict__ edge_to_col,
    int32_t *__restrict__ col_to_row, int32_t *__restrict__ win_unique)
{
    sort_windows<THREADS, KPT, K>(blockIdx.x, gridDim.x, n_rows, win_h, win_list, list_len, rp, ci, edge_to_col,
                                  col_to_row, win_unique);
}

// The three one-wavefront classes (up to 64, 128, 256 entries) in one launch: workgroups 0 .. g0-1 walk the
// first class list, the next g1 the second, the rest the third (lists n_win apart, counts one apart).
template <typename K>
__global__ __launch_bounds__(kWave) void sgt_window_sort_small_kernel(
    int32_t n_rows, int32_t win_h, int64_t n_win, const int32_t *__restrict__ lists,
    const int32_t *__restrict__ cls_count, int32_t g0, int32_t g1, const int32_t *__restrict__ rp,
    const int32_t *__restrict__ ci, int32_t *__restrict__ edge_to_col, int32_t *__restrict__ col_to_row,
    int32_t *__restrict__ win_unique)
{
    const int32_t b = blockIdx.x, g2 = gridDim.x - g0 - g1;
    if (b < g0)
        sort_windows<kWave, 1, K>(b, g0, n_rows, win_h, lists, cls_count, rp, ci, edge_to_col, col_to_row, win_unique);
    else if (b < g0 + g1)
        sort_windows<kWave, 2, K>(b - g0, g1, n_rows, win_h, lists + n_win, cls_count + 1, rp, ci, edge_to_col,
                                  col_to_row, win_unique);
    else
        sort_windows<kWave, 4, K>(b - g0 - g1, g2, n_rows, win_h, lists + 2 * n_win, cls_count + 2, rp, ci, edge_to_col,
                                  col_to_row, win_unique);
}

// Large class: bitmap over the column space, one workgroup per window.  `bitmap` must be zero on
// entry; `prefix` is plain scratch; both hold n_words entries per workgroup.  The words are split
// into one contiguous range per wavefront, so every pass over them is coalesced and only one
// workgroup-wide scan (of the 16 wavefront totals) is needed.
constexpr int kBitmapThreads = 1024;
constexpr int kBitmapWaves = kBitmapThreads / kWave;
constexpr int kEdgeUnroll = 4;

__global__ __launch_bounds__(kBitmapThreads) void sgt_window_bitmap_kernel(
    int32_t n_rows, int32_t win_h, int64_t n_words, const int32_t *__restrict__ large_list,
    const int32_t *__restrict__ rp, const int32_t *__restrict__ ci, uint32_t *bitmap, int32_t *prefix,
    int32_t *__restrict__ edge_to_col, int32_t *__restrict__ tmp_clean, int32_t *__restrict__ win_unique)
{
    __shared__ int s_tmp[kBitmapWaves + 1];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int64_t w = large_list[blockIdx.x];
    uint32_t *bm = bitmap + (int64_t)blockIdx.x * n_words;
    int32_t *pf = prefix + (int64_t)blockIdx.x * n_words;
    int32_t lo, hi;
    window_edge_range(rp, n_rows, win_h, w, &lo, &hi);

    // 1. one bit per edge
    for (int64_t e0 = lo + threadIdx.x; e0 < hi; e0 += (int64_t)kBitmapThreads * kEdgeUnroll) {
        uint32_t c[kEdgeUnroll];
#pragma unroll
        for (int u = 0; u < kEdgeUnroll; ++u) {
            int64_t e = e0 + (int64_t)u * kBitmapThreads;
            c[u] = e < hi ? (uint32_t)ci[e] : 0xFFFFFFFFu;
        }
#pragma unroll
        for (int u = 0; u < kEdgeUnroll; ++u)
            if (c[u] != 0xFFFFFFFFu) atomicOr(&bm[c[u] >> 5], 1u << (c[u] & 31));
    }
    // The barrier (with its workgroup-scope fence) orders the workgroup's atomics before the reads
    // below; all waves of a workgroup share one CU cache and nobody read the bitmap earlier in this
    // kernel, so no stale copy can exist.  Device-scope fences are not needed (and cost an L2
    // write-back each).
    __syncthreads();

    // 2. per-wavefront popcount of its word range, then the offsets of the wavefronts
    int64_t wpw = (n_words + kBitmapWaves - 1) / kBitmapWaves;
    wpw = (wpw + kWave - 1) / kWave * kWave;
    int64_t k_begin = (int64_t)wave * wpw;
    if (k_begin > n_words) k_begin = n_words;
    int64_t k_end = k_begin + wpw;
    if (k_end > n_words) k_end = n_words;
    int cnt = 0;
    for (int64_t k = k_begin + lane; k < k_end; k += kWave) cnt += __popc(bm[k]);
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) cnt += __shfl_xor(cnt, off, kWave);
    int total;
    int wave_off = block_exclusive_scan(lane == 0 ? cnt : 0, s_tmp, &total);
    wave_off = __shfl(wave_off, 0, kWave);

    // 3. prefix of every word, and the unique list itself (bit positions in ascending order)
    int carry = wave_off;
    for (int64_t k0 = k_begin; k0 < k_end; k0 += kWave) {
        const int64_t k = k0 + lane;
        uint32_t bits = k < k_end ? bm[k] : 0u;
        const int p = __popc(bits);
        const int incl = wave_inclusive_scan(p);
        int pos = carry + incl - p;
        if (k < k_end) pf[k] = pos;
        while (bits) {
            int b = __ffs(bits) - 1;
            bits &= bits - 1;
            tmp_clean[lo + pos] = (int32_t)(k * 32 + b);
            ++pos;
        }
        carry += __shfl(incl, kWave - 1, kWave);
    }
    if (threadIdx.x == 0) win_unique[w] = total;
    __syncthreads();

    // 4. rank of every edge's column
    for (int64_t e0 = lo + threadIdx.x; e0 < hi; e0 += (int64_t)kBitmapThreads * kEdgeUnroll) {
        uint32_t c[kEdgeUnroll], bits[kEdgeUnroll];
        int32_t base[kEdgeUnroll];
#pragma unroll
        for (int u = 0; u < kEdgeUnroll; ++u) {
            int64_t e = e0 + (int64_t)u * kBitmapThreads;
            c[u] = e < hi ? (uint32_t)ci[e] : 0u;
        }
#pragma unroll
        for (int u = 0; u < kEdgeUnroll; ++u) {
            bits[u] = bm[c[u] >> 5];
            base[u] = pf[c[u] >> 5];
        }
#pragma unroll
        for (int u = 0; u < kEdgeUnroll; ++u) {
            int64_t e = e0 + (int64_t)u * kBitmapThreads;
            if (e < hi) edge_to_col[e] = base[u] + __popc(bits[u] & ((1u << (c[u] & 31)) - 1u));
        }
    }
}

// Bitmap class when the column space fits in LDS (gfx950 gives a workgroup up to 160 KB): one bit per
// column plus the running count in front of every group of kPfGroup words.  Setting the bits and looking
// the ranks up are LDS operations instead of L2 atomics and gathers, and no device scratch has to be
// cleared.  Needs lds_bitmap_bytes(n_words) <= kLdsBitmapMax.  One workgroup fills a compute unit's LDS, so
// the kernel is launched with one workgroup per compute unit and the workgroups draw windows from a counter
// until the class list is used up (hub windows differ in size by two orders of magnitude; the counter keeps
// everybody busy).  The loop is software-pipelined against the chain of dependent round trips that opens a
// window (counter -> list -> row_ptr -> columns): the counter is drawn at the start of the window before,
// the window's id and range are fetched by one thread in two separate phases of that window, and its first
// batch of columns is requested before the ranks of the current window are written.  The edge loops keep
// kLdsEdgeUnroll column loads per thread in flight: a hub window of a power-law graph has 10^5 entries, and
// one load per thread and round trip would make it the critical path of the whole translation.
constexpr int kPfGroup = 8;
constexpr size_t kLdsBitmapMax = 160 * 1024 - 256;
constexpr int kLdsEdgeUnroll = 16;
inline size_t lds_bitmap_bytes(int64_t n_words)
{
    return (size_t)(n_words + (n_words + kPfGroup - 1) / kPfGroup + 1) * 4;
}

__global__ __launch_bounds__(kBitmapThreads) void sgt_window_lds_bitmap_kernel(
    int32_t n_rows, int32_t win_h, int32_t n_words, const int32_t *__restrict__ large_list,
    const int32_t *__restrict__ large_part, const int32_t *__restrict__ list_len, int32_t *ticket,
    const int32_t *__restrict__ rp,
    const int32_t *__restrict__ ci, int32_t *__restrict__ edge_to_col, int32_t *__restrict__ col_to_row,
    int32_t *__restrict__ win_unique)
{
    extern __shared__ uint32_t s_words[];          // bitmap, then the group prefixes
    __shared__ int s_tmp[kBitmapWaves + 1];
    __shared__ int32_t s_next[5];                  // next item: list position, window id, edge range, part
    uint32_t *bm = s_words;
    int32_t *gpf = reinterpret_cast<int32_t *>(s_words + n_words);
    const int32_t n_items = *list_len;
    constexpr int64_t kStep = (int64_t)kBitmapThreads * kLdsEdgeUnroll;
    // every thread owns a contiguous run of R words (R odd: the lanes of a wavefront then read different
    // banks), so that the owners' bit counts are in column order
    const int32_t R = ((n_words + kBitmapThreads - 1) / kBitmapThreads) | 1;
    const int32_t kb = min((int32_t)threadIdx.x * R, n_words), ke = min(kb + R, n_words);

    if (threadIdx.x == 0) {
        const int32_t it = atomicAdd(ticket, 1);
        int32_t w = 0, lo = 0, hi = 0, pp = 1 << 8;
        if (it < n_items) {
            w = large_list[it];
            pp = large_part[it];
            window_edge_range(rp, n_rows, win_h, w, &lo, &hi);
        }
        s_next[0] = it;
        s_next[1] = w;
        s_next[2] = lo;
        s_next[3] = hi;
        s_next[4] = pp;
    }
    __syncthreads();
    int32_t item = s_next[0], w = s_next[1], lo = s_next[2], hi = s_next[3], pp = s_next[4];
    uint32_t c_first[kLdsEdgeUnroll];
#pragma unroll
    for (int u = 0; u < kLdsEdgeUnroll; ++u) {
        const int64_t e = (int64_t)lo + threadIdx.x + (int64_t)u * kBitmapThreads;
        c_first[u] = e < hi ? (uint32_t)ci[e] : 0xFFFFFFFFu;
    }

    while (item < n_items) {                       // the same value in every thread: all leave together
        int32_t next_item = 0, next_w = 0, next_pp = 1 << 8;
        if (threadIdx.x == 0) next_item = atomicAdd(ticket, 1);
        for (int32_t k = threadIdx.x; k < n_words; k += kBitmapThreads) bm[k] = 0u;
        __syncthreads();                           // also: everybody has read s_next

        // 1. one bit per edge
#pragma unroll
        for (int u = 0; u < kLdsEdgeUnroll; ++u)
            if (c_first[u] != 0xFFFFFFFFu) atomicOr(&bm[c_first[u] >> 5], 1u << (c_first[u] & 31));
        for (int64_t e0 = (int64_t)lo + kStep + threadIdx.x; e0 < hi; e0 += kStep) {
            uint32_t c[kLdsEdgeUnroll];
#pragma unroll
            for (int u = 0; u < kLdsEdgeUnroll; ++u) {
                const int64_t e = e0 + (int64_t)u * kBitmapThreads;
                c[u] = e < hi ? (uint32_t)ci[e] : 0xFFFFFFFFu;
            }
#pragma unroll
            for (int u = 0; u < kLdsEdgeUnroll; ++u)
                if (c[u] != 0xFFFFFFFFu) atomicOr(&bm[c[u] >> 5], 1u << (c[u] & 31));
        }
        if (threadIdx.x == 0 && next_item < n_items) {                                 // used two phases on
            next_w = large_list[next_item];
            next_pp = large_part[next_item];
        }
        __syncthreads();

        // 2. bits in the words this thread owns; one workgroup-wide scan gives the count in front of them.
        //    (A scan per 64 words instead costs a chain of cross-lane steps per row.)
        int cnt = 0;
        for (int32_t k = kb; k < ke; ++k) cnt += __popc(bm[k]);
        int total;
        int pos = block_exclusive_scan(cnt, s_tmp, &total);
        int32_t next_lo = 0, next_hi = 0;
        if (threadIdx.x == 0 && next_item < n_items) window_edge_range(rp, n_rows, win_h, next_w, &next_lo, &next_hi);

        // 3. the count in front of every group of words
        for (int32_t k = kb; k < ke; ++k) {
            if ((k % kPfGroup) == 0) gpf[k / kPfGroup] = pos;
            pos += __popc(bm[k]);
        }
        if (threadIdx.x == 0) {
            win_unique[w] = total;
            s_next[0] = next_item;
            s_next[1] = next_w;
            s_next[2] = next_lo;
            s_next[3] = next_hi;
            s_next[4] = next_pp;
        }
        __syncthreads();

        // The next window's first batch of columns is requested now; it arrives while the ranks are written.
        const int32_t n_item = s_next[0], n_w = s_next[1], n_lo = s_next[2], n_hi = s_next[3], n_pp = s_next[4];
        uint32_t c_next[kLdsEdgeUnroll];
#pragma unroll
        for (int u = 0; u < kLdsEdgeUnroll; ++u) {
            const int64_t e = (int64_t)n_lo + threadIdx.x + (int64_t)u * kBitmapThreads;
            c_next[u] = e < n_hi ? (uint32_t)ci[e] : 0xFFFFFFFFu;
        }

        // 4. rank of every edge's column: group prefix + the words of the group in front of it + the bits below
        auto rank_of = [&](uint32_t c) {
            const int32_t wi = (int32_t)(c >> 5);
            const int32_t g0 = wi / kPfGroup * kPfGroup;
            int r = gpf[wi / kPfGroup] + __popc(bm[wi] & ((1u << (c & 31)) - 1u));
#pragma unroll
            for (int j = 0; j < kPfGroup - 1; ++j)
                if (g0 + j < wi) r += __popc(bm[g0 + j]);
            return r;
        };
        // The rank of an edge's column is also that column's place in the window's unique list, so the list is
        // written from here: every entry of a column stores the same value at the same place, and the entries
        // of a sorted row have rising, mostly neighbouring ranks, so these stores coalesce.  (Walking the
        // bitmap and writing each word's columns from the thread that owns the word serialises a hub window's
        // 10^5 stores in a few wavefronts.)
        // A window listed in several parts: every part has built the whole bitmap (the bits are the cheaper
        // half, and every part needs all of them) and ranks its share of the entries; every column occurs in
        // some entry, so the parts together write the whole unique list.
        const int32_t part = pp & 255, n_parts = pp >> 8;
        int64_t r_lo = lo, r_hi = hi;
        if (n_parts == 1) {
#pragma unroll
            for (int u = 0; u < kLdsEdgeUnroll; ++u)
                if (c_first[u] != 0xFFFFFFFFu) {
                    const int r = rank_of(c_first[u]);
                    edge_to_col[(int64_t)lo + threadIdx.x + (int64_t)u * kBitmapThreads] = r;
                    col_to_row[lo + r] = (int32_t)c_first[u];
                }
            r_lo = (int64_t)lo + kStep;
        } else {
            const int64_t len = (int64_t)hi - lo;
            r_lo = lo + len * part / n_parts;
            r_hi = lo + len * (part + 1) / n_parts;
        }
        for (int64_t e0 = r_lo + threadIdx.x; e0 < r_hi; e0 += kStep) {
            uint32_t c[kLdsEdgeUnroll];
#pragma unroll
            for (int u = 0; u < kLdsEdgeUnroll; ++u) {
                const int64_t e = e0 + (int64_t)u * kBitmapThreads;
                c[u] = e < r_hi ? (uint32_t)ci[e] : 0xFFFFFFFFu;
            }
#pragma unroll
            for (int u = 0; u < kLdsEdgeUnroll; ++u) {
                const int64_t e = e0 + (int64_t)u * kBitmapThreads;
                if (c[u] != 0xFFFFFFFFu) {
                    const int r = rank_of(c[u]);
                    edge_to_col[e] = r;
                    col_to_row[lo + r] = (int32_t)c[u];
                }
            }
        }
        item = n_item;
        w = n_w;
        lo = n_lo;
        hi = n_hi;
        pp = n_pp;
#pragma unroll
        for (int u = 0; u < kLdsEdgeUnroll; ++u) c_first[u] = c_next[u];
        __syncthreads();                           // ranks are read before the bitmap is cleared again
    }
}

// ---- per-window path choice ------------------------------------------------------------------------
__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long v)
{
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// Per window: win_partition = ceil(U_w / tile_w) (Algorithm 1), the path flag under the given policy,
// and the totals (tiles, tile-path windows, their edges) with one atomic per wavefront.
struct PathArgs {
    int32_t n_rows, win_h, tile_w;
    int policy;
    float min_reuse;
    const int32_t *rp;
    int32_t *win_partition;
    uint8_t *win_path;
    unsigned long long *counts;
};

struct PathTotals {
    unsigned long long tiles = 0, tile_win = 0, tile_nnz = 0, tile_many = 0, tile_unique = 0;
};

__device__ __forceinline__ void choose_window(const PathArgs &a, int64_t w, int32_t uw, PathTotals &t)
{
    int32_t lo, hi;
    window_edge_range(a.rp, a.n_rows, a.win_h, w, &lo, &hi);
    const int32_t nnz_w = hi - lo;
    const unsigned long long tiles = (unsigned long long)(((int64_t)uw + a.tile_w - 1) / a.tile_w);
    a.win_partition[w] = (int32_t)tiles;
    bool tile = false;
    if (a.policy == TCG_POLICY_TILE) tile = uw > 0;
    else if (a.policy == TCG_POLICY_AUTO)
        // Windows with shared neighbours, but not hub windows: the tile kernels keep a window's
        // condensed columns (or its whole condensed adjacency) in LDS, which needs compact windows.
        tile = (a.win_h == 16 || a.win_h == 32) && uw > 0 && uw <= kTileMaxUnique &&
               (float)nnz_w >= a.min_reuse * (float)uw;
    // windows of 32 rows: class kTileFew only (twice the edges of a 16-row window fit in registers)
    if (a.win_h == 32 && a.policy == TCG_POLICY_AUTO && nnz_w > 2 * kTileFewEdges) tile = false;
    const bool many = tile && a.win_h == 16 && nnz_w > kTileFewEdges && uw <= kTileMaxUnique;
    a.win_path[w] = tile ? (many ? kTileMany : kTileFew) : 0;
    t.tiles += tiles;
    if (tile) {
        t.tile_win += 1;
        t.tile_nnz += (unsigned long long)nnz_w;
        t.tile_unique += (unsigned long long)uw;
    }
    if (many) {
        t.tile_many += 1;
        atomicMax(&a.counts[4], (unsigned long long)uw);
    }
}

// Every lane of the wavefront calls it.
__device__ __forceinline__ void flush_path_totals(const PathArgs &a, const PathTotals &t)
{
    const unsigned long long tiles = wave_sum_u64(t.tiles), tile_win = wave_sum_u64(t.tile_win),
                             tile_nnz = wave_sum_u64(t.tile_nnz), tile_many = wave_sum_u64(t.tile_many),
                             tile_unique = wave_sum_u64(t.tile_unique);
    if ((threadIdx.x & (kWave - 1)) == 0) {
        if (tiles) atomicAdd(&a.counts[0], tiles);
        if (tile_win) atomicAdd(&a.counts[1], tile_win);
        if (tile_nnz) atomicAdd(&a.counts[2], tile_nnz);
        if (tile_many) atomicAdd(&a.counts[3], tile_many);
        if (tile_unique) atomicAdd(&a.counts[5], tile_unique);
    }
}

__global__ __launch_bounds__(256) void choose_path_kernel(PathArgs a, int64_t n_win, const int32_t *win_unique_ptr)
{
    const int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    PathTotals t;
    if (w < n_win) choose_window(a, w, win_unique_ptr[w + 1] - win_unique_ptr[w], t);
    flush_path_totals(a, t);
}

// First step of the scan of the windows' unique counts (sums of blocks of kScanBlock windows) and, in the same
// pass over the counts, the path choice of every window.
__global__ __launch_bounds__(kScanThreads) void unique_sums_choose_kernel(const int32_t *__restrict__ win_unique,
                                                                          int64_t n_win, int32_t *__restrict__ block_sums,
                                                                          PathArgs a)
{
    __shared__ int tmp[kScanThreads / kWave + 1];
    const int64_t i0 = (int64_t)blockIdx.x * kScanBlock + (int64_t)threadIdx.x * kScanItems;
    int sum = 0;
    PathTotals t;
#pragma unroll 4
    for (int k = 0; k < kScanItems; ++k)
        if (i0 + k < n_win) {
            const int32_t uw = win_unique[i0 + k];
            sum += uw;
            choose_window(a, i0 + k, uw, t);
        }
    flush_path_totals(a, t);
    int total;
    (void)block_exclusive_scan(sum, tmp, &total);
    if (threadIdx.x == 0) block_sums[blockIdx.x] = total;
}

// ---- gather plan, step 2: offsets -----------------------------------------------------------------
// One workgroup turns the per-block counts into offsets, decides (from U, now known) whether the
// single-segment rows are ordered by length, and writes the plan sizes and the die table.
// Order of the finished segment list: first the segments of split rows (n_slots of them, sorted by
// start column in a later step, cut into 2 * kXcds bands of equal length), then the single-segment rows:
// by length class and row when the windows share few neighbours (4 U > 3 nnz), else by row alone, which
// keeps the rows of a window next to each other (that matters when they share neighbours).
template <typename Load, typename Store>
__device__ __forceinline__ int block_scan_sequence(int64_t n, Load load, Store store, int *tmp)
{
    int carry = 0;
    for (int64_t base = 0; base < n; base += (int64_t)blockDim.x * 4) {
        const int64_t i0 = base + (int64_t)threadIdx.x * 4;
        int v[4];
        int sum = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            v[k] = (i0 + k < n) ? load(i0 + k) : 0;
            sum += v[k];
        }
        int total;
        int run = carry + block_exclusive_scan(sum, tmp, &total);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (i0 + k < n) store(i0 + k, run);
            run += v[k];
        }
        carry += total;
    }
    return carry;
}

constexpr int kBands = 2 * kXcds;

// phase 0 (needs row_ptr only): offsets of the split rows and their segments, the bands of the die table.
// phase 1 (needs U): offsets of the single-segment rows, the rest of the result block.
__global__ __launch_bounds__(1024) void plan_scan_kernel(int phase, int64_t nb, const int32_t *__restrict__ block_sums,
                                                         int64_t nnz, int64_t n_win,
                                                         const int32_t *__restrict__ win_unique_ptr,
                                                         int32_t *__restrict__ long_off, int32_t *__restrict__ slot_off,
                                                         int32_t *__restrict__ tail_off, BuildInfo *info,
                                                         int32_t *__restrict__ long_slot_ptr,
                                                         const int32_t *__restrict__ win_unique,
                                                         int32_t *__restrict__ win_unique_ptr_out,
                                                         int32_t *__restrict__ unique_block_sums, int64_t n_unique_blocks,
                                                         PathArgs pa)
{
    __shared__ int tmp[1024 / kWave + 1];
    if (phase == 0) {
        const int n_long = block_scan_sequence(nb, [&](int64_t i) { return block_sums[i]; },
                                               [&](int64_t i, int v) { long_off[i] = v; }, tmp);
        const int n_slots = block_scan_sequence(nb, [&](int64_t i) { return block_sums[nb + i]; },
                                                [&](int64_t i, int v) { slot_off[i] = v; }, tmp);
        if (threadIdx.x == 0) {
            info->n_long = n_long;
            info->n_slots = n_slots;
            long_slot_ptr[n_long] = n_slots;
            // Die l walks bands l and 2 * kXcds - 1 - l of the split rows' segments (sorted by start column, so
            // a band is a range of columns: its X rows stay in that die's L2, and pairing a band of popular
            // columns with a band of rare ones spreads the L2 misses evenly), then its share of the tail.
            for (int l = 0; l < kXcds; ++l) {
                const int b2 = kBands - 1 - l;
                int32_t *t = info->lane_tab + kLaneTabStride * l;
                t[0] = (int32_t)((int64_t)n_slots * l / kBands);
                t[1] = (int32_t)((int64_t)n_slots * (l + 1) / kBands) - t[0];
                t[2] = (int32_t)((int64_t)n_slots * b2 / kBands);
                t[3] = (int32_t)((int64_t)n_slots * (b2 + 1) / kBands) - t[2];
                t[4] = n_slots;
            }
        }
        return;
    }
    // U: with few windows the exclusive scan of their unique counts and their path choice happen here; with
    // many (one workgroup would be slow) unique_sums_choose_kernel has been over the counts, this kernel scans
    // its block sums in place, and scan_apply_kernel finishes.
    int64_t U;
    if (win_unique) {
        U = block_scan_sequence(n_win, [&](int64_t i) { return win_unique[i]; },
                                [&](int64_t i, int v) { win_unique_ptr_out[i] = v; }, tmp);
        if (threadIdx.x == 0) win_unique_ptr_out[n_win] = (int32_t)U;
        PathTotals t;
        for (int64_t w0 = 0; w0 < n_win; w0 += blockDim.x)
            if (w0 + threadIdx.x < n_win) choose_window(pa, w0 + threadIdx.x, win_unique[w0 + threadIdx.x], t);
        flush_path_totals(pa, t);
    } else {
        U = block_scan_sequence(n_unique_blocks, [&](int64_t i) { return unique_block_sums[i]; },
                                [&](int64_t i, int v) { unique_block_sums[i] = v; }, tmp);
        if (threadIdx.x == 0) unique_block_sums[n_unique_blocks] = (int32_t)U;
    }
    const int sort_tail = 4 * U > 3 * (nnz > 0 ? nnz : 1) ? 1 : 0;
    int n_single;
    if (sort_tail) {
        // class-major: all blocks of class 0, then all blocks of class 1, ...
        n_single = block_scan_sequence((int64_t)kTailClasses * nb, [&](int64_t i) { return block_sums[2 * nb + i]; },
                                       [&](int64_t i, int v) { tail_off[i] = v; }, tmp);
    } else {
        n_single = block_scan_sequence(nb,
                                       [&](int64_t i) {
                                           int t = 0;
#pragma unroll
                                           for (int c = 0; c < kTailClasses; ++c) t += block_sums[(2 + c) * nb + i];
                                           return t;
                                       },
                                       [&](int64_t i, int v) { tail_off[i] = v; }, tmp);
    }
    if (threadIdx.x == 0) {
        info->n_seg = info->n_slots + n_single;
        info->sort_tail = sort_tail;
        info->total_unique = (int32_t)U;
        for (int l = 0; l < kXcds; ++l) info->lane_tab[kLaneTabStride * l + 5] = n_single;
    }
}

// ---- gather plan, step 3: the segment list -----------------------------------------------------------
// A thread takes four consecutive rows of its workgroup's block.  Single-segment rows go straight to their
// final place (stable inside a length class: block offset + the rows of the same class in front of this one
// inside the block).  Split rows get their entry in long_row / long_slot_ptr; their segments ("slots",
// numbered in row order) are written with the start column as sort key by all threads of the workgroup
// together -- a hub row has hundreds of segments.  One workgroup-wide scan carries all the counts: split
// rows, their segments, and the eight class counts packed two to a word (a block has 1024 rows).
// Sort key of a split row's segment: its start column at a relative resolution of 1/8 (the column itself
// below 16, else 8 steps per power of two) -- monotone in the column, at most 8 bits, so one pass of the
// radix sort orders the segments.  Skewed graphs keep their popular columns at small ids, where this key
// is fine-grained; equal steps in the column id would put a third of all segments into the first bucket.
constexpr int kSegKeyBits = 8;
__device__ __forceinline__ int32_t seg_sort_key(uint32_t c)
{
    if (c < 16u) return (int32_t)c;
    const int e = 31 - __clz(c);
    return 16 + (e - 4) * 8 + (int32_t)((c >> (e - 3)) & 7u);
}
constexpr int kFillVals = 2 + kTailClasses / 2;

struct FillCounts {
    int v[kFillVals];
};

__device__ __forceinline__ FillCounts block_exclusive_scan_counts(const FillCounts &in, int (*tmp)[kFillVals],
                                                                  FillCounts *total)
{
    const int lane = threadIdx.x & (kWave - 1), wid = threadIdx.x >> 6;
    constexpr int NW = 256 / kWave;
    FillCounts incl = in;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
#pragma unroll
        for (int k = 0; k < kFillVals; ++k) {
            const int t = __shfl_up(incl.v[k], off, kWave);
            if (lane >= off) incl.v[k] += t;
        }
    }
    if (lane == kWave - 1)
#pragma unroll
        for (int k = 0; k < kFillVals; ++k) tmp[wid][k] = incl.v[k];
    __syncthreads();
    FillCounts res;
#pragma unroll
    for (int k = 0; k < kFillVals; ++k) {
        int before = 0, all = 0;
#pragma unroll
        for (int w2 = 0; w2 < NW; ++w2) {
            const int t = tmp[w2][k];
            if (w2 < wid) before += t;
            all += t;
        }
        res.v[k] = before + incl.v[k] - in.v[k];
        total->v[k] = all;
    }
    return res;
}

// phase 0: split rows and their slots (needs row_ptr only); phase 1: single-segment rows (needs sort_tail).
__global__ __launch_bounds__(256) void seg_fill_kernel(
    int phase, int32_t n_rows, const int32_t *__restrict__ rp, const int32_t *__restrict__ ci, BuildInfo *info,
    int64_t nb, const int32_t *__restrict__ long_off, const int32_t *__restrict__ slot_off,
    const int32_t *__restrict__ tail_off, int32_t *__restrict__ seg_row,
    int32_t *__restrict__ seg_ebeg, int32_t *__restrict__ seg_dst, int32_t *__restrict__ long_row,
    int32_t *__restrict__ long_slot_ptr, int32_t *__restrict__ long_ebeg, int32_t *__restrict__ long_len,
    int32_t *__restrict__ gchunk_li, int32_t *__restrict__ gchunk_c, int32_t *__restrict__ slot_row,
    int32_t *__restrict__ slot_ebeg, int32_t *__restrict__ slot_key, int32_t slot_len)
{
    constexpr int RPT = kRowBlock / 256;           // rows per thread
    __shared__ int s_tmp[256 / kWave][kFillVals];
    // One buffer for both phases (the first keeps the block's split rows in it, the second its single-segment rows):
    // with 12 KB the workgroup fits beside the bitmap kernel, whose workgroups leave under 20 KB of a compute
    // unit's LDS free for the whole of their run -- with 24 KB this kernel waited for them to end.
    __shared__ int32_t s_rows[3 * kRowBlock + 1];
    int32_t *const s_lrow = s_rows, *const s_le0 = s_rows + kRowBlock, *const s_lslot = s_rows + 2 * kRowBlock;
    int32_t *const s_trow = s_rows, *const s_te0 = s_rows + kRowBlock, *const s_tdeg = s_rows + 2 * kRowBlock;
    const int sort_tail = phase == 1 ? info->sort_tail : 0;
    const int32_t n_slots = info->n_slots;
    const int32_t long_base = long_off[blockIdx.x], slot_base = slot_off[blockIdx.x];

    const int64_t r0 = (int64_t)blockIdx.x * kRowBlock + (int64_t)threadIdx.x * RPT;
    int32_t e0[RPT], deg[RPT];
    int cls[RPT];
    FillCounts mine;
#pragma unroll
    for (int k = 0; k < kFillVals; ++k) mine.v[k] = 0;
#pragma unroll
    for (int k = 0; k < RPT; ++k) {
        e0[k] = 0;
        deg[k] = 0;
        cls[k] = -1;
        if (r0 + k < n_rows) {
            e0[k] = rp[r0 + k];
            deg[k] = rp[r0 + k + 1] - e0[k];
            if (deg[k] > kSegLen) {
                mine.v[0] += 1;
                mine.v[1] += (deg[k] + slot_len - 1) / slot_len;
            } else {
                cls[k] = sort_tail ? length_class(deg[k]) : 0;
#pragma unroll
                for (int c = 0; c < kTailClasses; ++c)
                    if (cls[k] == c) mine.v[2 + c / 2] += 1 << (16 * (c & 1));
            }
        }
    }
    FillCounts total;
    const FillCounts before = block_exclusive_scan_counts(mine, s_tmp, &total);

    // Single-segment rows are put in (class, row) order in LDS first, so that the workgroup writes its piece
    // of every class as one contiguous run.
    __shared__ int s_cstart[kTailClasses + 1];
    int cstart[kTailClasses];
    {
        int run = 0;
#pragma unroll
        for (int c = 0; c < kTailClasses; ++c) {
            cstart[c] = run;
            run += (total.v[2 + c / 2] >> (16 * (c & 1))) & 0xFFFF;
        }
        if (threadIdx.x == 0) {
#pragma unroll
            for (int c = 0; c < kTailClasses; ++c) s_cstart[c] = cstart[c];
            s_cstart[kTailClasses] = run;
        }
    }
    int lrank = before.v[0], srank = before.v[1];
    int seen[kTailClasses];
#pragma unroll
    for (int c = 0; c < kTailClasses; ++c) seen[c] = cstart[c] + ((before.v[2 + c / 2] >> (16 * (c & 1))) & 0xFFFF);
#pragma unroll
    for (int k = 0; k < RPT; ++k) {
        if (r0 + k >= n_rows) continue;
        if (cls[k] < 0) {
            if (phase != 0) continue;
            if (blockIdx.y == 0) {
                long_row[long_base + lrank] = (int32_t)(r0 + k);
                long_slot_ptr[long_base + lrank] = slot_base + srank;
                long_ebeg[long_base + lrank] = e0[k];
                long_len[long_base + lrank] = deg[k];
            }
            // the few very long rows are listed apart, cut into pieces of kGiantChunk entries (the pieces of a row
            // are consecutive; the rows come in any order: the list only says who works on what)
            if (blockIdx.y == 0 && deg[k] > kGiantRow) {
                const int32_t pieces = (deg[k] + kGiantChunk - 1) / kGiantChunk;
                const int32_t at = atomicAdd(&info->n_gchunks, pieces);
                for (int32_t c = 0; c < pieces; ++c) {
                    gchunk_li[at + c] = long_base + lrank;
                    gchunk_c[at + c] = c;
                }
            }
            s_lrow[lrank] = (int32_t)(r0 + k);
            s_le0[lrank] = e0[k];
            s_lslot[lrank] = srank;
            ++lrank;
            srank += (deg[k] + slot_len - 1) / slot_len;
        } else if (phase == 1) {
            int lp = 0;
#pragma unroll
            for (int c = 0; c < kTailClasses; ++c)
                if (cls[k] == c) lp = seen[c]++;
            s_trow[lp] = (int32_t)(r0 + k);
            s_te0[lp] = e0[k];
            s_tdeg[lp] = deg[k];
        }
    }
    const int n_lrows = total.v[0], n_lsegs = total.v[1];
    if (threadIdx.x == 0 && phase == 0) s_lslot[n_lrows] = n_lsegs;
    __syncthreads();
    for (int i = threadIdx.x; phase == 1 && i < s_cstart[kTailClasses]; i += 256) {
        int c = 0;
#pragma unroll
        for (int c2 = 1; c2 < kTailClasses; ++c2)
            if (i >= s_cstart[c2]) c = c2;
        const int64_t tb = sort_tail ? tail_off[(int64_t)c * nb + blockIdx.x] : tail_off[blockIdx.x];
        const int64_t p = (int64_t)n_slots + tb + (i - s_cstart[c]);
        seg_row[p] = s_trow[i];
        seg_ebeg[p] = s_te0[i];
        seg_dst[p] = -1 - s_tdeg[i];     // below zero: written straight to the result; carries the row's length
    }
    // the slots of the block's split rows: four per thread and step, their start columns gathered together.  The
    // block that holds the hub rows of a power-law graph has 10^5 slots, so large graphs launch the first phase
    // with several workgroups per row block (gridDim.y), which share the block's slots in turns of 1024.
    for (int32_t s0 = threadIdx.x + 4 * 256 * blockIdx.y; phase == 0 && s0 < n_lsegs; s0 += 4 * 256 * gridDim.y) {
        int32_t eb[4], row[4];
        uint32_t col[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int32_t sl = s0 + u * 256;
            eb[u] = -1;
            if (sl >= n_lsegs) continue;
            int a = 0, b = n_lrows;                // last split row whose first slot is <= sl
            while (b - a > 1) {
                const int mid = (a + b) >> 1;
                if (s_lslot[mid] <= sl) a = mid; else b = mid;
            }
            eb[u] = s_le0[a] + (sl - s_lslot[a]) * slot_len;
            row[u] = s_lrow[a];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) col[u] = eb[u] >= 0 ? (uint32_t)ci[eb[u]] : 0u;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (eb[u] < 0) continue;
            const int32_t g = slot_base + s0 + u * 256;
            slot_row[g] = row[u];
            slot_ebeg[g] = eb[u];
            slot_key[g] = seg_sort_key(col[u]);
        }
    }
}

// Split rows' segments in their final order: position i of the list takes slot order[i] (order == nullptr:
// slot order).  seg_dst is the slot number, which is also where the segment's partial sum goes, with the code of
// the slot length above it unless the segment is the last of its row (slots are numbered in row order, so the
// next slot tells).
__global__ void seg_permute_kernel(const BuildInfo *info, const int32_t *__restrict__ order,
                                   const int32_t *__restrict__ slot_row, const int32_t *__restrict__ slot_ebeg,
                                   int32_t *__restrict__ seg_row, int32_t *__restrict__ seg_ebeg,
                                   int32_t *__restrict__ seg_dst, int32_t full_code)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= info->n_slots) return;
    const int32_t k = order ? order[i] : (int32_t)i;
    const int32_t row = slot_row[k];
    const bool full = k + 1 < info->n_slots && slot_row[k + 1] == row;
    seg_row[i] = row;
    seg_ebeg[i] = slot_ebeg[k];
    seg_dst[i] = full ? (k | (full_code << kSegSlotBits)) : k;
}

// The per-window lists are kept where the translation wrote them, each at its window's edge offset (a
// window never has more distinct columns than entries).  The exported col_to_row is the same lists back to
// back: one workgroup per window copies its list to win_unique_ptr[w].
__global__ __launch_bounds__(256) void pack_unique_kernel(int32_t n_rows, int32_t win_h,
                                                          const int32_t *__restrict__ rp,
                                                          const int32_t *__restrict__ loose,
                                                          const int32_t *__restrict__ win_unique_ptr,
                                                          int32_t *__restrict__ packed)
{
    const int64_t w = blockIdx.x;
    int32_t lo, hi;
    window_edge_range(rp, n_rows, win_h, w, &lo, &hi);
    const int32_t u0 = win_unique_ptr[w];
    const int32_t uw = win_unique_ptr[w + 1] - u0;
    for (int32_t k = threadIdx.x; k < uw; k += 256) packed[u0 + k] = loose[lo + k];
}

// One device allocation carved into 256-byte aligned pieces.
struct Arena {
    char *base = nullptr;
    size_t size = 0, used = 0;
    static size_t align(size_t b) { return (b + 255) & ~(size_t)255; }
    void want(size_t bytes) { size += align(std::max<size_t>(bytes, 4)); }
    int commit()
    {
        void *q = nullptr;
        int st = pool_alloc(&q, std::max<size_t>(size, 256));
        base = static_cast<char *>(q);
        return st;
    }
    template <typename T> T *take(int64_t count)
    {
        T *p = reinterpret_cast<T *>(base + used);
        used += align(std::max<size_t>((size_t)std::max<int64_t>(count, 0) * sizeof(T), 4));
        return p;
    }
};

// Returns the block to the pool on scope exit.  On the normal path the stream is idle by then; an early
// error return may leave kernels in flight that still use the block, so the stream is drained first.
struct ScopedFree {
    void *p = nullptr;
    hipStream_t s = nullptr;
    ~ScopedFree()
    {
        if (!p) return;
        (void)hipStreamSynchronize(s);
        pool_free(p);
    }
};

}  // namespace

int64_t scan_workspace_elems(int64_t n) { return ceil_div(std::max<int64_t>(n, 1), kScanBlock) + 2; }

int exclusive_scan_i32(const int32_t *d_in, int32_t *d_out, int64_t n, int32_t *d_work, hipStream_t s)
{
    // Up to a few thousand elements per thread-round a single workgroup is quicker than three launches.
    if (n <= 8 * kScanBlock) {
        hipLaunchKernelGGL(scan_single_kernel, dim3(1), dim3(1024), 0, s, d_in, d_out, n);
        return launch_status("scan_single_kernel");
    }
    const int64_t nb = ceil_div(n, kScanBlock);
    hipLaunchKernelGGL(scan_block_sum_kernel, dim3((unsigned)nb), dim3(kScanThreads), 0, s, d_in, n, d_work);
    hipLaunchKernelGGL(scan_single_kernel, dim3(1), dim3(1024), 0, s, d_work, d_work, nb);
    hipLaunchKernelGGL(scan_apply_kernel, dim3((unsigned)nb), dim3(kScanThreads), 0, s, d_in, d_out, n, d_work, nb);
    return launch_status("scan kernels");
}

static PathArgs path_args(const tcg_meta *m, tcg_policy policy, float min_reuse)
{
    return PathArgs{m->n_rows,     m->win_h,          m->tile_w,     (int)policy, min_reuse,
                    m->d_row_ptr,  m->d_win_partition, m->d_win_path, m->d_counters};
}

static void launch_choose_path(tcg_meta *m, tcg_policy policy, float min_reuse, hipStream_t s)
{
    if (m->n_win > 0)
        hipLaunchKernelGGL(choose_path_kernel, dim3((unsigned)ceil_div(m->n_win, 256)), dim3(256), 0, s,
                           path_args(m, policy, min_reuse), m->n_win, m->d_win_unique_ptr);
}

// counts: [0] tiles, [1] tile-path windows, [2] their edges, [3] windows of class kTileMany, [4] their widest,
// [5] distinct columns summed over the tile-path windows
static int finish_choose_path(tcg_meta *m, tcg_policy policy, float min_reuse, const unsigned long long *h, hipStream_t s)
{
    m->policy = policy;
    m->min_reuse = min_reuse;
    m->total_tiles = (int64_t)h[0];
    m->n_tile_win = (int64_t)h[1];
    m->nnz_tile = (int64_t)h[2];
    m->n_tile_many = (int64_t)h[3];
    m->max_unique_many = (int64_t)h[4];
    m->unique_tile = (int64_t)h[5];
    // A handful of qualifying windows is not worth a kernel launch that visits every window (18 us on a
    // million-node graph): under the automatic policy the tile path is used from 2 % of the stored entries on.
    if (policy == TCG_POLICY_AUTO && m->n_tile_win > 0 && m->nnz_tile * 50 < m->nnz) {
        TCG_HIP(hipMemsetAsync(m->d_win_path, 0, (size_t)m->n_win, s));
        m->n_tile_win = m->nnz_tile = m->n_tile_many = m->max_unique_many = m->unique_tile = 0;
    }
    return TCG_OK;
}

int choose_paths(tcg_meta *m, tcg_policy policy, float min_reuse, hipStream_t s)
{
    if (policy == TCG_POLICY_TILE && m->win_h != 16 && m->win_h != 32) return TCG_EINVAL;
    if (min_reuse <= 0.f) min_reuse = kDefaultMinReuse;
    TCG_HIP(hipMemsetAsync(m->d_counters, 0, 8 * sizeof(unsigned long long), s));
    launch_choose_path(m, policy, min_reuse, s);
    TCG_TRY(launch_status("choose_path_kernel"));
    unsigned long long h[8];
    TCG_HIP(hipMemcpyAsync(h, m->d_counters, sizeof(h), hipMemcpyDeviceToHost, s));
    TCG_HIP(hipStreamSynchronize(s));
    TCG_TRY(finish_choose_path(m, policy, min_reuse, h, s));
    TCG_HIP(hipStreamSynchronize(s));
    return TCG_OK;
}

// Tile counts for a tile width: per window ceil(U_w / tile_w), and the number of aligned tile_w-wide column
// blocks of the original matrix that hold an entry of the window (heads of runs of equal column / tile_w in
// the window's ascending list).  One workgroup per window, grid stride; totals by one atomic per workgroup.
__global__ __launch_bounds__(256) void tile_stats_kernel(int32_t n_rows, int32_t win_h, int64_t n_win, int32_t tile_w,
                                                         const int32_t *__restrict__ rp,
                                                         const int32_t *__restrict__ win_unique_ptr,
                                                         const int32_t *__restrict__ col_to_row,
                                                         unsigned long long *out)
{
    __shared__ unsigned long long s_red[256 / kWave];
    unsigned long long blocks = 0, tiles = 0;
    for (int64_t w = blockIdx.x; w < n_win; w += gridDim.x) {
        int32_t lo, hi;
        window_edge_range(rp, n_rows, win_h, w, &lo, &hi);
        const int32_t uw = win_unique_ptr[w + 1] - win_unique_ptr[w];
        if (threadIdx.x == 0) tiles += (unsigned long long)(((int64_t)uw + tile_w - 1) / tile_w);
        // eight entries per thread in flight: a hub window has 10^5 distinct columns
        constexpr int kUnroll = 8;
        for (int32_t k0 = threadIdx.x; k0 < uw; k0 += 256 * kUnroll) {
            int32_t cur[kUnroll], prev[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int32_t k = k0 + u * 256;
                cur[u] = k < uw ? col_to_row[lo + k] : 0;
                prev[u] = k < uw && k > 0 ? col_to_row[lo + k - 1] : 0;
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int32_t k = k0 + u * 256;
                if (k < uw && (k == 0 || cur[u] / tile_w != prev[u] / tile_w)) ++blocks;
            }
        }
    }
    blocks = wave_sum_u64(blocks);
    if ((threadIdx.x & (kWave - 1)) == 0) s_red[threadIdx.x >> 6] = blocks;
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long t = 0;
        for (int i = 0; i < 256 / kWave; ++i) t += s_red[i];
        if (tiles) atomicAdd(&out[0], tiles);
        if (t) atomicAdd(&out[1], t);
    }
}

int tile_stats(const tcg_meta *m, int32_t tile_w, int64_t *translated, int64_t *untranslated, hipStream_t s)
{
    unsigned long long *out = m->d_counters + 6;        // the two spare slots of the counter block
    TCG_HIP(hipMemsetAsync(out, 0, 2 * sizeof(unsigned long long), s));
    if (m->n_win > 0) {
        hipLaunchKernelGGL(tile_stats_kernel, dim3((unsigned)std::min<int64_t>(m->n_win, 4096)), dim3(256), 0, s, m->n_rows,
                           m->win_h, m->n_win, tile_w, m->d_row_ptr, m->d_win_unique_ptr, m->d_col_to_row, out);
        TCG_TRY(launch_status("tile_stats_kernel"));
    }
    unsigned long long h[2] = {0, 0};
    TCG_HIP(hipMemcpyAsync(h, out, sizeof(h), hipMemcpyDeviceToHost, s));
    TCG_HIP(hipStreamSynchronize(s));
    if (translated) *translated = (int64_t)h[0];
    if (untranslated) *untranslated = (int64_t)h[1];
    return TCG_OK;
}

int export_col_to_row(const tcg_meta *m, int32_t *d_packed, hipStream_t s)
{
    if (m->n_win == 0 || m->total_unique == 0) return TCG_OK;
    hipLaunchKernelGGL(pack_unique_kernel, dim3((unsigned)m->n_win), dim3(256), 0, s, m->n_rows, m->win_h, m->d_row_ptr,
                       m->d_col_to_row, m->d_win_unique_ptr, d_packed);
    return launch_status("pack_unique_kernel");
}

template <int THREADS, int KPT>
static void launch_sort_class(const tcg_meta *m, int cls, int64_t max_windows, int64_t grid_cap, bool wide_keys,
                              const int32_t *lists, const BuildInfo *info, int32_t *win_unique, hipStream_t s)
{
    if (max_windows <= 0) return;
    const unsigned grid = (unsigned)std::min<int64_t>(max_windows, grid_cap);
    const int32_t *list = lists + (int64_t)cls * m->n_win;
    if (wide_keys)
        hipLaunchKernelGGL((sgt_window_sort_kernel<THREADS, KPT, uint64_t>), dim3(grid), dim3(THREADS), 0, s, m->n_rows,
                           m->win_h, list, info->cls_count + cls, m->d_row_ptr, m->d_col_idx, m->d_edge_to_col,
                           m->d_col_to_row, win_unique);
    else
        hipLaunchKernelGGL((sgt_window_sort_kernel<THREADS, KPT, uint32_t>), dim3(grid), dim3(THREADS), 0, s, m->n_rows,
                           m->win_h, list, info->cls_count + cls, m->d_row_ptr, m->d_col_idx, m->d_edge_to_col,
                           m->d_col_to_row, win_unique);
}

static void launch_sort_small(const tcg_meta *m, int64_t most0, int64_t most1, int64_t most2, bool wide_keys,
                              const int32_t *lists, const BuildInfo *info, int32_t *win_unique, hipStream_t s)
{
    if (most0 <= 0) return;
    const int32_t g0 = (int32_t)std::min<int64_t>(most0, 12288), g1 = (int32_t)std::min<int64_t>(std::max<int64_t>(most1, 1), 4096),
                  g2 = (int32_t)std::min<int64_t>(std::max<int64_t>(most2, 1), 4096);
    if (wide_keys)
        hipLaunchKernelGGL(sgt_window_sort_small_kernel<uint64_t>, dim3((unsigned)(g0 + g1 + g2)), dim3(kWave), 0, s,
                           m->n_rows, m->win_h, m->n_win, lists, info->cls_count, g0, g1, m->d_row_ptr, m->d_col_idx,
                           m->d_edge_to_col, m->d_col_to_row, win_unique);
    else
        hipLaunchKernelGGL(sgt_window_sort_small_kernel<uint32_t>, dim3((unsigned)(g0 + g1 + g2)), dim3(kWave), 0, s,
                           m->n_rows, m->win_h, m->n_win, lists, info->cls_count, g0, g1, m->d_row_ptr, m->d_col_idx,
                           m->d_edge_to_col, m->d_col_to_row, win_unique);
}

// Pinned host slots for the result block of a build (allocated once; builds running at the same time take
// different slots).
constexpr int kHostSlots = 16;
static std::mutex g_slot_mu;
static BuildInfo *g_slot_base = nullptr;
static unsigned g_slot_busy = 0;
static bool g_slot_failed = false;
struct HostSlot {
    BuildInfo *info = nullptr;
    int index = -1;
    HostSlot()
    {
        std::lock_guard<std::mutex> lock(g_slot_mu);
        if (!g_slot_base && !g_slot_failed) {
            void *p = nullptr;
            if (hipHostMalloc(&p, sizeof(BuildInfo) * kHostSlots, hipHostMallocDefault) == hipSuccess)
                g_slot_base = static_cast<BuildInfo *>(p);
            else {
                (void)hipGetLastError();
                g_slot_failed = true;
            }
        }
        if (!g_slot_base) return;
        for (int i = 0; i < kHostSlots; ++i)
            if (!((g_slot_busy >> i) & 1u)) {
                g_slot_busy |= 1u << i;
                index = i;
                info = g_slot_base + i;
                return;
            }
    }
    ~HostSlot()
    {
        if (index < 0) return;
        std::lock_guard<std::mutex> lock(g_slot_mu);
        g_slot_busy &= ~(1u << index);
    }
    HostSlot(const HostSlot &) = delete;
    HostSlot &operator=(const HostSlot &) = delete;
};

// Two more streams per device.  After the first kernel a translation has three independent branches: the
// bitmap-class kernel (its hub windows make it the longest kernel, while it needs one workgroup per compute
// unit only), the sorted classes, and the part of the gather plan that depends on row_ptr alone (a chain of
// small launches).  They run side by side and meet again before U is formed.  Default priority, created once.
struct SideStream {
    hipStream_t stream = nullptr, plan_stream = nullptr;
    hipEvent_t fork = nullptr, join = nullptr, plan_join = nullptr;
};
static std::mutex g_side_mu;
static SideStream g_side[64];

static int side_stream(int device, SideStream **out)
{
    if (device < 0 || device >= 64) return TCG_EINVAL;
    std::lock_guard<std::mutex> lock(g_side_mu);
    SideStream &sd = g_side[device];
    if (!sd.stream) {
        TCG_HIP(hipStreamCreateWithFlags(&sd.stream, hipStreamNonBlocking));
        TCG_HIP(hipStreamCreateWithFlags(&sd.plan_stream, hipStreamNonBlocking));
        TCG_HIP(hipEventCreateWithFlags(&sd.fork, hipEventDisableTiming));
        TCG_HIP(hipEventCreateWithFlags(&sd.join, hipEventDisableTiming));
        TCG_HIP(hipEventCreateWithFlags(&sd.plan_join, hipEventDisableTiming));
    }
    *out = &sd;
    return TCG_OK;
}

// Waits for the side stream when the scope ends (a no-op on the normal path, where the main stream has
// already waited for it; it matters when an error return leaves its kernel in flight).
struct SideGuard {
    hipStream_t s = nullptr, s2 = nullptr;
    ~SideGuard()
    {
        if (s) (void)hipStreamSynchronize(s);
        if (s2) (void)hipStreamSynchronize(s2);
    }
};

// Host side of a translation.  Every size the kernels need is either known from (n_rows, nnz) or read by
// them from device memory, so everything is enqueued back to back and the host waits once, at the end,
// for the block of small results (sizes of the plan, U, the die table, the path totals).  Buffers whose
// exact size is only known then are sized by their bounds: a row has at least one segment and a split row
// (more than kSegLen entries) at most deg / kSegLen + 1, and a window has no more distinct columns than
// entries.
int sgt_build_impl(tcg_meta *m, int validate, hipStream_t s)
{
    const int32_t n = m->n_rows;
    const int64_t nnz = m->nnz;
    const int64_t n_win = m->n_win;
    const int64_t nb_rows = ceil_div(std::max<int64_t>(n, 0), kRowBlock);
    const int64_t long_bound = nnz / (kSegLen + 1) + 1;
    const int slot_len = slot_length(m->n_cols);
    const int64_t slot_bound = nnz / slot_len + long_bound;
    const int64_t seg_bound = (int64_t)n + slot_bound;
    if (seg_bound >= (int64_t)INT32_MAX) return TCG_ERANGE;
    // Windows above kSortCap entries form the bitmap class: in LDS when the bitmap over the column space fits.
    const int64_t n_words = ceil_div(m->n_cols, 32);
    const bool lds_bitmap = lds_bitmap_bytes(n_words) <= kLdsBitmapMax;
    // The LDS bitmap is quicker than sorting from about a thousand entries on; the bitmap in device memory
    // only beyond the largest sorted class.
    const int32_t sort_cap = lds_bitmap ? kLdsBitmapFrom : kSortCap;
    int col_bits = 1;
    while (col_bits < 31 && ((int64_t)1 << col_bits) < (int64_t)m->n_cols) ++col_bits;

    // Kept: the translated graph, the gather plan, the block of small results.
    Arena keep;
    keep.want(n_win * 4);             // win_partition
    keep.want((n_win + 1) * 4);       // win_unique_ptr
    keep.want(nnz * 4);               // edge_to_col
    keep.want(nnz * 4);               // col_to_row (each window's list at its edge offset)
    keep.want(n_win);                 // win_path
    keep.want(sizeof(BuildInfo));
    for (int i = 0; i < 3; ++i) keep.want(seg_bound * 4);
    keep.want(long_bound * 4);
    keep.want((long_bound + 1) * 4);
    keep.want(long_bound * 4);
    keep.want(long_bound * 4);
    const int64_t gchunk_bound = nnz / kGiantChunk + nnz / (kGiantRow + 1) + 1;
    keep.want(gchunk_bound * 4);
    keep.want(gchunk_bound * 4);
    TCG_TRY(keep.commit());
    m->owned[m->n_owned++] = keep.base;
    m->d_win_partition = keep.take<int32_t>(n_win);
    m->d_win_unique_ptr = keep.take<int32_t>(n_win + 1);
    m->d_edge_to_col = keep.take<int32_t>(nnz);
    m->d_col_to_row = keep.take<int32_t>(nnz);
    m->d_win_path = keep.take<uint8_t>(n_win);
    BuildInfo *info = keep.take<BuildInfo>(1);
    m->d_seg_row = keep.take<int32_t>(seg_bound);
    m->d_seg_ebeg = keep.take<int32_t>(seg_bound);
    m->d_seg_dst = keep.take<int32_t>(seg_bound);
    m->d_long_row = keep.take<int32_t>(long_bound);
    m->d_long_slot_ptr = keep.take<int32_t>(long_bound + 1);
    m->d_long_ebeg = keep.take<int32_t>(long_bound);
    m->d_long_len = keep.take<int32_t>(long_bound);
    m->d_gchunk_li = keep.take<int32_t>(gchunk_bound);
    m->d_gchunk_c = keep.take<int32_t>(gchunk_bound);
    m->d_lane_tab = info->lane_tab;
    m->d_counters = info->counters;

    // Temporaries of the build.
    const size_t sort_bytes = radix_sort_scratch_bytes(slot_bound);
    const int64_t scan_elems = scan_workspace_elems(n_win);
    Arena tmp;
    tmp.want((n_win + 1) * 4);                      // win_unique
    const int64_t hub_extra = (int64_t)(kHubMaxParts - 1) * (nnz / kHubEntries + 1);   // items beyond one per window
    tmp.want(((int64_t)kClasses * n_win + hub_extra) * 4);        // class lists (the bitmap class last)
    tmp.want((n_win + hub_extra) * 4);                            // parts of the bitmap class's items
    tmp.want((int64_t)kPlanSums * nb_rows * 4);     // per-row-block counts
    tmp.want((nb_rows + 1) * 4);                    // long_off
    tmp.want((nb_rows + 1) * 4);                    // slot_off
    tmp.want((int64_t)kTailClasses * nb_rows * 4);  // tail_off
    tmp.want(scan_elems * 4);
    for (int i = 0; i < 5; ++i) tmp.want(slot_bound * 4);   // slot_row, slot_ebeg, slot_key, sorted keys, order
    tmp.want(sort_bytes);
    TCG_TRY(tmp.commit());
    ScopedFree tmp_guard{tmp.base, s};
    int32_t *win_unique = tmp.take<int32_t>(n_win + 1);
    int32_t *lists = tmp.take<int32_t>((int64_t)kClasses * n_win + hub_extra);
    int32_t *large_part = tmp.take<int32_t>(n_win + hub_extra);
    int32_t *block_sums = tmp.take<int32_t>((int64_t)kPlanSums * nb_rows);
    int32_t *long_off = tmp.take<int32_t>(nb_rows + 1);
    int32_t *slot_off = tmp.take<int32_t>(nb_rows + 1);
    int32_t *tail_off = tmp.take<int32_t>((int64_t)kTailClasses * nb_rows);
    int32_t *scan_work = tmp.take<int32_t>(scan_elems);
    int32_t *slot_row = tmp.take<int32_t>(slot_bound);
    int32_t *slot_ebeg = tmp.take<int32_t>(slot_bound);
    int32_t *slot_key = tmp.take<int32_t>(slot_bound);
    int32_t *key_sorted = tmp.take<int32_t>(slot_bound);
    int32_t *order = tmp.take<int32_t>(slot_bound);
    void *sort_scratch = tmp.take<char>((int64_t)sort_bytes);

    TCG_HIP(hipMemsetAsync(info, 0, sizeof(BuildInfo), s));

    if (validate) {
        // Both checks run before anything follows row_ptr into col_idx (the column check walks 0 .. nnz-1).
        hipLaunchKernelGGL(validate_csr_kernel, dim3((unsigned)std::min<int64_t>(ceil_div((int64_t)n + 1, 256), 4096)),
                           dim3(256), 0, s, n, nnz, m->d_row_ptr, &info->flag);
        if (nnz > 0)
            hipLaunchKernelGGL(validate_cols_kernel, dim3((unsigned)std::min<int64_t>(ceil_div(nnz, 256), 8192)),
                               dim3(256), 0, s, m->n_cols, nnz, m->d_col_idx, &info->flag);
        TCG_TRY(launch_status("validate kernels"));
        int h = 0;
        TCG_HIP(hipMemcpyAsync(&h, &info->flag, sizeof(int), hipMemcpyDeviceToHost, s));
        TCG_HIP(hipStreamSynchronize(s));
        if (h) return TCG_ECSR;
    }

    // Per-row-block counts of the gather plan and the window classes (both depend on row_ptr only).
    if (nb_rows + ceil_div(n_win, 256) > 0) {
        hipLaunchKernelGGL(prep_kernel, dim3((unsigned)(nb_rows + ceil_div(n_win, 256))), dim3(256), 0, s, n, m->win_h,
                           n_win, m->d_row_ptr, nb_rows, block_sums, lists, info->cls_count, win_unique, sort_cap, large_part,
                           lds_bitmap ? kHubEntries : INT_MAX, slot_len);
        TCG_TRY(launch_status("prep_kernel"));
    }

    // Fork: the caller's stream keeps the sorted classes; the bitmap class and the first part of the gather plan
    // go to the library's two side streams (see SideStream).
    ScopedFree bitmap_guard{nullptr, s};
    SideGuard side_guard;
    SideStream *side = nullptr;
    // Small graphs stay on the caller's stream: their kernels are over before the next one is enqueued, so there
    // is nothing to overlap, and the hand-over between streams costs 10-20 us (measured: 2,048 nodes 118 -> 100 us,
    // 20,000 nodes 114 -> 100 us per build; 100,000 nodes with hub windows 160 -> 180 us the other way round).
    const bool forked = nnz >= kForkMinEntries;
    hipStream_t bitmap_stream = s, plan_stream = s;
    if (forked) {
        TCG_TRY(side_stream(m->device, &side));
        std::lock_guard<std::mutex> lock(g_side_mu);
        TCG_HIP(hipEventRecord(side->fork, s));
        TCG_HIP(hipStreamWaitEvent(side->stream, side->fork, 0));
        TCG_HIP(hipStreamWaitEvent(side->plan_stream, side->fork, 0));
        side_guard.s = bitmap_stream = side->stream;
        side_guard.s2 = plan_stream = side->plan_stream;
    }

    // Branch 1: the bitmap class (its hub windows take longest, so it starts first).
    const int64_t large_most = std::min<int64_t>(n_win, nnz / ((int64_t)sort_cap + 1));
    if (large_most > 0 && lds_bitmap) {
        const size_t lds = lds_bitmap_bytes(n_words);
        static bool raised = false;       // more than 64 KB of dynamic LDS has to be asked for once
        if (!raised) {
            TCG_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(sgt_window_lds_bitmap_kernel),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBitmapMax));
            raised = true;
        }
        static int n_cu = 0;              // one workgroup per compute unit
        if (n_cu <= 0 && (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, m->device) != hipSuccess ||
                          n_cu <= 0))
            n_cu = 256;
        const unsigned grid = (unsigned)std::min<int64_t>(large_most + hub_extra, n_cu);
        hipLaunchKernelGGL(sgt_window_lds_bitmap_kernel, dim3(grid), dim3(kBitmapThreads), lds, bitmap_stream, n, m->win_h,
                           (int32_t)n_words, lists + (int64_t)kClsLarge * n_win, large_part, info->cls_count + kClsLarge,
                           &info->ticket,
                           m->d_row_ptr, m->d_col_idx, m->d_edge_to_col, m->d_col_to_row, win_unique);
        TCG_TRY(launch_status("sgt_window_lds_bitmap_kernel"));
    } else if (large_most > 0) {
        // Column space too wide for LDS: the bitmap lives in device scratch, sized by the number of windows
        // in the class, which the host has to fetch first (the one extra wait of this rare path).
        hipStream_t bs = bitmap_stream;
        int32_t n_large = 0;
        TCG_HIP(hipMemcpyAsync(&n_large, info->cls_count + kClsLarge, sizeof(int32_t), hipMemcpyDeviceToHost, bs));
        TCG_HIP(hipStreamSynchronize(bs));
        if (n_large > 0) {
            const int64_t budget_words = (int64_t)(128ll << 20) / 4;  // 128 MiB per scratch array
            const int64_t batch = std::max<int64_t>(1, std::min<int64_t>(n_large, budget_words / n_words));
            uint32_t *bitmap = nullptr;
            TCG_TRY(dev_alloc(&bitmap, 2 * batch * n_words));
            bitmap_guard.p = bitmap;
            int32_t *prefix = reinterpret_cast<int32_t *>(bitmap + batch * n_words);
            for (int64_t b0 = 0; b0 < n_large; b0 += batch) {
                const int64_t nb = std::min<int64_t>(batch, n_large - b0);
                TCG_HIP(hipMemsetAsync(bitmap, 0, (size_t)(nb * n_words) * sizeof(uint32_t), bs));
                hipLaunchKernelGGL(sgt_window_bitmap_kernel, dim3((unsigned)nb), dim3(kBitmapThreads), 0, bs, n,
                                   m->win_h, n_words, lists + (int64_t)kClsLarge * n_win + b0, m->d_row_ptr, m->d_col_idx,
                                   bitmap, prefix, m->d_edge_to_col, m->d_col_to_row, win_unique);
                TCG_TRY(launch_status("sgt_window_bitmap_kernel"));
            }
        }
    }

    // Branch 2 (enqueued before the third, whose kernels are short: the host takes a few microseconds per launch,
    // and these kernels are on the critical path): the sorted classes, one launch each beyond the three smallest (a column and a position inside
    // the window must fit 32 bits for 32-bit sort keys, else 64-bit ones).  A class with at least `lo` entries
    // per window has at most nnz / lo windows; the kernels read the real count on the device.
    {
        auto most = [&](int64_t least_entries) { return std::min<int64_t>(n_win, nnz / least_entries); };
        launch_sort_small(m, most(1), most(65), most(129), col_bits + 8 > 32, lists, info, win_unique, s);
        launch_sort_class<128, 4>(m, 3, most(257), 4096, col_bits + 9 > 32, lists, info, win_unique, s);
        launch_sort_class<256, 4>(m, 4, most(513), 2048, col_bits + 10 > 32, lists, info, win_unique, s);
        if (sort_cap > 1024) launch_sort_class<512, 4>(m, 5, most(1025), 1024, col_bits + 11 > 32, lists, info, win_unique, s);
        if (sort_cap > 2048) launch_sort_class<1024, 4>(m, 6, most(2049), 512, col_bits + 12 > 32, lists, info, win_unique, s);
        TCG_TRY(launch_status("sgt_window_sort_kernel"));
    }

    // Branch 3: the gather plan as far as it needs row_ptr only -- split rows, their segments sorted by start
    // column (segments that run one after the other on a die then read neighbouring -- on skewed graphs largely
    // the same -- X rows).
    {
        hipStream_t ps = plan_stream;
        // (256 threads: a workgroup of 1024 waits a long time for sixteen free wavefront slots on one compute unit
        // while the sort kernels' small workgroups keep taking them)
        hipLaunchKernelGGL(plan_scan_kernel, dim3(1), dim3(256), 0, ps, 0, nb_rows, block_sums, nnz, n_win,
                           m->d_win_unique_ptr, long_off, slot_off, tail_off, info, m->d_long_slot_ptr,
                           (const int32_t *)nullptr, (int32_t *)nullptr, (int32_t *)nullptr, (int64_t)0,
                           path_args(m, TCG_POLICY_AUTO, kDefaultMinReuse));
        if (nb_rows > 0) {
            hipLaunchKernelGGL(seg_fill_kernel, dim3((unsigned)nb_rows, forked ? kSlotSharers : 1), dim3(256), 0, ps, 0, n, m->d_row_ptr, m->d_col_idx,
                               info, nb_rows, long_off, slot_off, tail_off, m->d_seg_row, m->d_seg_ebeg, m->d_seg_dst,
                               m->d_long_row, m->d_long_slot_ptr, m->d_long_ebeg, m->d_long_len, m->d_gchunk_li, m->d_gchunk_c, slot_row, slot_ebeg,
                               slot_key, slot_len);
            TCG_TRY(launch_status("plan kernels"));
            const bool sorted = sort_bytes > 0 && slot_bound > 1;
            if (sorted)
                TCG_TRY(radix_sort_pairs(slot_key, nullptr, slot_bound, &info->n_slots, kSegKeyBits, key_sorted, order,
                                         sort_scratch, ps));
            hipLaunchKernelGGL(seg_permute_kernel, dim3((unsigned)ceil_div(slot_bound, 256)), dim3(256), 0, ps, info,
                               sorted ? order : (const int32_t *)nullptr, slot_row, slot_ebeg, m->d_seg_row, m->d_seg_ebeg,
                               m->d_seg_dst, segment_full_code(slot_len));
        }
        TCG_TRY(launch_status("plan kernels"));
    }

    // Join.
    {
        if (forked) {
            std::lock_guard<std::mutex> lock(g_side_mu);
            TCG_HIP(hipEventRecord(side->join, side->stream));
            TCG_HIP(hipEventRecord(side->plan_join, side->plan_stream));
            TCG_HIP(hipStreamWaitEvent(s, side->join, 0));
            TCG_HIP(hipStreamWaitEvent(s, side->plan_join, 0));
        }
    }

    // With every window translated: U, and the part of the plan that depends on it (the order of the
    // single-segment rows).
    const bool scan_inside = n_win <= (1 << 14);        // one workgroup scans this many counts in a few microseconds
    const int64_t n_ublocks = ceil_div(n_win, kScanBlock);
    const PathArgs pa = path_args(m, TCG_POLICY_AUTO, kDefaultMinReuse);
    if (!scan_inside)
        hipLaunchKernelGGL(unique_sums_choose_kernel, dim3((unsigned)n_ublocks), dim3(kScanThreads), 0, s, win_unique,
                           n_win, scan_work, pa);
    hipLaunchKernelGGL(plan_scan_kernel, dim3(1), dim3(1024), 0, s, 1, nb_rows, block_sums, nnz, n_win,
                       m->d_win_unique_ptr, long_off, slot_off, tail_off, info, m->d_long_slot_ptr,
                       scan_inside ? win_unique : (const int32_t *)nullptr, m->d_win_unique_ptr, scan_work, n_ublocks,
                       pa);
    if (!scan_inside)
        hipLaunchKernelGGL(scan_apply_kernel, dim3((unsigned)n_ublocks), dim3(kScanThreads), 0, s, win_unique,
                           m->d_win_unique_ptr, n_win, scan_work, n_ublocks);
    if (nb_rows > 0)
        hipLaunchKernelGGL(seg_fill_kernel, dim3((unsigned)nb_rows), dim3(256), 0, s, 1, n, m->d_row_ptr, m->d_col_idx,
                           info, nb_rows, long_off, slot_off, tail_off, m->d_seg_row, m->d_seg_ebeg,
                           m->d_seg_dst, m->d_long_row, m->d_long_slot_ptr, m->d_long_ebeg, m->d_long_len, m->d_gchunk_li, m->d_gchunk_c, slot_row, slot_ebeg,
                               slot_key, slot_len);
    TCG_TRY(launch_status("plan and path kernels"));

    // The result block comes back through pinned host memory (a copy to pageable memory is staged by the
    // runtime and takes longer); a build that finds all slots taken copies to its stack instead.
    BuildInfo h_stack;
    HostSlot slot;
    BuildInfo *hp = slot.info ? slot.info : &h_stack;
    TCG_HIP(hipMemcpyAsync(hp, info, sizeof(BuildInfo), hipMemcpyDeviceToHost, s));
    TCG_HIP(hipStreamSynchronize(s));                       // the one wait of a build
    const BuildInfo &h = *hp;
    m->n_seg = h.n_seg;
    m->n_long = h.n_long;
    m->n_gchunks = h.n_gchunks;
    m->n_slots = h.n_slots;
    m->total_unique = h.total_unique;
    for (int i = 0; i < kLaneTabStride * kXcds; ++i) m->h_lane_tab[i] = h.lane_tab[i];
    TCG_TRY(finish_choose_path(m, TCG_POLICY_AUTO, kDefaultMinReuse, h.counters, s));

    // Scratch of the split rows (sized exactly, now that n_slots is known): fp32 partial sums for feature widths
    // up to kPartialInitD and the (maximum, denominator) pairs of the fused attention.
    {
        Arena part;
        part.want(m->n_slots * kPartialInitD * 4);
        part.want(m->n_slots * 2 * 4);
        TCG_TRY(part.commit());
        m->owned[m->n_owned++] = part.base;
        m->d_partial = part.take<float>(m->n_slots * kPartialInitD);
        m->partial_elems = m->n_slots * kPartialInitD;
        m->partial_owned = false;
        m->d_partial_ml = part.take<float>(m->n_slots * 2);
    }
    return TCG_OK;   // temporaries are freed by the guards; the stream is idle here (or drains a last fill)
}

}  // namespace tcg
