// Sparse Graph Translation on the GPU (Algorithm 1 and section 4.1 of the paper) and the
// execution plan derived from it.
//
// The paper notes that row windows are independent, so each window is translated by one
// workgroup.  Four size classes, all producing the same canonical result (ascending unique
// column list, rank of every edge's column in it):
//   tiny   (<= 128 edges)    bitonic network in LDS, one wavefront
//   small  (<= 1024 edges)   same, 256 threads
//   medium (<= 4096 edges)   same, 256 threads, 32 KB of LDS
//   large  (>  4096 edges)   a bitmap over the column space in device scratch: set a bit per
//                            edge, prefix-popcount the words, rank = prefix + popcount below.
//                            Hub windows of power-law graphs land here; the cost is
//                            O(n_cols / 32 + nnz_w) per window.
// Every window first writes its unique list at its own edge offset of a temporary array (the
// list is never longer than the window's edge range); once all U_w are known a prefix sum gives
// win_unique_ptr and the lists are packed into col_to_row.
//
// Host side: three stream synchronisations per build (class / plan sizes, U, final counters) and a
// handful of arena allocations; everything else is enqueued back to back.
#include "common.h"

#include <limits.h>

#include <algorithm>

namespace tcg {

namespace {

constexpr int kTinyCap = 128;
constexpr int kSmallCap = 1024;
constexpr int kMediumCap = 4096;   // 2 x 16 KB of static LDS

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

// ---- window classification -----------------------------------------------------------------------
// Appends every non-empty window to the list of its size class (order inside a list is irrelevant:
// a window's result depends on the window only); empty windows get U_w = 0 here.
// counts[0..3] = tiny, small, medium, large.
__global__ __launch_bounds__(256) void classify_windows_kernel(int32_t n_rows, int32_t win_h, int64_t n_win,
                                                               const int32_t *rp, int32_t *lists, int *counts,
                                                               int32_t *win_unique, int32_t medium_cap)
{
    const int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int lane = threadIdx.x & (kWave - 1);
    int cls = -1;
    if (w < n_win) {
        int32_t lo, hi;
        window_edge_range(rp, n_rows, win_h, w, &lo, &hi);
        const int32_t cnt = hi - lo;
        if (cnt == 0) win_unique[w] = 0;
        else cls = cnt <= kTinyCap ? 0 : cnt <= kSmallCap ? 1 : cnt <= medium_cap ? 2 : 3;
    }
    // One atomic per wavefront and class instead of one per window.
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const unsigned long long mask = __ballot(cls == c);
        if (mask == 0) continue;
        const int leader = __ffsll((long long)mask) - 1;
        int base = 0;
        if (lane == leader) base = atomicAdd(&counts[c], __popcll(mask));
        base = __shfl(base, leader, kWave);
        if (cls == c) lists[(int64_t)c * n_win + base + __popcll(mask & ((1ull << lane) - 1ull))] = (int32_t)w;
    }
}

// Tiny, small and medium classes: one workgroup per listed window.
template <int THREADS, int CAP>
__global__ __launch_bounds__(THREADS) void sgt_window_lds_kernel(
    int32_t n_rows, int32_t win_h, const int32_t *__restrict__ win_list, const int32_t *__restrict__ rp,
    const int32_t *__restrict__ ci, int32_t *__restrict__ edge_to_col, int32_t *__restrict__ tmp_clean,
    int32_t *__restrict__ win_unique)
{
    __shared__ int32_t s_key[CAP];
    __shared__ int32_t s_rank[CAP];
    __shared__ int s_tmp[(THREADS + kWave - 1) / kWave + 1];

    const int64_t w = win_list[blockIdx.x];
    int32_t lo, hi;
    window_edge_range(rp, n_rows, win_h, w, &lo, &hi);
    const int cnt = hi - lo;          // 1 <= cnt <= CAP by classification
    int n_pad = 2;
    while (n_pad < cnt) n_pad <<= 1;

    for (int i = threadIdx.x; i < n_pad; i += THREADS) s_key[i] = i < cnt ? ci[lo + i] : INT_MAX;
    __syncthreads();

    // Bitonic sorting network, ascending.
    for (int k = 2; k <= n_pad; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int t = threadIdx.x; t < (n_pad >> 1); t += THREADS) {
                int a = ((t & ~(j - 1)) << 1) | (t & (j - 1));
                int b = a | j;
                int32_t ka = s_key[a], kb = s_key[b];
                bool up = (a & k) == 0;
                if ((ka > kb) == up) {
                    s_key[a] = kb;
                    s_key[b] = ka;
                }
            }
            __syncthreads();
        }
    }

    // Head flags of the sorted run and their prefix count: rank of position i = #heads in [0, i] - 1.
    const int ipt = n_pad >= THREADS ? n_pad / THREADS : 1;
    const int i0 = threadIdx.x * ipt;
    int local = 0;
    for (int k = 0; k < ipt; ++k) {
        int i = i0 + k;
        if (i < cnt && (i == 0 || s_key[i] != s_key[i - 1])) ++local;
    }
    int total;
    int run = block_exclusive_scan(local, s_tmp, &total);
    for (int k = 0; k < ipt; ++k) {
        int i = i0 + k;
        if (i < cnt) {
            bool head = (i == 0 || s_key[i] != s_key[i - 1]);
            if (head) {
                tmp_clean[lo + run] = s_key[i];
                ++run;
            }
            s_rank[i] = run - 1;
        }
    }
    if (threadIdx.x == 0) win_unique[w] = total;
    __syncthreads();

    // Every edge looks its column up in the sorted run (first position not below it).
    for (int e = threadIdx.x; e < cnt; e += THREADS) {
        int32_t c = ci[lo + e];
        int l = 0, h = cnt;
        while (l < h) {
            int mid = (l + h) >> 1;
            if (s_key[mid] < c) l = mid + 1; else h = mid;
        }
        edge_to_col[lo + e] = s_rank[l];
    }
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

// Large class when the column space fits: the same bitmap, but in LDS (gfx950 gives a workgroup up to
// 160 KB): one bit per column plus the running count in front of every group of kPfGroup words.
// Setting the bits and looking the ranks up are LDS operations instead of L2 atomics and gathers, and
// no device scratch has to be cleared.  Needs lds_bitmap_bytes(n_words) <= kLdsBitmapMax.
constexpr int kPfGroup = 8;
constexpr int kLdsBitmapFrom = 1024;
constexpr size_t kLdsBitmapMax = 160 * 1024 - 256;
inline size_t lds_bitmap_bytes(int64_t n_words)
{
    return (size_t)(n_words + (n_words + kPfGroup - 1) / kPfGroup + 1) * 4;
}

__global__ __launch_bounds__(kBitmapThreads) void sgt_window_lds_bitmap_kernel(
    int32_t n_rows, int32_t win_h, int32_t n_words, const int32_t *__restrict__ large_list,
    const int32_t *__restrict__ rp, const int32_t *__restrict__ ci, int32_t *__restrict__ edge_to_col,
    int32_t *__restrict__ tmp_clean, int32_t *__restrict__ win_unique)
{
    extern __shared__ uint32_t s_words[];          // bitmap, then the group prefixes
    __shared__ int s_tmp[kBitmapWaves + 1];
    uint32_t *bm = s_words;
    int32_t *gpf = reinterpret_cast<int32_t *>(s_words + n_words);
    const int64_t w = large_list[blockIdx.x];
    int32_t lo, hi;
    window_edge_range(rp, n_rows, win_h, w, &lo, &hi);

    // The first batch of columns is requested before the bitmap is cleared (its latency hides under the
    // clearing) and kept for step 4: windows of up to kBitmapThreads * kEdgeUnroll entries read their
    // columns once.
    uint32_t c_first[kEdgeUnroll];
#pragma unroll
    for (int u = 0; u < kEdgeUnroll; ++u) {
        const int64_t e = (int64_t)lo + threadIdx.x + (int64_t)u * kBitmapThreads;
        c_first[u] = e < hi ? (uint32_t)ci[e] : 0xFFFFFFFFu;
    }
    for (int32_t k = threadIdx.x; k < n_words; k += kBitmapThreads) bm[k] = 0u;
    __syncthreads();

    // 1. one bit per edge
#pragma unroll
    for (int u = 0; u < kEdgeUnroll; ++u)
        if (c_first[u] != 0xFFFFFFFFu) atomicOr(&bm[c_first[u] >> 5], 1u << (c_first[u] & 31));
    for (int64_t e0 = (int64_t)lo + (int64_t)kBitmapThreads * kEdgeUnroll + threadIdx.x; e0 < hi;
         e0 += (int64_t)kBitmapThreads * kEdgeUnroll) {
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
    __syncthreads();

    // 2. every thread owns a contiguous run of R words (R odd: the lanes of a wavefront then read
    //    different banks) and counts its bits; one workgroup-wide scan gives the count in front of
    //    every run.  (A scan per 64 words instead costs a chain of cross-lane steps per row.)
    const int32_t R = ((n_words + kBitmapThreads - 1) / kBitmapThreads) | 1;
    const int32_t kb = min((int32_t)threadIdx.x * R, n_words), ke = min(kb + R, n_words);
    int cnt = 0;
    for (int32_t k = kb; k < ke; ++k) cnt += __popc(bm[k]);
    int total;
    int pos = block_exclusive_scan(cnt, s_tmp, &total);

    // 3. the count in front of every group of words, and the unique list (bit positions ascending)
    for (int32_t k = kb; k < ke; ++k) {
        uint32_t bits = bm[k];
        if ((k % kPfGroup) == 0) gpf[k / kPfGroup] = pos;
        while (bits) {
            const int b = __ffs(bits) - 1;
            bits &= bits - 1;
            tmp_clean[lo + pos] = k * 32 + b;
            ++pos;
        }
    }
    if (threadIdx.x == 0) win_unique[w] = total;
    __syncthreads();

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
#pragma unroll
    for (int u = 0; u < kEdgeUnroll; ++u)
        if (c_first[u] != 0xFFFFFFFFu)
            edge_to_col[(int64_t)lo + threadIdx.x + (int64_t)u * kBitmapThreads] = rank_of(c_first[u]);
    for (int64_t e0 = (int64_t)lo + (int64_t)kBitmapThreads * kEdgeUnroll + threadIdx.x; e0 < hi;
         e0 += (int64_t)kBitmapThreads * kEdgeUnroll) {
        uint32_t c[kEdgeUnroll];
#pragma unroll
        for (int u = 0; u < kEdgeUnroll; ++u) {
            int64_t e = e0 + (int64_t)u * kBitmapThreads;
            c[u] = e < hi ? (uint32_t)ci[e] : 0u;
        }
#pragma unroll
        for (int u = 0; u < kEdgeUnroll; ++u) {
            int64_t e = e0 + (int64_t)u * kBitmapThreads;
            if (e < hi) edge_to_col[e] = rank_of(c[u]);
        }
    }
}

// Packs the per-window lists into col_to_row.  One wavefront per window; windows of the large
// class are copied by sgt_pack_large_kernel with many workgroups each.
__global__ __launch_bounds__(kWave) void sgt_pack_kernel(int32_t n_rows, int32_t win_h,
                                                         const int32_t *__restrict__ rp,
                                                         const int32_t *__restrict__ tmp_clean,
                                                         const int32_t *__restrict__ win_unique_ptr,
                                                         int32_t *__restrict__ col_to_row, int32_t medium_cap)
{
    const int64_t w = blockIdx.x;
    int32_t lo, hi;
    window_edge_range(rp, n_rows, win_h, w, &lo, &hi);
    const int32_t u0 = win_unique_ptr[w];
    const int32_t uw = win_unique_ptr[w + 1] - u0;
    if (hi - lo <= medium_cap)
        for (int k = threadIdx.x; k < uw; k += kWave) col_to_row[u0 + k] = tmp_clean[lo + k];
}

constexpr int kPackSplit = 16;   // workgroups per large window

__global__ __launch_bounds__(256) void sgt_pack_large_kernel(int32_t n_rows, int32_t win_h,
                                                             const int32_t *__restrict__ large_list,
                                                             const int32_t *__restrict__ rp,
                                                             const int32_t *__restrict__ tmp_clean,
                                                             const int32_t *__restrict__ win_unique_ptr,
                                                             int32_t *__restrict__ col_to_row)
{
    const int64_t w = large_list[blockIdx.x];
    int32_t lo, hi;
    window_edge_range(rp, n_rows, win_h, w, &lo, &hi);
    const int32_t u0 = win_unique_ptr[w];
    const int32_t uw = win_unique_ptr[w + 1] - u0;
    const int32_t chunk = (uw + kPackSplit - 1) / kPackSplit;
    const int32_t k0 = blockIdx.y * chunk;
    const int32_t k1 = min(k0 + chunk, uw);
    for (int32_t k = k0 + threadIdx.x; k < k1; k += 256) col_to_row[u0 + k] = tmp_clean[lo + k];
}

// ---- gather plan ------------------------------------------------------------------------------

__global__ void seg_count_kernel(int32_t n_rows, const int32_t *rp, int32_t *seg_cnt, int32_t *long_flag,
                                 int32_t *slot_cnt)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_rows) return;
    int32_t deg = rp[i + 1] - rp[i];
    int32_t segs = deg <= kSegLen ? 1 : (deg + kSegLen - 1) / kSegLen;
    seg_cnt[i] = segs;
    long_flag[i] = segs > 1;
    slot_cnt[i] = segs > 1 ? segs : 0;
}

__global__ void seg_fill_kernel(int32_t n_rows, const int32_t *rp, const int32_t *seg_off,
                                const int32_t *long_off, const int32_t *slot_off, int32_t *seg_row,
                                int32_t *seg_ebeg, int32_t *seg_dst, int32_t *long_row,
                                int32_t *long_slot_ptr, int64_t n_long)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_rows) return;
    int32_t s0 = seg_off[i], segs = seg_off[i + 1] - s0;
    int32_t e0 = rp[i];
    bool is_long = segs > 1;
    int32_t slot0 = slot_off[i];
    for (int32_t k = 0; k < segs; ++k) {
        seg_row[s0 + k] = (int32_t)i;
        seg_ebeg[s0 + k] = e0 + k * kSegLen;
        seg_dst[s0 + k] = is_long ? slot0 + k : -1;
    }
    if (is_long) {
        int32_t li = long_off[i];
        long_row[li] = (int32_t)i;
        long_slot_ptr[li] = slot0;
        if (li == n_long - 1) long_slot_ptr[n_long] = slot0 + segs;
    }
}

// ---- column bands: XCD-aware ordering of the segment list ---------------------------------------
// Each accelerator die has its own L2.  Segments of split (long) rows cover a narrow range of the
// row's columns, so sending all segments whose columns fall in the same band to the same die makes
// that die's L2 hold only its bands' X rows: the hot rows are cached once per chip instead of once per
// die.  The 2 * kXcds bands are chosen from a histogram of the split rows' segment start columns so
// that every band gets about the same number of segments; die l takes bands l and 2 * kXcds - 1 - l,
// which pairs a band of frequently used columns with a band of rarely used ones (on skewed graphs the
// popular columns are a narrow id range), so that the L2 misses -- and with them the traffic on each
// die's link to memory -- are spread evenly over the dies.  Single-segment rows are not banded; runs of
// them are dealt out to the dies round-robin.  Any grouping is correct: the order of the segment
// list only changes where a segment runs.
constexpr int kBands = 2 * kXcds;
constexpr int kHistBins = 8192;    // 32 KB of LDS per workgroup in band_hist_kernel

__device__ __forceinline__ int column_bin(int32_t c, int32_t n_cols)
{
    return (int)(((int64_t)c * kHistBins) / (n_cols > 0 ? n_cols : 1));
}

// Histogram of the split rows' segment start columns.  Start columns of hub rows pile up in a few
// bins, so every workgroup first counts in LDS and then adds its non-zero bins to the global array.
__global__ __launch_bounds__(256) void band_hist_kernel(int64_t n_seg, const int32_t *seg_dst,
                                                        const int32_t *seg_ebeg, const int32_t *ci,
                                                        int32_t n_cols, int32_t *hist)
{
    __shared__ int32_t s_hist[kHistBins];
    for (int b = threadIdx.x; b < kHistBins; b += blockDim.x) s_hist[b] = 0;
    __syncthreads();
    for (int64_t sgi = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; sgi < n_seg;
         sgi += (int64_t)gridDim.x * blockDim.x)
        if (seg_dst[sgi] >= 0) atomicAdd(&s_hist[column_bin(ci[seg_ebeg[sgi]], n_cols)], 1);
    __syncthreads();
    for (int b = threadIdx.x; b < kHistBins; b += blockDim.x)
        if (s_hist[b]) atomicAdd(&hist[b], s_hist[b]);
}

// Category of a segment in the final order: 0 .. kBands-1 = column band of a split row's segment;
// kBands + c = single-segment row of length class c.  With sort_tail the classes follow the number of
// gather iterations a row needs (longest first), so that the lane groups of a wavefront get rows of
// similar length; without it every single-segment row is class 0 and the tail stays in row order,
// which keeps the rows of a window next to each other (that matters when they share neighbours).
constexpr int kTailClasses = 8;
constexpr int kCats = kBands + kTailClasses;
constexpr int kPartThreads = 256;

__device__ __forceinline__ int segment_category(int64_t sgi, const int32_t *seg_row, const int32_t *seg_dst,
                                                const int32_t *seg_ebeg, const int32_t *rp, const int32_t *ci,
                                                int32_t n_cols, const int32_t *hist_excl, int sort_tail)
{
    if (seg_dst[sgi] >= 0) {
        const int64_t total = hist_excl[kHistBins];
        const int64_t before = hist_excl[column_bin(ci[seg_ebeg[sgi]], n_cols)];
        int b = (int)((before * kBands) / (total > 0 ? total : 1));
        return b > kBands - 1 ? kBands - 1 : b;
    }
    if (!sort_tail) return kBands;
    const int32_t r = seg_row[sgi];
    const int32_t deg = rp[r + 1] - rp[r];
    const int cls = deg > 96 ? 0 : deg > 64 ? 1 : deg > 48 ? 2 : deg > 32 ? 3 : deg > 24 ? 4 : deg > 16 ? 5 : deg > 8 ? 6 : 7;
    return kBands + cls;
}

// Pass 1 of the stable partition: category of every segment and per-workgroup category counts
// (block_cnt[cat * n_blocks + block]).
__global__ __launch_bounds__(kPartThreads) void cat_count_kernel(
    int64_t n_seg, const int32_t *seg_row, const int32_t *seg_dst, const int32_t *seg_ebeg, const int32_t *rp,
    const int32_t *ci, int32_t n_cols, const int32_t *hist_excl, int sort_tail, uint8_t *seg_cat,
    int32_t *block_cnt, int64_t n_blocks)
{
    __shared__ int s_cnt[kCats];
    if (threadIdx.x < kCats) s_cnt[threadIdx.x] = 0;
    __syncthreads();
    const int64_t sgi = (int64_t)blockIdx.x * kPartThreads + threadIdx.x;
    if (sgi < n_seg) {
        const int c = segment_category(sgi, seg_row, seg_dst, seg_ebeg, rp, ci, n_cols, hist_excl, sort_tail);
        seg_cat[sgi] = (uint8_t)c;
        atomicAdd(&s_cnt[c], 1);
    }
    __syncthreads();
    if (threadIdx.x < kCats) block_cnt[(int64_t)threadIdx.x * n_blocks + blockIdx.x] = s_cnt[threadIdx.x];
}

// Pass 2: block_off = exclusive scan of block_cnt (category-major = the final order).  Inside a
// workgroup a segment's rank among the segments of its category is found with wavefront ballots, so
// the partition is stable (row order is kept inside every category) and deterministic.
__global__ __launch_bounds__(kPartThreads) void cat_scatter_kernel(
    int64_t n_seg, const uint8_t *seg_cat, const int32_t *block_off, int64_t n_blocks, const int32_t *in_row,
    const int32_t *in_ebeg, const int32_t *in_dst, int32_t *out_row, int32_t *out_ebeg, int32_t *out_dst)
{
    __shared__ int s_wave_cnt[kPartThreads / kWave][kCats];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const int64_t sgi = (int64_t)blockIdx.x * kPartThreads + threadIdx.x;
    const int cat = sgi < n_seg ? (int)seg_cat[sgi] : -1;
    int rank_in_wave = 0;
    for (int c = 0; c < kCats; ++c) {
        const unsigned long long mask = __ballot(cat == c);
        if (lane == 0) s_wave_cnt[wave][c] = __popcll(mask);
        if (cat == c) rank_in_wave = __popcll(mask & ((1ull << lane) - 1ull));
    }
    __syncthreads();
    if (cat < 0) return;
    int32_t p = block_off[(int64_t)cat * n_blocks + blockIdx.x] + rank_in_wave;
    for (int w2 = 0; w2 < wave; ++w2) p += s_wave_cnt[w2][cat];
    out_row[p] = in_row[sgi];
    out_ebeg[p] = in_ebeg[sgi];
    out_dst[p] = in_dst[sgi];
}

// Ordering of the split rows' segments inside the bands: key = the leading kSegSortBits bits of a segment's
// start column (three passes of the radix sort; a finer order buys nothing).
constexpr int kSegSortBits = 12;
__global__ void seg_start_col_kernel(int64_t n, const int32_t *seg_ebeg, const int32_t *ci, int shift, int32_t *keys)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) keys[i] = ci[seg_ebeg[i]] >> shift;
}

__global__ void seg_permute_kernel(int64_t n, const int32_t *order, const int32_t *in_row, const int32_t *in_ebeg,
                                   const int32_t *in_dst, int32_t *out_row, int32_t *out_ebeg, int32_t *out_dst)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int32_t k = order[i];
    out_row[i] = in_row[k];
    out_ebeg[i] = in_ebeg[k];
    out_dst[i] = in_dst[k];
}

// lane_tab[kLaneTabStride * l] = {band l start, count, band (kBands-1-l) start, count, tail start,
// count} (see plan_segment()).  block_off == nullptr: no ordering, the whole list is the tail.
__global__ void lane_table_kernel(int64_t n_seg, const int32_t *block_off, int64_t n_blocks, int32_t *lane_tab)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    const int32_t u_start = block_off ? block_off[(int64_t)kBands * n_blocks] : 0;
    const int32_t u_count = (int32_t)n_seg - u_start;
    for (int l = 0; l < kXcds; ++l) {
        const int b2 = kBands - 1 - l;
        int32_t *t = lane_tab + kLaneTabStride * l;
        t[0] = block_off ? block_off[(int64_t)l * n_blocks] : 0;
        t[1] = block_off ? block_off[(int64_t)(l + 1) * n_blocks] - t[0] : 0;
        t[2] = block_off ? block_off[(int64_t)b2 * n_blocks] : 0;
        t[3] = block_off ? block_off[(int64_t)(b2 + 1) * n_blocks] - t[2] : 0;
        t[4] = u_start;
        t[5] = u_count;
    }
}

__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long v)
{
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// Per window: win_partition = ceil(U_w / tile_w) (Algorithm 1), the path flag under the given policy,
// and the totals (tiles, tile-path windows, their edges) with one atomic per wavefront.
__global__ __launch_bounds__(256) void choose_path_kernel(int32_t n_rows, int32_t win_h, int32_t tile_w,
                                                          int64_t n_win, const int32_t *rp,
                                                          const int32_t *win_unique_ptr, int policy,
                                                          float min_reuse, int32_t *win_partition,
                                                          uint8_t *win_path, unsigned long long *counts)
{
    const int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    unsigned long long tiles = 0, tile_win = 0, tile_nnz = 0, tile_many = 0, tile_unique = 0;
    if (w < n_win) {
        int32_t lo, hi;
        window_edge_range(rp, n_rows, win_h, w, &lo, &hi);
        const int32_t uw = win_unique_ptr[w + 1] - win_unique_ptr[w];
        const int32_t nnz_w = hi - lo;
        tiles = (unsigned long long)(((int64_t)uw + tile_w - 1) / tile_w);
        win_partition[w] = (int32_t)tiles;
        bool tile = false;
        if (policy == TCG_POLICY_TILE) tile = uw > 0;
        else if (policy == TCG_POLICY_AUTO)
            // Windows with shared neighbours, but not hub windows: the tile kernels keep a window's
            // condensed columns (or its whole condensed adjacency) in LDS, which needs compact windows.
            tile = (win_h == 16 || win_h == 32) && uw > 0 && uw <= kTileMaxUnique && (float)nnz_w >= min_reuse * (float)uw;
        // windows of 32 rows: class kTileFew only (twice the edges of a 16-row window fit in registers)
        if (win_h == 32 && policy == TCG_POLICY_AUTO && nnz_w > 2 * kTileFewEdges) tile = false;
        const bool many = tile && win_h == 16 && nnz_w > kTileFewEdges && uw <= kTileMaxUnique;
        win_path[w] = tile ? (many ? kTileMany : kTileFew) : 0;
        if (tile) {
            tile_win = 1;
            tile_nnz = (unsigned long long)nnz_w;
            tile_unique = (unsigned long long)uw;
        }
        if (many) {
            tile_many = 1;
            atomicMax(&counts[4], (unsigned long long)uw);
        }
    }
    tiles = wave_sum_u64(tiles);
    tile_win = wave_sum_u64(tile_win);
    tile_nnz = wave_sum_u64(tile_nnz);
    tile_many = wave_sum_u64(tile_many);
    tile_unique = wave_sum_u64(tile_unique);
    if ((threadIdx.x & (kWave - 1)) == 0) {
        if (tiles) atomicAdd(&counts[0], tiles);
        if (tile_win) atomicAdd(&counts[1], tile_win);
        if (tile_nnz) atomicAdd(&counts[2], tile_nnz);
        if (tile_many) atomicAdd(&counts[3], tile_many);
        if (tile_unique) atomicAdd(&counts[5], tile_unique);
    }
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
    if (n <= kScanBlock) {
        hipLaunchKernelGGL(scan_single_kernel, dim3(1), dim3(1024), 0, s, d_in, d_out, n);
        return launch_status("scan_single_kernel");
    }
    const int64_t nb = ceil_div(n, kScanBlock);
    hipLaunchKernelGGL(scan_block_sum_kernel, dim3((unsigned)nb), dim3(kScanThreads), 0, s, d_in, n, d_work);
    hipLaunchKernelGGL(scan_single_kernel, dim3(1), dim3(1024), 0, s, d_work, d_work, nb);
    hipLaunchKernelGGL(scan_apply_kernel, dim3((unsigned)nb), dim3(kScanThreads), 0, s, d_in, d_out, n, d_work, nb);
    return launch_status("scan kernels");
}

int choose_paths(tcg_meta *m, tcg_policy policy, float min_reuse, hipStream_t s)
{
    if (policy == TCG_POLICY_TILE && m->win_h != 16 && m->win_h != 32) return TCG_EINVAL;
    if (min_reuse <= 0.f) min_reuse = kDefaultMinReuse;
    // [0] tiles, [1] tile-path windows, [2] their edges, [3] windows of class kTileMany, [4] their widest,
    // [5] distinct columns summed over the tile-path windows
    unsigned long long *counts = m->d_counters;
    TCG_HIP(hipMemsetAsync(counts, 0, 6 * sizeof(unsigned long long), s));
    if (m->n_win > 0) {
        hipLaunchKernelGGL(choose_path_kernel, dim3((unsigned)ceil_div(m->n_win, 256)), dim3(256), 0, s,
                           m->n_rows, m->win_h, m->tile_w, m->n_win, m->d_row_ptr, m->d_win_unique_ptr,
                           (int)policy, min_reuse, m->d_win_partition, m->d_win_path, counts);
        TCG_TRY(launch_status("choose_path_kernel"));
    }
    unsigned long long h[6];
    TCG_HIP(hipMemcpyAsync(h, counts, sizeof(h), hipMemcpyDeviceToHost, s));
    TCG_HIP(hipStreamSynchronize(s));
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
        TCG_HIP(hipStreamSynchronize(s));
        m->n_tile_win = m->nnz_tile = m->n_tile_many = m->max_unique_many = m->unique_tile = 0;
    }
    return TCG_OK;
}

__global__ void collect3_kernel(const int32_t *a, const int32_t *b, const int32_t *c, int *out)
{
    if (threadIdx.x == 0) {
        out[0] = *a;
        out[1] = *b;
        out[2] = *c;
    }
}

int sgt_build_impl(tcg_meta *m, int validate, hipStream_t s)
{
    const int32_t n = m->n_rows;
    const int64_t nnz = m->nnz;
    const int64_t n_win = m->n_win;
    const int64_t scan_elems = scan_workspace_elems(std::max<int64_t>(n, n_win));
    // Windows above medium_cap entries form the large class (bitmap over the column space).  When that
    // bitmap fits in LDS it is cheaper than sorting from kLdsBitmapFrom entries on, so the class starts there.
    const bool lds_bitmap = lds_bitmap_bytes(ceil_div(m->n_cols, 32)) <= kLdsBitmapMax;
    const int32_t medium_cap = lds_bitmap ? std::min(kLdsBitmapFrom, kMediumCap) : kMediumCap;

    // Arena 0 (kept): the translated graph except col_to_row, the path flags, a few counters.
    Arena keep;
    keep.want(n_win * 4);             // win_partition
    keep.want((n_win + 1) * 4);       // win_unique_ptr
    keep.want(nnz * 4);               // edge_to_col
    keep.want(n_win);                 // win_path
    keep.want(8 * 8);                 // counters
    TCG_TRY(keep.commit());
    m->owned[m->n_owned++] = keep.base;
    m->d_win_partition = keep.take<int32_t>(n_win);
    m->d_win_unique_ptr = keep.take<int32_t>(n_win + 1);
    m->d_edge_to_col = keep.take<int32_t>(nnz);
    m->d_win_path = keep.take<uint8_t>(n_win);
    m->d_counters = keep.take<unsigned long long>(8);

    // Temporaries of the build.
    Arena tmp;
    tmp.want(nnz * 4);                // tmp_clean
    tmp.want((n_win + 1) * 4);        // win_unique
    tmp.want(4 * n_win * 4);          // class lists
    for (int i = 0; i < 3; ++i) tmp.want(((int64_t)n + 1) * 4);   // segment counts / offsets
    tmp.want(scan_elems * 4);         // scan workspace
    tmp.want(16 * 4);                 // class counts + validation flag
    TCG_TRY(tmp.commit());
    ScopedFree tmp_guard{tmp.base, s};
    int32_t *tmp_clean = tmp.take<int32_t>(nnz);
    int32_t *win_unique = tmp.take<int32_t>(n_win + 1);
    int32_t *lists = tmp.take<int32_t>(4 * n_win);
    int32_t *seg_off = tmp.take<int32_t>((int64_t)n + 1);
    int32_t *long_off = tmp.take<int32_t>((int64_t)n + 1);
    int32_t *slot_off = tmp.take<int32_t>((int64_t)n + 1);
    int32_t *scan_work = tmp.take<int32_t>(scan_elems);
    int *small_ints = tmp.take<int>(16);   // [0..3] class counts, [4..6] plan totals, [8] validation flag
    TCG_HIP(hipMemsetAsync(small_ints, 0, 16 * sizeof(int), s));

    if (validate) {
        int *flag = small_ints + 8;
        hipLaunchKernelGGL(validate_csr_kernel, dim3((unsigned)std::min<int64_t>(ceil_div((int64_t)n + 1, 256), 4096)),
                           dim3(256), 0, s, n, nnz, m->d_row_ptr, flag);
        TCG_TRY(launch_status("validate_csr_kernel"));
        int h = 0;
        TCG_HIP(hipMemcpyAsync(&h, flag, sizeof(int), hipMemcpyDeviceToHost, s));
        TCG_HIP(hipStreamSynchronize(s));
        if (h) return TCG_ECSR;  // do not touch col_idx through a broken row_ptr
        if (nnz > 0) {
            hipLaunchKernelGGL(validate_cols_kernel, dim3((unsigned)std::min<int64_t>(ceil_div(nnz, 256), 8192)),
                               dim3(256), 0, s, m->n_cols, nnz, m->d_col_idx, flag);
            TCG_TRY(launch_status("validate_cols_kernel"));
            TCG_HIP(hipMemcpyAsync(&h, flag, sizeof(int), hipMemcpyDeviceToHost, s));
            TCG_HIP(hipStreamSynchronize(s));
            if (h) return TCG_ECSR;
        }
    }

    // Window classes and segment counts (both depend on row_ptr only).
    if (n_win > 0) {
        hipLaunchKernelGGL(classify_windows_kernel, dim3((unsigned)ceil_div(n_win, 256)), dim3(256), 0, s, n,
                           m->win_h, n_win, m->d_row_ptr, lists, small_ints, win_unique, medium_cap);
        TCG_TRY(launch_status("classify_windows_kernel"));
    }
    if (n > 0) {
        hipLaunchKernelGGL(seg_count_kernel, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, s, n, m->d_row_ptr,
                           seg_off, long_off, slot_off);
        TCG_TRY(launch_status("seg_count_kernel"));
    }
    TCG_TRY(exclusive_scan_i32(seg_off, seg_off, n, scan_work, s));
    TCG_TRY(exclusive_scan_i32(long_off, long_off, n, scan_work, s));
    TCG_TRY(exclusive_scan_i32(slot_off, slot_off, n, scan_work, s));
    // One copy for everything the host needs here (every separate small copy costs tens of microseconds):
    // the three totals are collected next to the class counts first.
    hipLaunchKernelGGL(collect3_kernel, dim3(1), dim3(64), 0, s, seg_off + n, long_off + n, slot_off + n,
                       small_ints + 4);
    int h_small[7] = {0, 0, 0, 0, 0, 0, 0};
    TCG_HIP(hipMemcpyAsync(h_small, small_ints, sizeof(h_small), hipMemcpyDeviceToHost, s));
    TCG_HIP(hipStreamSynchronize(s));                                           // sync 1
    const int h_cls[4] = {h_small[0], h_small[1], h_small[2], h_small[3]};
    const int32_t h_plan[3] = {h_small[4], h_small[5], h_small[6]};
    m->n_seg = h_plan[0];
    m->n_long = h_plan[1];
    m->n_slots = h_plan[2];

    // Arena 1 (kept): the gather plan.
    Arena plan;
    plan.want(m->n_seg * 4);
    plan.want(m->n_seg * 4);
    plan.want(m->n_seg * 4);
    plan.want(m->n_long * 4);
    plan.want((m->n_long + 1) * 4);
    plan.want(kLaneTabStride * kXcds * 4);
    plan.want(m->n_slots * kPartialInitD * 4);   // partial sums of split rows for D <= kPartialInitD
    plan.want(m->n_slots * 2 * 4);               // (maximum, denominator) per split-row segment
    TCG_TRY(plan.commit());
    m->owned[m->n_owned++] = plan.base;
    m->d_seg_row = plan.take<int32_t>(m->n_seg);
    m->d_seg_ebeg = plan.take<int32_t>(m->n_seg);
    m->d_seg_dst = plan.take<int32_t>(m->n_seg);
    m->d_long_row = plan.take<int32_t>(m->n_long);
    m->d_long_slot_ptr = plan.take<int32_t>(m->n_long + 1);
    m->d_lane_tab = plan.take<int32_t>(kLaneTabStride * kXcds);
    m->d_partial = plan.take<float>(m->n_slots * kPartialInitD);
    m->partial_elems = m->n_slots * kPartialInitD;
    m->partial_owned = false;
    m->d_partial_ml = plan.take<float>(m->n_slots * 2);

    // Per-window translation, one launch per size class.
    if (h_cls[0] > 0)
        hipLaunchKernelGGL((sgt_window_lds_kernel<kWave, kTinyCap>), dim3((unsigned)h_cls[0]), dim3(kWave), 0, s, n,
                           m->win_h, lists, m->d_row_ptr, m->d_col_idx, m->d_edge_to_col, tmp_clean, win_unique);
    if (h_cls[1] > 0)
        hipLaunchKernelGGL((sgt_window_lds_kernel<256, kSmallCap>), dim3((unsigned)h_cls[1]), dim3(256), 0, s, n,
                           m->win_h, lists + n_win, m->d_row_ptr, m->d_col_idx, m->d_edge_to_col, tmp_clean,
                           win_unique);
    if (h_cls[2] > 0)
        hipLaunchKernelGGL((sgt_window_lds_kernel<256, kMediumCap>), dim3((unsigned)h_cls[2]), dim3(256), 0, s, n,
                           m->win_h, lists + 2 * n_win, m->d_row_ptr, m->d_col_idx, m->d_edge_to_col, tmp_clean,
                           win_unique);
    TCG_TRY(launch_status("sgt_window_lds_kernel"));
    ScopedFree bitmap_guard{nullptr, s};
    const int64_t n_words_all = ceil_div(m->n_cols, 32);
    if (h_cls[3] > 0 && lds_bitmap_bytes(n_words_all) <= kLdsBitmapMax) {
        const size_t lds = lds_bitmap_bytes(n_words_all);
        static bool raised = false;       // more than 64 KB of dynamic LDS has to be asked for once
        if (!raised) {
            TCG_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(sgt_window_lds_bitmap_kernel),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBitmapMax));
            raised = true;
        }
        hipLaunchKernelGGL(sgt_window_lds_bitmap_kernel, dim3((unsigned)h_cls[3]), dim3(kBitmapThreads), lds, s, n,
                           m->win_h, (int32_t)n_words_all, lists + 3 * n_win, m->d_row_ptr, m->d_col_idx,
                           m->d_edge_to_col, tmp_clean, win_unique);
        TCG_TRY(launch_status("sgt_window_lds_bitmap_kernel"));
    } else if (h_cls[3] > 0) {
        const int64_t n_large = h_cls[3];
        const int64_t n_words = n_words_all;
        const int64_t budget_words = (int64_t)(128ll << 20) / 4;  // 128 MiB per scratch array
        const int64_t batch = std::max<int64_t>(1, std::min<int64_t>(n_large, budget_words / n_words));
        uint32_t *bitmap = nullptr;
        TCG_TRY(dev_alloc(&bitmap, 2 * batch * n_words));
        bitmap_guard.p = bitmap;
        int32_t *prefix = reinterpret_cast<int32_t *>(bitmap + batch * n_words);
        for (int64_t b0 = 0; b0 < n_large; b0 += batch) {
            const int64_t nb = std::min<int64_t>(batch, n_large - b0);
            TCG_HIP(hipMemsetAsync(bitmap, 0, (size_t)(nb * n_words) * sizeof(uint32_t), s));
            hipLaunchKernelGGL(sgt_window_bitmap_kernel, dim3((unsigned)nb), dim3(kBitmapThreads), 0, s, n,
                               m->win_h, n_words, lists + 3 * n_win + b0, m->d_row_ptr, m->d_col_idx, bitmap,
                               prefix, m->d_edge_to_col, tmp_clean, win_unique);
            TCG_TRY(launch_status("sgt_window_bitmap_kernel"));
        }
    }

    TCG_TRY(exclusive_scan_i32(win_unique, m->d_win_unique_ptr, n_win, scan_work, s));
    int32_t total_unique = 0;
    TCG_HIP(hipMemcpyAsync(&total_unique, m->d_win_unique_ptr + n_win, sizeof(int32_t), hipMemcpyDeviceToHost, s));
    TCG_HIP(hipStreamSynchronize(s));                                           // sync 2
    m->total_unique = total_unique;

    // Segment list: row order first, then a stable partition into column bands (split rows) and the
    // tail of single-segment rows.  When the windows share few neighbours (U close to nnz) the tail is
    // ordered by row length as well; otherwise it keeps the row order.
    const int64_t n_pblocks = ceil_div(std::max<int64_t>(m->n_seg, 1), kPartThreads);
    const int sort_tail = (double)m->total_unique > 0.75 * (double)std::max<int64_t>(nnz, 1) ? 1 : 0;
    const bool ordered = (m->n_slots > 0 || sort_tail) && (int64_t)kCats * n_pblocks + 1 < (int64_t)INT32_MAX;
    Arena ptmp;
    const int64_t cnt_elems = (int64_t)kCats * n_pblocks + 1;
    const int64_t pscan_elems = scan_workspace_elems(std::max<int64_t>(cnt_elems, kHistBins));
    if (ordered) {
        for (int i = 0; i < 3; ++i) ptmp.want(m->n_seg * 4);
        ptmp.want(m->n_seg);
        ptmp.want(cnt_elems * 4);
        ptmp.want((kHistBins + 1) * 4);
        ptmp.want(pscan_elems * 4);
        TCG_TRY(ptmp.commit());
    }
    ScopedFree ptmp_guard{ptmp.base, s};
    if (n > 0) {
        int32_t *row_o = m->d_seg_row, *ebeg_o = m->d_seg_ebeg, *dst_o = m->d_seg_dst;
        if (ordered) {
            row_o = ptmp.take<int32_t>(m->n_seg);
            ebeg_o = ptmp.take<int32_t>(m->n_seg);
            dst_o = ptmp.take<int32_t>(m->n_seg);
        }
        hipLaunchKernelGGL(seg_fill_kernel, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, s, n, m->d_row_ptr,
                           seg_off, long_off, slot_off, row_o, ebeg_o, dst_o, m->d_long_row, m->d_long_slot_ptr,
                           m->n_long);
        TCG_TRY(launch_status("seg_fill_kernel"));
        if (ordered) {
            uint8_t *seg_cat = ptmp.take<uint8_t>(m->n_seg);
            int32_t *block_cnt = ptmp.take<int32_t>(cnt_elems);
            int32_t *hist = ptmp.take<int32_t>(kHistBins + 1);
            int32_t *pscan = ptmp.take<int32_t>(pscan_elems);
            const unsigned sgrid = (unsigned)n_pblocks;
            TCG_HIP(hipMemsetAsync(hist, 0, (kHistBins + 1) * sizeof(int32_t), s));
            hipLaunchKernelGGL(band_hist_kernel, dim3(std::min<unsigned>(sgrid, 512u)), dim3(256), 0, s, m->n_seg, dst_o,
                               ebeg_o, m->d_col_idx, m->n_cols, hist);
            TCG_TRY(exclusive_scan_i32(hist, hist, kHistBins, pscan, s));
            hipLaunchKernelGGL(cat_count_kernel, dim3(sgrid), dim3(kPartThreads), 0, s, m->n_seg, row_o, dst_o, ebeg_o,
                               m->d_row_ptr, m->d_col_idx, m->n_cols, hist, sort_tail, seg_cat, block_cnt, n_pblocks);
            TCG_TRY(exclusive_scan_i32(block_cnt, block_cnt, cnt_elems - 1, pscan, s));
            hipLaunchKernelGGL(cat_scatter_kernel, dim3(sgrid), dim3(kPartThreads), 0, s, m->n_seg, seg_cat, block_cnt,
                               n_pblocks, row_o, ebeg_o, dst_o, m->d_seg_row, m->d_seg_ebeg, m->d_seg_dst);
            hipLaunchKernelGGL(lane_table_kernel, dim3(1), dim3(64), 0, s, m->n_seg, block_cnt, n_pblocks, m->d_lane_tab);
            TCG_TRY(launch_status("segment ordering kernels"));
            // Inside the bands: by start column (the bands are ranges of start columns, so one stable sort of all
            // split-row segments keeps them in place).  Segments that run one after the other on a die then
            // read neighbouring -- on skewed graphs largely the same -- X rows.
            const int64_t ns = m->n_slots;
            if (ns > 1 && radix_sort_scratch_bytes(ns) > 0) {
                const size_t arr = ((size_t)ns * 4 + 255) & ~(size_t)255;
                PoolBuf sb;
                sb.s = s;
                TCG_TRY(pool_alloc(&sb.p, 7 * arr + radix_sort_scratch_bytes(ns)));
                char *base = static_cast<char *>(sb.p);
                int32_t *keys = reinterpret_cast<int32_t *>(base), *keys_o = reinterpret_cast<int32_t *>(base + arr),
                        *order = reinterpret_cast<int32_t *>(base + 2 * arr), *t_row = reinterpret_cast<int32_t *>(base + 3 * arr),
                        *t_ebeg = reinterpret_cast<int32_t *>(base + 4 * arr), *t_dst = reinterpret_cast<int32_t *>(base + 5 * arr);
                void *sort_scratch = base + 7 * arr;
                int bits = 1;
                while (bits < 31 && ((int64_t)1 << bits) < (int64_t)m->n_cols) ++bits;
                const int shift = bits > kSegSortBits ? bits - kSegSortBits : 0;   // the leading bits are enough
                const unsigned g = (unsigned)ceil_div(ns, 256);
                hipLaunchKernelGGL(seg_start_col_kernel, dim3(g), dim3(256), 0, s, ns, m->d_seg_ebeg, m->d_col_idx, shift,
                                   keys);
                TCG_TRY(radix_sort_pairs(keys, nullptr, ns, bits - shift, keys_o, order, sort_scratch, s));
                hipLaunchKernelGGL(seg_permute_kernel, dim3(g), dim3(256), 0, s, ns, order, m->d_seg_row, m->d_seg_ebeg,
                                   m->d_seg_dst, t_row, t_ebeg, t_dst);
                TCG_HIP(hipMemcpyAsync(m->d_seg_row, t_row, (size_t)ns * 4, hipMemcpyDeviceToDevice, s));
                TCG_HIP(hipMemcpyAsync(m->d_seg_ebeg, t_ebeg, (size_t)ns * 4, hipMemcpyDeviceToDevice, s));
                TCG_HIP(hipMemcpyAsync(m->d_seg_dst, t_dst, (size_t)ns * 4, hipMemcpyDeviceToDevice, s));
                TCG_TRY(launch_status("segment sort kernels"));
            }                                   // sb waits for the stream and returns the buffer
        }
    }
    if (!ordered) {
        hipLaunchKernelGGL(lane_table_kernel, dim3(1), dim3(64), 0, s, m->n_seg, (const int32_t *)nullptr, (int64_t)0,
                           m->d_lane_tab);
        TCG_TRY(launch_status("lane_table_kernel"));
    }
    TCG_HIP(hipMemcpyAsync(m->h_lane_tab, m->d_lane_tab, sizeof(m->h_lane_tab), hipMemcpyDeviceToHost, s));

    TCG_TRY(dev_alloc(&m->d_col_to_row, m->total_unique));
    m->owned[m->n_owned++] = m->d_col_to_row;
    if (n_win > 0) {
        hipLaunchKernelGGL(sgt_pack_kernel, dim3((unsigned)n_win), dim3(kWave), 0, s, n, m->win_h, m->d_row_ptr,
                           tmp_clean, m->d_win_unique_ptr, m->d_col_to_row, medium_cap);
        TCG_TRY(launch_status("sgt_pack_kernel"));
        if (h_cls[3] > 0) {
            hipLaunchKernelGGL(sgt_pack_large_kernel, dim3((unsigned)h_cls[3], kPackSplit), dim3(256), 0, s, n,
                               m->win_h, lists + 3 * n_win, m->d_row_ptr, tmp_clean, m->d_win_unique_ptr,
                               m->d_col_to_row);
            TCG_TRY(launch_status("sgt_pack_large_kernel"));
        }
    }
    TCG_TRY(choose_paths(m, TCG_POLICY_AUTO, 0.f, s));                          // sync 3
    return TCG_OK;   // temporaries are freed by the guards; the stream is idle here
}

}  // namespace tcg
