// Sparse Graph Translation on the GPU (Algorithm 1 and section 4.1 of the paper) and the
// execution plan derived from it.
//
// The paper notes that row windows are independent, so each window is translated by one
// workgroup.  Three size classes, all producing the same canonical result (ascending unique
// column list, rank of every edge's column in it):
//   small  (<= 1024 edges)   sort in LDS with a bitonic network, 256 threads
//   medium (<= 4096 edges)   same, 1024 threads, 32 KB of LDS
//   large  (>  4096 edges)   a bitmap over the column space in device scratch: set a bit per
//                            edge, prefix-popcount the words, rank = prefix + popcount below.
//                            Hub windows of power-law graphs land here; the cost is
//                            O(n_cols / 32 + nnz_w) per window.
// Every window first writes its unique list at its own edge offset of a temporary array (the
// list is never longer than the window's edge range); once all U_w are known a prefix sum gives
// win_unique_ptr and the lists are packed into col_to_row.
#include "common.h"

#include <limits.h>

#include <algorithm>

namespace tcg {

namespace {

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
    const int nw = blockDim.x >> 6;
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

constexpr int kScanThreads = 1024;
constexpr int kScanItems = 4;

__global__ __launch_bounds__(kScanThreads) void scan_kernel(const int32_t *in, int32_t *out, int64_t n)
{
    __shared__ int tmp[kScanThreads / kWave + 1];
    int carry = 0;
    for (int64_t base = 0; base < n; base += (int64_t)kScanThreads * kScanItems) {
        int64_t i0 = base + (int64_t)threadIdx.x * kScanItems;
        int v[kScanItems];
        int sum = 0;
#pragma unroll
        for (int k = 0; k < kScanItems; ++k) {
            v[k] = (i0 + k < n) ? in[i0 + k] : 0;
            sum += v[k];
        }
        int total;
        int run = carry + block_exclusive_scan(sum, tmp, &total);
#pragma unroll
        for (int k = 0; k < kScanItems; ++k) {
            if (i0 + k < n) out[i0 + k] = run;
            run += v[k];
        }
        carry += total;
    }
    if (threadIdx.x == 0) out[n] = carry;
}

// CSR sanity check: flag bit 0 = row_ptr ends wrong, bit 1 = not monotone, bit 2 = column range.
__global__ void validate_csr_kernel(int32_t n_rows, int32_t n_cols, int64_t nnz, const int32_t *rp,
                                    const int32_t *ci, int *flag)
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

// Appends the windows of the large class to a list (order is irrelevant: each window's result
// only depends on the window).
__global__ void collect_large_kernel(int32_t n_rows, int32_t win_h, int64_t n_win, const int32_t *rp,
                                     int32_t *large_list, int *n_large)
{
    int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (w >= n_win) return;
    int32_t lo, hi;
    window_edge_range(rp, n_rows, win_h, w, &lo, &hi);
    if (hi - lo > kMediumCap) large_list[atomicAdd(n_large, 1)] = (int32_t)w;
}

// Small and medium classes.  One workgroup per window; windows of another class return at once.
template <int THREADS, int CAP, int MIN_EXCL>
__global__ __launch_bounds__(THREADS) void sgt_window_lds_kernel(
    int32_t n_rows, int32_t win_h, const int32_t *rp, const int32_t *ci, int32_t *edge_to_col,
    int32_t *tmp_clean, int32_t *win_unique)
{
    __shared__ int32_t s_key[CAP];
    __shared__ int32_t s_rank[CAP];
    __shared__ int s_tmp[THREADS / kWave + 1];

    const int64_t w = blockIdx.x;
    int32_t lo, hi;
    window_edge_range(rp, n_rows, win_h, w, &lo, &hi);
    const int cnt = hi - lo;
    if (cnt <= MIN_EXCL || cnt > CAP) {
        if (cnt == 0 && MIN_EXCL == 0 && threadIdx.x == 0) win_unique[w] = 0;
        return;
    }
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
// entry; `prefix` is plain scratch; both hold n_words entries per workgroup.
constexpr int kBitmapThreads = 1024;

__global__ __launch_bounds__(kBitmapThreads) void sgt_window_bitmap_kernel(
    int32_t n_rows, int32_t win_h, int64_t n_words, const int32_t *large_list, const int32_t *rp,
    const int32_t *ci, uint32_t *bitmap, int32_t *prefix, int32_t *edge_to_col, int32_t *tmp_clean,
    int32_t *win_unique)
{
    __shared__ int s_tmp[kBitmapThreads / kWave + 1];
    const int64_t w = large_list[blockIdx.x];
    uint32_t *bm = bitmap + (int64_t)blockIdx.x * n_words;
    int32_t *pf = prefix + (int64_t)blockIdx.x * n_words;
    int32_t lo, hi;
    window_edge_range(rp, n_rows, win_h, w, &lo, &hi);

    for (int64_t e = lo + threadIdx.x; e < hi; e += kBitmapThreads) {
        uint32_t c = (uint32_t)ci[e];
        atomicOr(&bm[c >> 5], 1u << (c & 31));
    }
    __threadfence();
    __syncthreads();

    const int64_t wpt = (n_words + kBitmapThreads - 1) / kBitmapThreads;
    const int64_t w0 = (int64_t)threadIdx.x * wpt;
    int local = 0;
    for (int64_t k = w0; k < w0 + wpt && k < n_words; ++k)
        local += __popc(__hip_atomic_load(&bm[k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    int total;
    int run = block_exclusive_scan(local, s_tmp, &total);
    for (int64_t k = w0; k < w0 + wpt && k < n_words; ++k) {
        uint32_t bits = __hip_atomic_load(&bm[k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        pf[k] = run;
        int pos = run;
        while (bits) {
            int b = __ffs(bits) - 1;
            bits &= bits - 1;
            tmp_clean[lo + pos] = (int32_t)(k * 32 + b);
            ++pos;
        }
        run = pos;
    }
    if (threadIdx.x == 0) win_unique[w] = total;
    __threadfence();
    __syncthreads();

    for (int64_t e = lo + threadIdx.x; e < hi; e += kBitmapThreads) {
        uint32_t c = (uint32_t)ci[e];
        uint32_t bits = __hip_atomic_load(&bm[c >> 5], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        int32_t base = __hip_atomic_load(&pf[c >> 5], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        edge_to_col[e] = base + __popc(bits & ((1u << (c & 31)) - 1u));
    }
}

// Packs the per-window lists into col_to_row and derives win_partition (ceil(U_w / tile_w)).
__global__ __launch_bounds__(256) void sgt_pack_kernel(int32_t n_rows, int32_t win_h, int32_t tile_w,
                                                       const int32_t *rp, const int32_t *tmp_clean,
                                                       const int32_t *win_unique_ptr, int32_t *col_to_row,
                                                       int32_t *win_partition,
                                                       unsigned long long *total_tiles)
{
    const int64_t w = blockIdx.x;
    int32_t lo, hi;
    window_edge_range(rp, n_rows, win_h, w, &lo, &hi);
    const int32_t u0 = win_unique_ptr[w];
    const int32_t uw = win_unique_ptr[w + 1] - u0;
    for (int k = threadIdx.x; k < uw; k += blockDim.x) col_to_row[u0 + k] = tmp_clean[lo + k];
    if (threadIdx.x == 0) {
        int32_t tiles = (int32_t)(((int64_t)uw + tile_w - 1) / tile_w);
        win_partition[w] = tiles;
        if (tiles) atomicAdd(total_tiles, (unsigned long long)tiles);
    }
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
    if (i >= n_rows) {
        return;
    }
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

__global__ void choose_path_kernel(int32_t n_rows, int32_t win_h, int64_t n_win, const int32_t *rp,
                                   const int32_t *win_unique_ptr, int policy, float min_reuse,
                                   uint8_t *win_path, unsigned long long *counts)
{
    int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (w >= n_win) return;
    int32_t lo, hi;
    window_edge_range(rp, n_rows, win_h, w, &lo, &hi);
    int32_t uw = win_unique_ptr[w + 1] - win_unique_ptr[w];
    int32_t nnz_w = hi - lo;
    bool tile = false;
    if (policy == TCG_POLICY_TILE) tile = uw > 0;
    else if (policy == TCG_POLICY_AUTO) tile = win_h == 16 && uw > 0 && (float)nnz_w >= min_reuse * (float)uw;
    win_path[w] = tile ? 1 : 0;
    if (tile) {
        atomicAdd(&counts[0], 1ull);
        atomicAdd(&counts[1], (unsigned long long)nnz_w);
    }
}

template <typename T>
struct DevBuf {  // frees on scope exit unless released
    T *p = nullptr;
    ~DevBuf() { if (p) (void)hipFree(p); }
    T *release() { T *q = p; p = nullptr; return q; }
};

}  // namespace

int exclusive_scan_i32(const int32_t *d_in, int32_t *d_out, int64_t n, hipStream_t s)
{
    hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(kScanThreads), 0, s, d_in, d_out, n);
    return launch_status("scan_kernel");
}

static int build_gather_plan(tcg_meta *m, hipStream_t s)
{
    const int32_t n = m->n_rows;
    DevBuf<int32_t> seg_off, long_off, slot_off;
    TCG_TRY(dev_alloc(&seg_off.p, (int64_t)n + 1));
    TCG_TRY(dev_alloc(&long_off.p, (int64_t)n + 1));
    TCG_TRY(dev_alloc(&slot_off.p, (int64_t)n + 1));
    if (n > 0) {
        hipLaunchKernelGGL(seg_count_kernel, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, s, n,
                           m->d_row_ptr, seg_off.p, long_off.p, slot_off.p);
        TCG_TRY(launch_status("seg_count_kernel"));
    }
    TCG_TRY(exclusive_scan_i32(seg_off.p, seg_off.p, n, s));
    TCG_TRY(exclusive_scan_i32(long_off.p, long_off.p, n, s));
    TCG_TRY(exclusive_scan_i32(slot_off.p, slot_off.p, n, s));
    int32_t totals[3];
    TCG_HIP(hipMemcpyAsync(&totals[0], seg_off.p + n, sizeof(int32_t), hipMemcpyDeviceToHost, s));
    TCG_HIP(hipMemcpyAsync(&totals[1], long_off.p + n, sizeof(int32_t), hipMemcpyDeviceToHost, s));
    TCG_HIP(hipMemcpyAsync(&totals[2], slot_off.p + n, sizeof(int32_t), hipMemcpyDeviceToHost, s));
    TCG_HIP(hipStreamSynchronize(s));
    m->n_seg = totals[0];
    m->n_long = totals[1];
    m->n_slots = totals[2];
    TCG_TRY(dev_alloc(&m->d_seg_row, m->n_seg));
    TCG_TRY(dev_alloc(&m->d_seg_ebeg, m->n_seg));
    TCG_TRY(dev_alloc(&m->d_seg_dst, m->n_seg));
    TCG_TRY(dev_alloc(&m->d_long_row, m->n_long));
    TCG_TRY(dev_alloc(&m->d_long_slot_ptr, m->n_long + 1));
    if (n > 0) {
        hipLaunchKernelGGL(seg_fill_kernel, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, s, n,
                           m->d_row_ptr, seg_off.p, long_off.p, slot_off.p, m->d_seg_row, m->d_seg_ebeg,
                           m->d_seg_dst, m->d_long_row, m->d_long_slot_ptr, m->n_long);
        TCG_TRY(launch_status("seg_fill_kernel"));
    }
    TCG_HIP(hipStreamSynchronize(s));  // temporaries are freed on return
    return TCG_OK;
}

int choose_paths(tcg_meta *m, tcg_policy policy, float min_reuse, hipStream_t s)
{
    if (policy == TCG_POLICY_TILE && m->win_h != 16) return TCG_EINVAL;
    if (min_reuse <= 0.f) min_reuse = kDefaultMinReuse;
    DevBuf<unsigned long long> counts;
    TCG_TRY(dev_alloc(&counts.p, 2));
    TCG_HIP(hipMemsetAsync(counts.p, 0, 2 * sizeof(unsigned long long), s));
    if (m->n_win > 0) {
        hipLaunchKernelGGL(choose_path_kernel, dim3((unsigned)ceil_div(m->n_win, 256)), dim3(256), 0, s,
                           m->n_rows, m->win_h, m->n_win, m->d_row_ptr, m->d_win_unique_ptr, (int)policy,
                           min_reuse, m->d_win_path, counts.p);
        TCG_TRY(launch_status("choose_path_kernel"));
    }
    unsigned long long h[2];
    TCG_HIP(hipMemcpyAsync(h, counts.p, sizeof(h), hipMemcpyDeviceToHost, s));
    TCG_HIP(hipStreamSynchronize(s));
    m->policy = policy;
    m->min_reuse = min_reuse;
    m->n_tile_win = (int64_t)h[0];
    m->nnz_tile = (int64_t)h[1];
    return TCG_OK;
}

int sgt_build_impl(tcg_meta *m, int validate, hipStream_t s)
{
    const int32_t n = m->n_rows;
    const int64_t nnz = m->nnz;
    const int64_t n_win = m->n_win;

    if (validate) {
        DevBuf<int> flag;
        TCG_TRY(dev_alloc(&flag.p, 1));
        TCG_HIP(hipMemsetAsync(flag.p, 0, sizeof(int), s));
        hipLaunchKernelGGL(validate_csr_kernel, dim3((unsigned)std::min<int64_t>(ceil_div(n + 1, 256), 4096)),
                           dim3(256), 0, s, n, m->n_cols, nnz, m->d_row_ptr, m->d_col_idx, flag.p);
        TCG_TRY(launch_status("validate_csr_kernel"));
        int h = 0;
        TCG_HIP(hipMemcpyAsync(&h, flag.p, sizeof(int), hipMemcpyDeviceToHost, s));
        TCG_HIP(hipStreamSynchronize(s));
        if (h) return TCG_ECSR;  // do not touch col_idx through a broken row_ptr
        if (nnz > 0) {
            hipLaunchKernelGGL(validate_cols_kernel, dim3((unsigned)std::min<int64_t>(ceil_div(nnz, 256), 8192)),
                               dim3(256), 0, s, m->n_cols, nnz, m->d_col_idx, flag.p);
            TCG_TRY(launch_status("validate_cols_kernel"));
        }
        TCG_HIP(hipMemcpyAsync(&h, flag.p, sizeof(int), hipMemcpyDeviceToHost, s));
        TCG_HIP(hipStreamSynchronize(s));
        if (h) return TCG_ECSR;
    }

    TCG_TRY(dev_alloc(&m->d_win_partition, n_win));
    TCG_TRY(dev_alloc(&m->d_win_unique_ptr, n_win + 1));
    TCG_TRY(dev_alloc(&m->d_edge_to_col, nnz));
    TCG_TRY(dev_alloc(&m->d_win_path, n_win));

    DevBuf<int32_t> tmp_clean, win_unique, large_list;
    DevBuf<int> n_large_dev;
    DevBuf<unsigned long long> tiles_dev;
    TCG_TRY(dev_alloc(&tmp_clean.p, nnz));
    TCG_TRY(dev_alloc(&win_unique.p, n_win + 1));
    TCG_TRY(dev_alloc(&large_list.p, n_win));
    TCG_TRY(dev_alloc(&n_large_dev.p, 1));
    TCG_TRY(dev_alloc(&tiles_dev.p, 1));
    TCG_HIP(hipMemsetAsync(n_large_dev.p, 0, sizeof(int), s));
    TCG_HIP(hipMemsetAsync(tiles_dev.p, 0, sizeof(unsigned long long), s));

    int n_large = 0;
    if (n_win > 0) {
        hipLaunchKernelGGL(collect_large_kernel, dim3((unsigned)ceil_div(n_win, 256)), dim3(256), 0, s, n,
                           m->win_h, n_win, m->d_row_ptr, large_list.p, n_large_dev.p);
        TCG_TRY(launch_status("collect_large_kernel"));
        hipLaunchKernelGGL((sgt_window_lds_kernel<256, kSmallCap, 0>), dim3((unsigned)n_win), dim3(256), 0, s,
                           n, m->win_h, m->d_row_ptr, m->d_col_idx, m->d_edge_to_col, tmp_clean.p,
                           win_unique.p);
        TCG_TRY(launch_status("sgt_window_lds_kernel<small>"));
        hipLaunchKernelGGL((sgt_window_lds_kernel<1024, kMediumCap, kSmallCap>), dim3((unsigned)n_win),
                           dim3(1024), 0, s, n, m->win_h, m->d_row_ptr, m->d_col_idx, m->d_edge_to_col,
                           tmp_clean.p, win_unique.p);
        TCG_TRY(launch_status("sgt_window_lds_kernel<medium>"));
        TCG_HIP(hipMemcpyAsync(&n_large, n_large_dev.p, sizeof(int), hipMemcpyDeviceToHost, s));
        TCG_HIP(hipStreamSynchronize(s));
    }
    if (n_large > 0) {
        const int64_t n_words = ceil_div(m->n_cols, 32);
        const int64_t budget_words = (int64_t)(64ll << 20) / 4;  // 64 MiB per scratch array
        int64_t batch = std::max<int64_t>(1, std::min<int64_t>(n_large, budget_words / n_words));
        DevBuf<uint32_t> bitmap;
        DevBuf<int32_t> prefix;
        TCG_TRY(dev_alloc(&bitmap.p, batch * n_words));
        TCG_TRY(dev_alloc(&prefix.p, batch * n_words));
        for (int64_t b0 = 0; b0 < n_large; b0 += batch) {
            int64_t nb = std::min<int64_t>(batch, n_large - b0);
            TCG_HIP(hipMemsetAsync(bitmap.p, 0, (size_t)(nb * n_words) * sizeof(uint32_t), s));
            hipLaunchKernelGGL(sgt_window_bitmap_kernel, dim3((unsigned)nb), dim3(kBitmapThreads), 0, s, n,
                               m->win_h, n_words, large_list.p + b0, m->d_row_ptr, m->d_col_idx, bitmap.p,
                               prefix.p, m->d_edge_to_col, tmp_clean.p, win_unique.p);
            TCG_TRY(launch_status("sgt_window_bitmap_kernel"));
        }
        TCG_HIP(hipStreamSynchronize(s));  // scratch is freed on scope exit
    }

    TCG_TRY(exclusive_scan_i32(win_unique.p, m->d_win_unique_ptr, n_win, s));
    int32_t total_unique = 0;
    TCG_HIP(hipMemcpyAsync(&total_unique, m->d_win_unique_ptr + n_win, sizeof(int32_t),
                           hipMemcpyDeviceToHost, s));
    TCG_HIP(hipStreamSynchronize(s));
    m->total_unique = total_unique;
    TCG_TRY(dev_alloc(&m->d_col_to_row, m->total_unique));
    if (n_win > 0) {
        hipLaunchKernelGGL(sgt_pack_kernel, dim3((unsigned)n_win), dim3(256), 0, s, n, m->win_h, m->tile_w,
                           m->d_row_ptr, tmp_clean.p, m->d_win_unique_ptr, m->d_col_to_row,
                           m->d_win_partition, tiles_dev.p);
        TCG_TRY(launch_status("sgt_pack_kernel"));
    }
    unsigned long long tiles = 0;
    TCG_HIP(hipMemcpyAsync(&tiles, tiles_dev.p, sizeof(tiles), hipMemcpyDeviceToHost, s));
    TCG_HIP(hipStreamSynchronize(s));
    m->total_tiles = (int64_t)tiles;

    TCG_TRY(build_gather_plan(m, s));
    TCG_TRY(choose_paths(m, TCG_POLICY_AUTO, 0.f, s));
    return TCG_OK;
}

}  // namespace tcg
