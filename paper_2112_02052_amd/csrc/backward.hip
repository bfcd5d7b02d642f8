// Building blocks of the backward pass.  The paper trains GNNs with these sparse operations
// (section 4) without spelling the gradients out; by the chain rule on Equations 1 and 2:
//   Y = (w (.) A) X :   dX = (w (.) A)^T dY            tcg_spmm on the transposed structure, w permuted
//                       dw[e] = < dY[row(e)], X[col(e)] >   tcg_sddmm_pq(P = dY, Q = X)
//   out[e] = <x_i,x_j>: dX = (g (.) A) X + (g (.) A)^T X    two tcg_spmm calls (g = d out)
//   p = row_softmax(v): dv[e] = p[e] (dp[e] - sum_row p dp)  tcg_row_softmax_backward
// This file holds the CSR transpose (a stable least-significant-digit radix sort of the entries by
// column, 4 bits per pass, so the result is unique and deterministic), the edge-value permutation
// and the softmax gradient.
#include "common.h"

namespace tcg {

namespace {

constexpr int kThreads = 256;
constexpr int kDigits = 16;   // 4-bit radix

// Pass 1 of a radix step: per-workgroup digit counts, block_cnt[digit * n_blocks + block].
__global__ __launch_bounds__(kThreads) void radix_count_kernel(const int32_t *__restrict__ keys, int64_t n,
                                                               int shift, int32_t *__restrict__ block_cnt,
                                                               int64_t n_blocks)
{
    __shared__ int s_cnt[kDigits];
    if (threadIdx.x < kDigits) s_cnt[threadIdx.x] = 0;
    __syncthreads();
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n) atomicAdd(&s_cnt[(keys[i] >> shift) & (kDigits - 1)], 1);
    __syncthreads();
    if (threadIdx.x < kDigits) block_cnt[(int64_t)threadIdx.x * n_blocks + blockIdx.x] = s_cnt[threadIdx.x];
}

// Pass 2: stable scatter.  block_off = exclusive scan of block_cnt (digit-major); inside a workgroup
// the rank of an element among the elements with its digit comes from wavefront ballots.
// vals_in == nullptr stands for the identity (first pass).
__global__ __launch_bounds__(kThreads) void radix_scatter_kernel(
    const int32_t *__restrict__ keys_in, const int32_t *__restrict__ vals_in, int64_t n, int shift,
    const int32_t *__restrict__ block_off, int64_t n_blocks, int32_t *__restrict__ keys_out,
    int32_t *__restrict__ vals_out)
{
    __shared__ int s_wave_cnt[kThreads / kWave][kDigits];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int32_t key = i < n ? keys_in[i] : 0;
    const int digit = i < n ? (key >> shift) & (kDigits - 1) : -1;
    int rank_in_wave = 0;
#pragma unroll
    for (int d = 0; d < kDigits; ++d) {
        const unsigned long long mask = __ballot(digit == d);
        if (lane == 0) s_wave_cnt[wave][d] = __popcll(mask);
        if (digit == d) rank_in_wave = __popcll(mask & ((1ull << lane) - 1ull));
    }
    __syncthreads();
    if (digit < 0) return;
    int32_t p = block_off[(int64_t)digit * n_blocks + blockIdx.x] + rank_in_wave;
    for (int w2 = 0; w2 < wave; ++w2) p += s_wave_cnt[w2][digit];
    keys_out[p] = key;
    vals_out[p] = vals_in ? vals_in[i] : (int32_t)i;
}

// After the sort: keys are the columns in ascending order, perm the input positions.  Writes the row
// pointers of the transpose (first position of every column, empty columns included) and the
// transposed column indices (= input row of the entry, found by bisection in the input row_ptr).
__global__ __launch_bounds__(kThreads) void transpose_finish_kernel(
    int32_t n_rows, int32_t n_cols, int64_t nnz, const int32_t *__restrict__ row_ptr,
    const int32_t *__restrict__ sorted_cols, const int32_t *__restrict__ perm, int32_t *__restrict__ out_row_ptr,
    int32_t *__restrict__ out_col_idx)
{
    const int64_t k = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (k >= nnz) return;
    const int32_t c = sorted_cols[k];
    const int32_t prev = k > 0 ? sorted_cols[k - 1] : -1;
    for (int32_t cc = prev + 1; cc <= c; ++cc) out_row_ptr[cc] = (int32_t)k;
    if (k == nnz - 1)
        for (int32_t cc = c + 1; cc <= n_cols; ++cc) out_row_ptr[cc] = (int32_t)nnz;
    const int32_t e = perm[k];
    int32_t lo = 0, hi = n_rows;          // last row r with row_ptr[r] <= e
    while (hi - lo > 1) {
        const int32_t mid = lo + (hi - lo) / 2;
        if (row_ptr[mid] <= e) lo = mid; else hi = mid;
    }
    out_col_idx[k] = lo;
}

__global__ void fill_i32_kernel(int32_t *p, int64_t n, int32_t v)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

__global__ void edge_gather_kernel(int64_t n, const int32_t *__restrict__ perm, const float *__restrict__ in,
                                   float *__restrict__ out)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = in[perm[i]];
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// dv[e] = p[e] * (dp[e] - sum over the row of p * dp).  Rows of at most kSegLen entries: kBwdGroup lanes
// per row with the row's entries in registers (four rows per wavefront); longer rows: one workgroup per
// row (the gather plan's list of split rows).
constexpr int kBwdGroup = 16;

__global__ __launch_bounds__(kThreads) void softmax_bwd_kernel(int32_t n_rows, const int32_t *__restrict__ row_ptr,
                                                               const float *p, const float *dp, float *dv)
{
    constexpr int G = kBwdGroup, SLOTS = kSegLen / G;
    const int gl = threadIdx.x % G;
    const int64_t row = ((int64_t)blockIdx.x * kThreads + threadIdx.x) / G;
    int32_t b = 0, e = 0;
    if (row < n_rows) {
        b = row_ptr[row];
        e = row_ptr[row + 1];
        if (e - b > kSegLen) e = b;             // a long row: not here
    }
    float pv[SLOTS], gv[SLOTS];
    float dot = 0.f;
#pragma unroll
    for (int i = 0; i < SLOTS; ++i) {
        const int32_t k = b + gl + G * i;
        pv[i] = k < e ? p[k] : 0.f;
        gv[i] = k < e ? dp[k] : 0.f;
        dot = fmaf(pv[i], gv[i], dot);
    }
#pragma unroll
    for (int off = 1; off < G; off <<= 1) dot += __shfl_xor(dot, off, kWave);
#pragma unroll
    for (int i = 0; i < SLOTS; ++i) {
        const int32_t k = b + gl + G * i;
        if (k < e) dv[k] = pv[i] * (gv[i] - dot);
    }
}

// Long rows (the gather plan's list of split rows), in two kernels over that list.  Up to kMidRow entries:
// one 256-thread workgroup per row, p and dp of the row in registers (eight values each per thread).
// Beyond: 1024-thread workgroups walk the list and take two passes over such a row, four values per
// thread in flight.
constexpr int kMidRow = 8 * kThreads;
constexpr int kLongThreads = 1024;
constexpr int kLongGridMax = 1024;

__global__ __launch_bounds__(kThreads) void softmax_bwd_mid_kernel(const int32_t *__restrict__ long_row,
                                                                   const int32_t *__restrict__ row_ptr, const float *p,
                                                                   const float *dp, float *dv)
{
    __shared__ float s_red[kThreads / kWave];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const int32_t row = long_row[blockIdx.x];
    const int32_t b = row_ptr[row], e = row_ptr[row + 1];
    if (e - b > kMidRow) return;
    float pv[8], gv[8];
    float dot = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int32_t k = b + threadIdx.x + kThreads * i;
        pv[i] = k < e ? p[k] : 0.f;
        gv[i] = k < e ? dp[k] : 0.f;
        dot = fmaf(pv[i], gv[i], dot);
    }
    dot = wave_sum(dot);
    if (lane == 0) s_red[wave] = dot;
    __syncthreads();
    dot = 0.f;
#pragma unroll
    for (int i = 0; i < kThreads / kWave; ++i) dot += s_red[i];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int32_t k = b + threadIdx.x + kThreads * i;
        if (k < e) dv[k] = pv[i] * (gv[i] - dot);
    }
}

__global__ __launch_bounds__(kLongThreads) void softmax_bwd_long_kernel(int32_t n_long,
                                                                        const int32_t *__restrict__ long_row,
                                                                        const int32_t *__restrict__ row_ptr,
                                                                        const float *p, const float *dp, float *dv)
{
    __shared__ float s_red[kLongThreads / kWave];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    for (int32_t li = blockIdx.x; li < n_long; li += gridDim.x) {     // the same trip count for every thread
        const int32_t row = long_row[li];
        const int32_t b = row_ptr[row], e = row_ptr[row + 1];
        if (e - b <= kMidRow) continue;                               // the whole workgroup skips together
        float dot = 0.f;
        for (int32_t k0 = b + threadIdx.x; k0 < e; k0 += 4 * kLongThreads) {
            float a[4], c[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const bool ok = k0 + u * kLongThreads < e;
                a[u] = ok ? p[k0 + u * kLongThreads] : 0.f;
                c[u] = ok ? dp[k0 + u * kLongThreads] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) dot = fmaf(a[u], c[u], dot);
        }
        dot = wave_sum(dot);
        if (lane == 0) s_red[wave] = dot;
        __syncthreads();
        dot = 0.f;
#pragma unroll
        for (int i = 0; i < kLongThreads / kWave; ++i) dot += s_red[i];
        for (int32_t k0 = b + threadIdx.x; k0 < e; k0 += 4 * kLongThreads) {
            float a[4], c[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const bool ok = k0 + u * kLongThreads < e;
                a[u] = ok ? p[k0 + u * kLongThreads] : 0.f;
                c[u] = ok ? dp[k0 + u * kLongThreads] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (k0 + u * kLongThreads < e) dv[k0 + u * kLongThreads] = a[u] * (c[u] - dot);
        }
        __syncthreads();                                              // s_red is reused by the next row
    }
}

}  // namespace

int row_softmax_backward_impl(const tcg_meta *m, const float *d_p, const float *d_dp, float *d_dv, hipStream_t s)
{
    if (m->n_rows == 0 || m->nnz == 0) return TCG_OK;
    hipLaunchKernelGGL(softmax_bwd_kernel, dim3((unsigned)ceil_div(m->n_rows, kThreads / kBwdGroup)), dim3(kThreads), 0, s,
                       m->n_rows, m->d_row_ptr, d_p, d_dp, d_dv);
    TCG_TRY(launch_status("softmax_bwd_kernel"));
    if (m->n_long > 0) {
        hipLaunchKernelGGL(softmax_bwd_mid_kernel, dim3((unsigned)m->n_long), dim3(kThreads), 0, s, m->d_long_row,
                           m->d_row_ptr, d_p, d_dp, d_dv);
        TCG_TRY(launch_status("softmax_bwd_mid_kernel"));
        hipLaunchKernelGGL(softmax_bwd_long_kernel, dim3((unsigned)std::min<int64_t>(m->n_long, kLongGridMax)),
                           dim3(kLongThreads), 0, s, (int32_t)m->n_long, m->d_long_row, m->d_row_ptr, d_p, d_dp, d_dv);
        TCG_TRY(launch_status("softmax_bwd_long_kernel"));
    }
    return TCG_OK;
}

int edge_gather_impl(int64_t n, const int32_t *d_perm, const float *d_in, float *d_out, hipStream_t s)
{
    if (n == 0) return TCG_OK;
    hipLaunchKernelGGL(edge_gather_kernel, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, s, n, d_perm, d_in, d_out);
    return launch_status("edge_gather_kernel");
}

size_t radix_sort_scratch_bytes(int64_t n)
{
    const int64_t n_blocks = ceil_div(n, kThreads);
    const int64_t cnt_elems = (int64_t)kDigits * n_blocks + 1;
    if (cnt_elems >= (int64_t)INT32_MAX) return 0;
    const size_t arr = ((size_t)n * 4 + 255) & ~(size_t)255;
    const size_t cnt_bytes = ((size_t)cnt_elems * 4 + 255) & ~(size_t)255;
    return 2 * arr + cnt_bytes + (size_t)scan_workspace_elems(cnt_elems) * 4;
}

int radix_sort_pairs(const int32_t *d_keys_in, const int32_t *d_vals_in, int64_t n, int bits, int32_t *d_keys_out,
                     int32_t *d_vals_out, void *d_scratch, hipStream_t s)
{
    if (n == 0) return TCG_OK;
    const int passes = (bits + 3) / 4;
    const int64_t n_blocks = ceil_div(n, kThreads);
    const int64_t cnt_elems = (int64_t)kDigits * n_blocks + 1;
    const size_t arr = ((size_t)n * 4 + 255) & ~(size_t)255;
    const size_t cnt_bytes = ((size_t)cnt_elems * 4 + 255) & ~(size_t)255;
    char *base = static_cast<char *>(d_scratch);
    int32_t *keys_b = reinterpret_cast<int32_t *>(base);
    int32_t *vals_b = reinterpret_cast<int32_t *>(base + arr);
    int32_t *block_cnt = reinterpret_cast<int32_t *>(base + 2 * arr);
    int32_t *scan_work = reinterpret_cast<int32_t *>(base + 2 * arr + cnt_bytes);

    const int32_t *kin = d_keys_in;
    const int32_t *vin = d_vals_in;
    for (int pass = 0; pass < passes; ++pass) {
        // Choose the outputs so that the last pass lands in the caller's arrays.
        const bool to_out = ((passes - 1 - pass) % 2) == 0;
        int32_t *kout = to_out ? d_keys_out : keys_b;
        int32_t *vout = to_out ? d_vals_out : vals_b;
        hipLaunchKernelGGL(radix_count_kernel, dim3((unsigned)n_blocks), dim3(kThreads), 0, s, kin, n, 4 * pass,
                           block_cnt, n_blocks);
        TCG_TRY(exclusive_scan_i32(block_cnt, block_cnt, cnt_elems - 1, scan_work, s));
        hipLaunchKernelGGL(radix_scatter_kernel, dim3((unsigned)n_blocks), dim3(kThreads), 0, s, kin, vin, n, 4 * pass,
                           block_cnt, n_blocks, kout, vout);
        TCG_TRY(launch_status("radix kernels"));
        kin = kout;
        vin = vout;
    }
    return TCG_OK;
}

int csr_transpose_impl(int32_t n_rows, int32_t n_cols, int64_t nnz, const int32_t *d_row_ptr,
                       const int32_t *d_col_idx, int32_t *d_out_row_ptr, int32_t *d_out_col_idx, int32_t *d_perm,
                       hipStream_t s)
{
    if (nnz == 0) {
        hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)ceil_div((int64_t)n_cols + 1, 256)), dim3(256), 0, s,
                           d_out_row_ptr, (int64_t)n_cols + 1, 0);
        return launch_status("fill_i32_kernel");
    }
    int bits = 1;
    while (bits < 31 && (1ll << bits) < (int64_t)n_cols) ++bits;
    const int64_t n_blocks = ceil_div(nnz, kThreads);
    if (radix_sort_scratch_bytes(nnz) == 0) return TCG_ERANGE;

    // Scratch: sorted keys plus the sort's own workspace; the caller's perm array receives the values.
    const size_t arr = ((size_t)nnz * 4 + 255) & ~(size_t)255;
    PoolBuf buf;
    buf.s = s;
    TCG_TRY(pool_alloc(&buf.p, arr + radix_sort_scratch_bytes(nnz)));
    char *base = static_cast<char *>(buf.p);
    int32_t *keys_sorted = reinterpret_cast<int32_t *>(base);
    TCG_TRY(radix_sort_pairs(d_col_idx, nullptr, nnz, bits, keys_sorted, d_perm, base + arr, s));
    const int32_t *kin = keys_sorted;
    hipLaunchKernelGGL(transpose_finish_kernel, dim3((unsigned)n_blocks), dim3(kThreads), 0, s, n_rows, n_cols, nnz,
                       d_row_ptr, kin, d_perm, d_out_row_ptr, d_out_col_idx);
    TCG_TRY(launch_status("transpose_finish_kernel"));
    TCG_HIP(hipStreamSynchronize(s));     // the scratch goes back to the pool on return
    return TCG_OK;
}

}  // namespace tcg
