// Building blocks of the backward pass.  The paper trains GNNs with these sparse operations
// (section 4) without spelling the gradients out; by the chain rule on Equations 1 and 2:
//   Y = (w (.) A) X :   dX = (w (.) A)^T dY            tcg_spmm on the transposed structure, w permuted
//                       dw[e] = < dY[row(e)], X[col(e)] >   tcg_sddmm_pq(P = dY, Q = X)
//   out[e] = <x_i,x_j>: dX = (g (.) A) X + (g (.) A)^T X    two tcg_spmm calls (g = d out)
//   p = row_softmax(v): dv[e] = p[e] (dp[e] - sum_row p dp)  tcg_row_softmax_backward
// This file holds the CSR transpose (a stable radix sort of the entries by column, radix.hip, so the
// result is unique and deterministic), the edge-value permutation and the softmax gradient.
#include "common.h"

namespace tcg {

namespace {

constexpr int kThreads = 256;
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

// dv[e] = p[e] * (dp[e] - sum over the row of p * dp).  Rows of at most kSegLen entries are taken from the
// tail of the gather plan's segment list (single-segment rows; rows without entries have an empty segment
// there and are skipped; on graphs without neighbour sharing the list is ordered by row length): a workgroup looks at the lengths of its 64
// rows and runs the variant that fits the longest -- G lanes per row, S entries of p and of dp per lane in
// registers, (G, S) = (4, 2) up to 8 entries, (8, 2) up to 16, (16, 2) up to 32, (16, 8) up to 128.
constexpr int kTailRows = 64;          // rows per workgroup

template <int G, int S>
__device__ __forceinline__ void softmax_bwd_rows(const int32_t *s_b, const int32_t *s_e, const float *p, const float *dp,
                                                 float *dv)
{
    constexpr int ROWS = kThreads / G;               // rows per pass of the workgroup
    const int gl = threadIdx.x % G;
#pragma unroll
    for (int pass = 0; pass < kTailRows / ROWS; ++pass) {
        const int r = pass * ROWS + threadIdx.x / G;
        const int32_t b = s_b[r], e = s_e[r];
        float pv[S], gv[S];
        float dot = 0.f;
#pragma unroll
        for (int i = 0; i < S; ++i) {
            const int32_t k = b + gl + G * i;
            pv[i] = k < e ? p[k] : 0.f;
            gv[i] = k < e ? dp[k] : 0.f;
            dot = fmaf(pv[i], gv[i], dot);
        }
#pragma unroll
        for (int off = 1; off < G; off <<= 1) dot += __shfl_xor(dot, off, kWave);
#pragma unroll
        for (int i = 0; i < S; ++i) {
            const int32_t k = b + gl + G * i;
            if (k < e) dv[k] = pv[i] * (gv[i] - dot);
        }
    }
}

// A row of the gather plan's list of split rows (more than kSegLen entries), by one 256-thread workgroup: up to
// 8 * 256 entries p and dp of the row sit in registers; a longer row takes two passes, eight values of each
// operand per thread in flight.  (More registers per thread would halve the resident wavefronts of the whole
// kernel, which the short rows need more than the long ones need the saved second read.)
__device__ __forceinline__ void softmax_bwd_long_row(int32_t b, int32_t e, const float *p, const float *dp, float *dv,
                                                     float *s_red)
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    if (e - b <= 8 * kThreads) {
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
        return;
    }
    float dot = 0.f;
    for (int32_t k0 = b + threadIdx.x; k0 < e; k0 += 8 * kThreads) {
        float a[8], c[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const bool ok = k0 + u * kThreads < e;
            a[u] = ok ? p[k0 + u * kThreads] : 0.f;
            c[u] = ok ? dp[k0 + u * kThreads] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) dot = fmaf(a[u], c[u], dot);
    }
    dot = wave_sum(dot);
    if (lane == 0) s_red[wave] = dot;
    __syncthreads();
    dot = 0.f;
#pragma unroll
    for (int i = 0; i < kThreads / kWave; ++i) dot += s_red[i];
    for (int32_t k0 = b + threadIdx.x; k0 < e; k0 += 8 * kThreads) {
        float a[8], c[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const bool ok = k0 + u * kThreads < e;
            a[u] = ok ? p[k0 + u * kThreads] : 0.f;
            c[u] = ok ? dp[k0 + u * kThreads] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (k0 + u * kThreads < e) dv[k0 + u * kThreads] = a[u] * (c[u] - dot);
    }
}

// One launch for all rows: workgroups 0 .. n_long - 1 take one split row each (dispatched first, so the long
// rows start at once and the short ones fill in around them), the workgroups behind them 64 single-segment rows
// each.
__global__ __launch_bounds__(kThreads) void softmax_bwd_kernel(int32_t n_long, const int32_t *__restrict__ long_row,
                                                               int32_t tail_start, int32_t tail_count,
                                                               const int32_t *__restrict__ seg_row,
                                                               const int32_t *__restrict__ seg_dst,
                                                               const int32_t *__restrict__ row_ptr, const float *p,
                                                               const float *dp, float *dv)
{
    __shared__ int32_t s_b[kTailRows], s_e[kTailRows];
    __shared__ float s_red[kThreads / kWave];
    __shared__ int s_max;
    if ((int32_t)blockIdx.x < n_long) {
        const int32_t row = long_row[blockIdx.x];
        softmax_bwd_long_row(row_ptr[row], row_ptr[row + 1], p, dp, dv, s_red);
        return;
    }
    if (threadIdx.x == 0) s_max = 0;
    __syncthreads();
    if (threadIdx.x < kTailRows) {
        const int64_t i = (int64_t)(blockIdx.x - n_long) * kTailRows + threadIdx.x;
        int32_t b = 0, e = 0;
        if (i < tail_count && seg_dst[tail_start + i] < 0) {          // a piece of a split row: not here
            const int32_t row = seg_row[tail_start + i];
            b = row_ptr[row];
            e = row_ptr[row + 1];
        }
        s_b[threadIdx.x] = b;
        s_e[threadIdx.x] = e;
        if (e > b) atomicMax(&s_max, e - b);
    }
    __syncthreads();
    const int longest = s_max;
    if (longest == 0) return;
    if (longest <= 8) softmax_bwd_rows<4, 2>(s_b, s_e, p, dp, dv);
    else if (longest <= 16) softmax_bwd_rows<8, 2>(s_b, s_e, p, dp, dv);
    else if (longest <= 32) softmax_bwd_rows<16, 2>(s_b, s_e, p, dp, dv);
    else softmax_bwd_rows<16, kSegLen / 16>(s_b, s_e, p, dp, dv);
}

}  // namespace

int row_softmax_backward_impl(const tcg_meta *m, const float *d_p, const float *d_dp, float *d_dv, hipStream_t s)
{
    if (m->n_rows == 0 || m->nnz == 0) return TCG_OK;
    const int32_t tail_start = m->h_lane_tab[4], tail_count = m->h_lane_tab[5];
    const int64_t grid = m->n_long + ceil_div(tail_count, kTailRows);
    if (grid > 0) {
        hipLaunchKernelGGL(softmax_bwd_kernel, dim3((unsigned)grid), dim3(kThreads), 0, s, (int32_t)m->n_long,
                           m->d_long_row, tail_start, tail_count, m->d_seg_row, m->d_seg_dst, m->d_row_ptr, d_p, d_dp,
                           d_dv);
        TCG_TRY(launch_status("softmax_bwd_kernel"));
    }
    return TCG_OK;
}

int edge_gather_impl(int64_t n, const int32_t *d_perm, const float *d_in, float *d_out, hipStream_t s)
{
    if (n == 0) return TCG_OK;
    hipLaunchKernelGGL(edge_gather_kernel, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, s, n, d_perm, d_in, d_out);
    return launch_status("edge_gather_kernel");
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
    TCG_TRY(radix_sort_pairs(d_col_idx, nullptr, nnz, nullptr, bits, keys_sorted, d_perm, base + arr, s));
    const int32_t *kin = keys_sorted;
    hipLaunchKernelGGL(transpose_finish_kernel, dim3((unsigned)n_blocks), dim3(kThreads), 0, s, n_rows, n_cols, nnz,
                       d_row_ptr, kin, d_perm, d_out_row_ptr, d_out_col_idx);
    TCG_TRY(launch_status("transpose_finish_kernel"));
    TCG_HIP(hipStreamSynchronize(s));     // the scratch goes back to the pool on return
    return TCG_OK;
}

}  // namespace tcg
