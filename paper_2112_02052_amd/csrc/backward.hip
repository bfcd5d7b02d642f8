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
// row_of[e] = the row that holds entry e of the input, for all entries.  A workgroup takes kRowsTile consecutive
// entries: two of its wavefronts find the rows of the first and the last of them (the last row r with
// row_ptr[r] <= e) by a 64-way search -- every lane probes one position, a ballot picks the interval, four
// rounds for a million rows -- and the wavefronts then walk that row range 64 rows at a time (pointers in one
// coalesced load), writing each row's number over its entries inside the tile: a lane on its own for rows of up
// to 8 entries, the wavefront together, 64 entries per step, for longer ones.  Dealing out rows instead of entries leaves the rows of the hubs, which
// sit side by side in skewed graphs, to one wavefront (145 us for 19 M entries).
constexpr int kRowsTile = 4096;

__global__ __launch_bounds__(kThreads) void entry_rows_kernel(int32_t n_rows, int64_t nnz,
                                                              const int32_t *__restrict__ row_ptr,
                                                              int32_t *__restrict__ row_of)
{
    __shared__ int32_t s_end[2];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int64_t lo = (int64_t)blockIdx.x * kRowsTile;
    const int64_t hi = min(lo + kRowsTile, nnz);
    if (lo >= hi) return;
    if (wave < 2) {
        const int64_t target = wave == 0 ? lo : hi - 1;
        int64_t a = 0, span = n_rows;                    // the row is in [a, a + span), row_ptr[a] <= target
        while (span > 1) {
            const int64_t step = (span + kWave - 1) / kWave;
            const int64_t p = a + lane * step;
            const bool ok = lane == 0 || (p < a + span && row_ptr[p] <= target);
            const int last = __popcll(__ballot(ok)) - 1;  // the pointers ascend, so the lanes that hold are a prefix
            const int64_t end = a + span;
            a += last * step;
            span = min(step, end - a);
        }
        if (lane == 0) s_end[wave] = (int32_t)a;
    }
    __syncthreads();
    const int32_t r_first = s_end[0], r_last = s_end[1];
    for (int64_t r0 = (int64_t)r_first + wave * kWave; r0 <= r_last; r0 += kThreads) {
        const int64_t r = r0 + lane;
        int64_t b = 0, e = 0;
        if (r <= r_last) {
            b = max((int64_t)row_ptr[r], lo);
            e = min((int64_t)row_ptr[r + 1], hi);
        }
        // rows of a few entries: every lane writes its own (neighbouring lanes, neighbouring addresses); where the
        // rows are that short a tile spans thousands of them, and a wavefront step per row took 40 us per tile
        const bool few = e - b <= 8;
        if (few)
            for (int64_t i = b; i < e; ++i) row_of[i] = (int32_t)r;
        unsigned long long todo = __ballot(!few);
        while (todo) {
            const int src = __ffsll(todo) - 1;
            todo &= todo - 1;
            const int64_t bb = __shfl(b, src, kWave), ee = __shfl(e, src, kWave);
            for (int64_t i = bb + lane; i < ee; i += kWave) row_of[i] = (int32_t)(r0 + src);
        }
    }
}

// After the sort: keys are the columns in ascending order, perm the input positions.  Writes the row
// pointers of the transpose (first position of every column, empty columns included) and the
// transposed column indices (= input row of the entry, one gather from row_of; a bisection in row_ptr per
// sorted entry, whose neighbours belong to unrelated rows, was twenty scattered loads and 0.73 of the
// 1.15 ms of a transpose of 19 M entries).
__global__ __launch_bounds__(kThreads) void transpose_finish_kernel(
    int32_t n_cols, int64_t nnz, const int32_t *__restrict__ row_of, const int32_t *__restrict__ sorted_cols,
    const int32_t *__restrict__ perm, int32_t *__restrict__ out_row_ptr, int32_t *__restrict__ out_col_idx)
{
    const int64_t k = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (k >= nnz) return;
    const int32_t row = row_of[perm[k]];
    const int32_t c = sorted_cols[k];
    const int32_t prev = k > 0 ? sorted_cols[k - 1] : -1;
    for (int32_t cc = prev + 1; cc <= c; ++cc) out_row_ptr[cc] = (int32_t)k;
    if (k == nnz - 1)
        for (int32_t cc = c + 1; cc <= n_cols; ++cc) out_row_ptr[cc] = (int32_t)nnz;
    out_col_idx[k] = row;
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

// dv[e] = p[e] * (dp[e] - sum over the row of p * dp), laid out like the row softmax (sddmm.hip): work is dealt
// out per wavefront without LDS or barriers -- 16 single-segment rows per wavefront from the tail of the gather
// plan's segment list (first edge in seg_ebeg, length in seg_dst), G lanes per row with S entries of p and of dp
// per lane in registers, (G, S) = (4, 2) up to 8 entries, (8, 2) up to 16, (16, 2) up to 32, (16, 8) up to 128;
// one wavefront per split row of up to kGiantRow entries; one workgroup per longer row, two passes with the
// next batch requested before the current one is worked on.
constexpr int kTailRowsPerWave = 16;             // lanes 0 .. 15 look the rows up (more rows per wavefront cost
                                                 // registers, and with them resident wavefronts: measured slower)

template <int G, int S>
__device__ __forceinline__ void softmax_bwd_tail_rows(int32_t b_l, int32_t len_l, const float *p, const float *dp,
                                                      float *dv)
{
    constexpr int RPP = kWave / G;                   // rows per pass of the wavefront
    constexpr int PASSES = kTailRowsPerWave / RPP;
    // The values of several passes are requested before the first result is stored (dv may be dp, so the compiler
    // keeps loads behind earlier stores): all passes, or two at a time where that would take too many registers.
    constexpr int BATCH = PASSES * S > 16 ? 16 / S : PASSES;
    const int lane = threadIdx.x & (kWave - 1);
    const int gl = lane % G;
#pragma unroll
    for (int p0 = 0; p0 < PASSES; p0 += BATCH) {
        float pv[BATCH][S], gv[BATCH][S];
        int32_t b[BATCH], e[BATCH];
#pragma unroll
        for (int q = 0; q < BATCH; ++q) {
            const int r = (p0 + q) * RPP + lane / G;
            b[q] = __shfl(b_l, r, kWave);
            e[q] = b[q] + __shfl(len_l, r, kWave);
#pragma unroll
            for (int i = 0; i < S; ++i) {
                const int32_t k = b[q] + gl + G * i;
                pv[q][i] = k < e[q] ? p[k] : 0.f;
                gv[q][i] = k < e[q] ? dp[k] : 0.f;
            }
        }
#pragma unroll
        for (int q = 0; q < BATCH; ++q) {
            float dot = 0.f;
#pragma unroll
            for (int i = 0; i < S; ++i) dot = fmaf(pv[q][i], gv[q][i], dot);
#pragma unroll
            for (int off = 1; off < G; off <<= 1) dot += __shfl_xor(dot, off, kWave);
#pragma unroll
            for (int i = 0; i < S; ++i) {
                const int32_t k = b[q] + gl + G * i;
                if (k < e[q]) dv[k] = pv[q][i] * (gv[q][i] - dot);
            }
        }
    }
}

template <int R>
__device__ __forceinline__ void softmax_bwd_row_wave(int32_t b, int32_t e, const float *p, const float *dp, float *dv)
{
    const int lane = threadIdx.x & (kWave - 1);
    float pv[R], gv[R];
    float dot = 0.f;
#pragma unroll
    for (int i = 0; i < R; ++i) {
        const int32_t k = b + lane + kWave * i;
        pv[i] = k < e ? p[k] : 0.f;
        gv[i] = k < e ? dp[k] : 0.f;
        dot = fmaf(pv[i], gv[i], dot);
    }
    dot = wave_sum(dot);
#pragma unroll
    for (int i = 0; i < R; ++i) {
        const int32_t k = b + lane + kWave * i;
        if (k < e) dv[k] = pv[i] * (gv[i] - dot);
    }
}

// The few longer rows: pieces of kGiantChunk entries from the plan's list, one workgroup per piece with both
// operands of the piece in registers, in two launches -- the first leaves every piece's sum of p * dp, in the
// second the workgroup of a piece adds the sums of its row's pieces in a fixed order and writes its results.
constexpr int kPieceVals = kGiantChunk / kThreads;
constexpr int kWavesPerBlock = kThreads / kWave;

struct RowPiece {
    int32_t b, e;            // the piece's entries
    int32_t first, count;    // the pieces of its row in the list
};

__device__ __forceinline__ RowPiece giant_piece(int32_t k, const int32_t *gchunk_li, const int32_t *gchunk_c,
                                             const int32_t *long_ebeg, const int32_t *long_len)
{
    const int32_t li = gchunk_li[k], c = gchunk_c[k];
    const int32_t rb = long_ebeg[li], len = long_len[li];
    RowPiece pc;
    pc.b = rb + c * kGiantChunk;
    pc.e = min(rb + len, pc.b + kGiantChunk);
    pc.first = k - c;
    pc.count = (len + kGiantChunk - 1) / kGiantChunk;
    return pc;
}

// Workgroup-wide sum in a fixed order; every thread of the workgroup calls it.
__device__ __forceinline__ float block_sum(float v, float *s_red)
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    v = wave_sum(v);
    if (lane == 0) s_red[wave] = v;
    __syncthreads();
    float r = s_red[0];
#pragma unroll
    for (int i = 1; i < kWavesPerBlock; ++i) r += s_red[i];
    return r;
}

__global__ __launch_bounds__(kThreads) void softmax_bwd_piece_sums_kernel(const int32_t *__restrict__ gchunk_li,
                                                                          const int32_t *__restrict__ gchunk_c,
                                                                          const int32_t *__restrict__ long_ebeg,
                                                                          const int32_t *__restrict__ long_len,
                                                                          const float *__restrict__ p,
                                                                          const float *__restrict__ dp,
                                                                          float *__restrict__ sums)
{
    __shared__ float s_red[kWavesPerBlock];
    const RowPiece pc = giant_piece((int32_t)blockIdx.x, gchunk_li, gchunk_c, long_ebeg, long_len);
    float a[kPieceVals], c[kPieceVals];
#pragma unroll
    for (int u = 0; u < kPieceVals; ++u) {
        const int32_t k = pc.b + threadIdx.x + u * kThreads;
        a[u] = k < pc.e ? p[k] : 0.f;
        c[u] = k < pc.e ? dp[k] : 0.f;
    }
    float dot = 0.f;
#pragma unroll
    for (int u = 0; u < kPieceVals; ++u) dot = fmaf(a[u], c[u], dot);
    dot = block_sum(dot, s_red);
    if (threadIdx.x == 0) sums[blockIdx.x] = dot;
}

__device__ __forceinline__ void softmax_bwd_piece(const RowPiece &pc, const float *sums, const float *p, const float *dp,
                                                  float *dv, float *s_red)
{
    float a[kPieceVals], c[kPieceVals];
#pragma unroll
    for (int u = 0; u < kPieceVals; ++u) {
        const int32_t k = pc.b + threadIdx.x + u * kThreads;
        a[u] = k < pc.e ? p[k] : 0.f;
        c[u] = k < pc.e ? dp[k] : 0.f;
    }
    float part = 0.f;
    for (int32_t i = threadIdx.x; i < pc.count; i += kThreads) part += sums[pc.first + i];
    const float dot = block_sum(part, s_red);
#pragma unroll
    for (int u = 0; u < kPieceVals; ++u) {
        const int32_t k = pc.b + threadIdx.x + u * kThreads;
        if (k < pc.e) dv[k] = a[u] * (c[u] - dot);
    }
}

// A split row of 1025 .. kGiantRow entries by one wavefront, 16 values of each operand per lane at a time: the sum
// over both halves first, then each half again for the results (both operands of the whole row in registers
// would cost the kernel half of its resident wavefronts).
__device__ __forceinline__ void softmax_bwd_row_wave_halves(int32_t b, int32_t e, const float *p, const float *dp,
                                                            float *dv)
{
    constexpr int R = 16;
    const int lane = threadIdx.x & (kWave - 1);
    float dot = 0.f;
#pragma unroll 1
    for (int h = 0; h < 2; ++h) {
        float a[R], c[R];
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const int32_t k = b + h * kWave * R + lane + kWave * i;
            a[i] = k < e ? p[k] : 0.f;
            c[i] = k < e ? dp[k] : 0.f;
        }
#pragma unroll
        for (int i = 0; i < R; ++i) dot = fmaf(a[i], c[i], dot);
    }
    dot = wave_sum(dot);
#pragma unroll 1
    for (int h = 0; h < 2; ++h) {
        float a[R], c[R];
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const int32_t k = b + h * kWave * R + lane + kWave * i;
            a[i] = k < e ? p[k] : 0.f;
            c[i] = k < e ? dp[k] : 0.f;
        }
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const int32_t k = b + h * kWave * R + lane + kWave * i;
            if (k < e) dv[k] = a[i] * (c[i] - dot);
        }
    }
}

__global__ __launch_bounds__(kThreads) void softmax_bwd_kernel(
    int32_t n_gchunks, const int32_t *__restrict__ gchunk_li, const int32_t *__restrict__ gchunk_c,
    const float *__restrict__ sums, int32_t n_long, const int32_t *__restrict__ long_ebeg,
    const int32_t *__restrict__ long_len, int32_t tail_start, int32_t tail_count,
    const int32_t *__restrict__ seg_ebeg, const int32_t *__restrict__ seg_dst, const float *p, const float *dp,
    float *dv)
{
    __shared__ float s_red[kWavesPerBlock];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    int32_t blk = blockIdx.x;
    if (blk < n_gchunks) {
        softmax_bwd_piece(giant_piece(blk, gchunk_li, gchunk_c, long_ebeg, long_len), sums, p, dp, dv, s_red);
        return;
    }
    blk -= n_gchunks;
    const int32_t n_long_blocks = (n_long + kWavesPerBlock - 1) / kWavesPerBlock;
    if (blk < n_long_blocks) {
        const int32_t li = blk * kWavesPerBlock + wave;
        if (li >= n_long) return;
        const int32_t b = long_ebeg[li], len = long_len[li];
        if (len <= 8 * kWave) softmax_bwd_row_wave<8>(b, b + len, p, dp, dv);
        else if (len <= 16 * kWave) softmax_bwd_row_wave<16>(b, b + len, p, dp, dv);
        else if (len <= kGiantRow) softmax_bwd_row_wave_halves(b, b + len, p, dp, dv);
        return;                                     // longer: handled in pieces
    }
    blk -= n_long_blocks;
    const int64_t i = ((int64_t)blk * kWavesPerBlock + wave) * kTailRowsPerWave + lane;
    int32_t b = 0, len = 0;
    if (lane < kTailRowsPerWave && i < tail_count) {
        b = seg_ebeg[tail_start + i];
        len = -1 - seg_dst[tail_start + i];                           // single-segment rows carry their length
    }
    int longest = len;
#pragma unroll
    for (int off = 1; off < kTailRowsPerWave; off <<= 1) longest = max(longest, __shfl_xor(longest, off, kWave));
    longest = __shfl(longest, 0, kWave);
    if (longest == 0) return;
    if (longest <= 8) softmax_bwd_tail_rows<4, 2>(b, len, p, dp, dv);
    else if (longest <= 16) softmax_bwd_tail_rows<8, 2>(b, len, p, dp, dv);
    else if (longest <= 32) softmax_bwd_tail_rows<16, 2>(b, len, p, dp, dv);
    else softmax_bwd_tail_rows<16, kSegLen / 16>(b, len, p, dp, dv);
}

}  // namespace

int row_softmax_backward_impl(const tcg_meta *m, const float *d_p, const float *d_dp, float *d_dv, hipStream_t s)
{
    if (m->n_rows == 0 || m->nnz == 0) return TCG_OK;
    const int32_t tail_start = m->h_lane_tab[4], tail_count = m->h_lane_tab[5];
    const int64_t grid = m->n_gchunks + ceil_div(m->n_long, kWavesPerBlock) +
                         ceil_div(tail_count, kWavesPerBlock * kTailRowsPerWave);
    float *sums = m->d_partial_ml;                       // one sum per piece; pieces <= slots
    if (m->n_gchunks > 0)
        hipLaunchKernelGGL(softmax_bwd_piece_sums_kernel, dim3((unsigned)m->n_gchunks), dim3(kThreads), 0, s,
                           m->d_gchunk_li, m->d_gchunk_c, m->d_long_ebeg, m->d_long_len, d_p, d_dp, sums);
    if (grid > 0) {
        hipLaunchKernelGGL(softmax_bwd_kernel, dim3((unsigned)grid), dim3(kThreads), 0, s, (int32_t)m->n_gchunks,
                           m->d_gchunk_li, m->d_gchunk_c, sums, (int32_t)m->n_long, m->d_long_ebeg, m->d_long_len,
                           tail_start, tail_count, m->d_seg_ebeg, m->d_seg_dst, d_p, d_dp, d_dv);
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
    if (radix_sort_scratch_bytes(nnz) == 0) return TCG_ERANGE;

    // Scratch: sorted keys, the row of every entry, and the sort's own workspace; the caller's perm array
    // receives the values.
    const size_t arr = ((size_t)nnz * 4 + 255) & ~(size_t)255;
    PoolBuf buf;
    buf.s = s;
    TCG_TRY(pool_alloc(&buf.p, 2 * arr + radix_sort_scratch_bytes(nnz)));
    char *base = static_cast<char *>(buf.p);
    int32_t *keys_sorted = reinterpret_cast<int32_t *>(base);
    int32_t *row_of = reinterpret_cast<int32_t *>(base + arr);
    hipLaunchKernelGGL(entry_rows_kernel, dim3((unsigned)ceil_div(nnz, kRowsTile)), dim3(kThreads), 0, s, n_rows, nnz,
                       d_row_ptr, row_of);
    TCG_TRY(radix_sort_pairs(d_col_idx, nullptr, nnz, nullptr, bits, keys_sorted, d_perm, base + 2 * arr, s));
    hipLaunchKernelGGL(transpose_finish_kernel, dim3((unsigned)ceil_div(nnz, kThreads)), dim3(kThreads), 0, s, n_cols,
                       nnz, row_of, keys_sorted, d_perm, d_out_row_ptr, d_out_col_idx);
    TCG_TRY(launch_status("transpose_finish_kernel"));
    TCG_HIP(hipStreamSynchronize(s));     // the scratch goes back to the pool on return
    return TCG_OK;
}

}  // namespace tcg
