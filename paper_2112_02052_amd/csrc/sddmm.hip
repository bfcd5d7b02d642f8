// Edge feature computation out[e] = <X[i], X[col_idx[e]]> (Equation 2 / Algorithm 3 of the
// paper), gather path, and the row-wise softmax of the attention-style workload.
//
// Same decomposition as the SpMM gather path: a group of G lanes owns a row segment, keeps its
// 16-byte slices of x_i in registers, streams the neighbour rows x_j through fully coalesced
// 16-byte loads (ids prefetched one iteration ahead), multiplies lane-locally and adds across
// the G lanes with wavefront shuffles.  UNROLL edges are reduced together by a butterfly that
// halves the number of live partial sums at every step, so the cross-lane cost is about one
// shuffle per edge instead of log2(G), and the results land in consecutive lanes for one
// coalesced store.  The output is already in edgeList order; no dense-to-sparse step is needed
// on this path.
#include "common.h"
#include "devutil.h"

namespace tcg {

// sddmm_tile.hip
int sddmm_tile_launch(tcg_meta *m, const void *d_P, int64_t ldp, const void *d_Q, int64_t ldq, tcg_dtype x_dt,
                      int32_t D, float *d_out, hipStream_t s);

namespace {

constexpr int kBlock = 256;
constexpr int64_t kSlabBytes = 256;                       // see sddmm_impl
constexpr int64_t kSlabMinMatrixBytes = (int64_t)64 << 20;

// After group_reduce with G >= UNROLL, lane (position in group) `l` holds the total of partial
// index idx(l): step off=1 keeps index parity = bit 0 of l as the LOWEST bit of the original
// index, the next step bit 1, and so on; so idx(l) = l mod UNROLL.
// PB: bytes a lane reads per piece; n_chunks = pieces per row.  16 is the normal case, smaller pieces
// serve rows that cannot be read in 16-byte chunks.
template <int DT, int G, int NCH, int UNROLL, int PB>
__global__ __launch_bounds__(kBlock) void sddmm_gather_kernel(
    const int32_t *__restrict__ lane_tab, const int32_t *__restrict__ seg_row, const int32_t *__restrict__ seg_ebeg,
    const int32_t *__restrict__ seg_dst, const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx,
    const char *__restrict__ P, int64_t ldp_bytes, const char *__restrict__ X, int64_t ldx_bytes, int32_t n_chunks,
    float *__restrict__ out, const uint8_t *__restrict__ win_path, int32_t win_h, int accumulate)
{
    using Pc = Piece<DT, PB>;
    constexpr bool ELEM = PB != 16;
    constexpr int VEC = Pc::VEC;
    const int lane = threadIdx.x % G;
    const int64_t seg = plan_segment(lane_tab, kBlock / G, threadIdx.x / G);
    if (seg < 0) return;              // G divides the wavefront: whole groups leave together
    const int32_t row = seg_row[seg];
    if (win_path != nullptr && win_path[row / win_h]) return;
    const int32_t eb = seg_ebeg[seg];
    const int32_t ee = segment_end(eb, seg_dst[seg], row, row_ptr);

    if (eb >= ee) return;                  // empty row: nothing to write, so its P row is not read either
    float xi[NCH][VEC];
    {
        const char *xr = P + (int64_t)row * ldp_bytes;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            int chunk = lane + c * G;
#pragma unroll
            for (int k = 0; k < VEC; ++k) xi[c][k] = 0.f;
            if (chunk < n_chunks) Pc::load(xr + (int64_t)chunk * Pc::BYTES, xi[c]);
        }
    }

    // Ids are read from clamped, valid positions (no predicate, issued back to back), a block of IDB entries -- a
    // whole cache line of them -- at a time and once per lane group: lane l takes entries l, l + G, ... of the block
    // and the values are handed round inside the group (every lane loading all of its step's ids costs more load
    // instructions than narrow rows do; asked for step by step, eight at a time, a line of ids had left the L2
    // again before the next step wanted it).  The next block's ids go out before this block's row loads.
    const int32_t last = ee - 1;
    const uint32_t ldx32 = (uint32_t)ldx_bytes;
    constexpr int IDB = G <= 4 ? 16 : (UNROLL * 8 < (G > 32 ? 64 : 32) ? UNROLL * 8 : (G > 32 ? 64 : 32));
    constexpr int PER = (IDB + G - 1) / G;
    constexpr int STEPS = IDB / UNROLL;
    auto request = [&](int32_t e0, int32_t (&mc)[PER]) {
#pragma unroll
        for (int k = 0; k < PER; ++k) mc[k] = col_idx[min(e0 + lane + k * G, last)];
    };
    int32_t mc[PER];
    request(eb, mc);

    for (int32_t e0 = eb; e0 < ee; e0 += IDB) {
        int32_t mc_next[PER];
        request(e0 + IDB, mc_next);
        // The block's scores are collected in the layout of its ids (lane l: entries l, l + G, ...) and leave
        // together at its end, as whole lines where the block covers them; what an earlier feature slab left is
        // read the same way, ahead of the rows.  (Eight scores at a time: 32-byte stores that reached memory
        // one by one, and a line of the earlier slab's scores read once per step.)
        float res[PER], prev[PER];
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            res[k] = 0.f;
            prev[k] = 0.f;
            if constexpr (G >= UNROLL) {
                if (accumulate && lane + k * G < IDB && e0 + lane + k * G < ee) prev[k] = out[e0 + lane + k * G];
            }
        }
        static_for<STEPS>([&](auto step) {
            constexpr int S = decltype(step)::value;
            const int32_t e = e0 + S * UNROLL;
            if (e < ee) {
                int32_t cn[UNROLL];
                block_ids<G, UNROLL, PER, S>(mc, cn);
                float p[UNROLL];
                if constexpr (!ELEM) {
                    uint4 raw[UNROLL][NCH];
#pragma unroll
                    for (int u = 0; u < UNROLL; ++u) {
                        const char *xr = X + (uint64_t)(uint32_t)cn[u] * ldx32;
#pragma unroll
                        for (int c = 0; c < NCH; ++c) {
                            int chunk = lane + c * G;
                            raw[u][c] = make_uint4(0, 0, 0, 0);
                            if (e + u < ee && chunk < n_chunks)
                                raw[u][c] = *reinterpret_cast<const uint4 *>(xr + (uint32_t)chunk * 16u);
                        }
                    }
#pragma unroll
                    for (int u = 0; u < UNROLL; ++u) {
                        float a = 0.f;
#pragma unroll
                        for (int c = 0; c < NCH; ++c) {
                            float v[VEC];
                            unpack16<DT>(raw[u][c], v);
#pragma unroll
                            for (int k = 0; k < VEC; ++k) a = fmaf(xi[c][k], v[k], a);
                        }
                        p[u] = a;
                    }
                } else {
                    float v[UNROLL][NCH][VEC];
#pragma unroll
                    for (int u = 0; u < UNROLL; ++u) {
                        const char *xr = X + (int64_t)cn[u] * ldx_bytes;
#pragma unroll
                        for (int c = 0; c < NCH; ++c) {
                            int chunk = lane + c * G;
#pragma unroll
                            for (int k = 0; k < VEC; ++k) v[u][c][k] = 0.f;
                            if (e + u < ee && chunk < n_chunks) Pc::load(xr + (int64_t)chunk * Pc::BYTES, v[u][c]);
                        }
                    }
#pragma unroll
                    for (int u = 0; u < UNROLL; ++u) {
                        float a = 0.f;
#pragma unroll
                        for (int c = 0; c < NCH; ++c)
#pragma unroll
                            for (int k = 0; k < VEC; ++k) a = fmaf(xi[c][k], v[u][c][k], a);
                        p[u] = a;
                    }
                }
                float r = group_reduce<G, UNROLL>(p, lane);
                if constexpr (G >= UNROLL) {
                    // lane j < UNROLL holds the score of entry S * UNROLL + j of the block, whose place is lane
                    // (S * UNROLL + j) % G, element (S * UNROLL + j) / G
                    constexpr int FIRST = (S * UNROLL) % G;
                    const float moved = FIRST == 0 ? r : __shfl(r, lane - FIRST, G);
                    if (lane >= FIRST && lane < FIRST + UNROLL) res[(S * UNROLL) / G] = moved;
                } else {
                    if (lane == 0) {
#pragma unroll
                        for (int u = 0; u < UNROLL; ++u)
                            if (e + u < ee) out[e + u] = accumulate ? out[e + u] + p[u] : p[u];
                    }
                }
            }
        });
        if constexpr (G >= UNROLL) {
            // streaming stores: the scores are not read again by this launch and should not take the rows' place in L2
#pragma unroll
            for (int k = 0; k < PER; ++k)
                if (lane + k * G < IDB && e0 + lane + k * G < ee)       // (a group wider than the block: its upper lanes idle)
                    __builtin_nontemporal_store(res[k] + prev[k], &out[e0 + lane + k * G]);
        }
#pragma unroll
        for (int k = 0; k < PER; ++k) mc[k] = mc_next[k];
    }
}

// Any D / alignment: one wavefront per segment, lanes stride over the feature dimension.
__global__ __launch_bounds__(kBlock) void sddmm_gather_generic_kernel(
    const int32_t *__restrict__ lane_tab, const int32_t *__restrict__ seg_row, const int32_t *__restrict__ seg_ebeg,
    const int32_t *__restrict__ seg_dst, const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx, const void *__restrict__ P,
    int64_t ldp, const void *__restrict__ X, int x_dt, int64_t ldx, int32_t D, float *__restrict__ out,
    const uint8_t *__restrict__ win_path, int32_t win_h)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t seg = plan_segment(lane_tab, kBlock / kWave, threadIdx.x >> 6);
    if (seg < 0) return;
    const int32_t row = seg_row[seg];
    if (win_path != nullptr && win_path[row / win_h]) return;
    const int32_t eb = seg_ebeg[seg];
    const int32_t ee = segment_end(eb, seg_dst[seg], row, row_ptr);
    for (int32_t e = eb; e < ee; ++e) {
        const int64_t j = col_idx[e];
        float a = 0.f;
        for (int32_t d = lane; d < D; d += kWave)
            a = fmaf(load_elem(P, (int64_t)row * ldp + d, x_dt), load_elem(X, j * ldx + d, x_dt), a);
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) a += __shfl_xor(a, off, kWave);
        if (lane == 0) out[e] = a;
    }
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
    return v;
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// ---- row softmax ----------------------------------------------------------------------------------
// The kernel is bound by memory latency, not bandwidth: a row is a short chain of dependent round trips (where
// is the row -> its values -> the result), so it is laid out for as many independent chains in flight as
// possible and as few links per chain as possible.  Work is dealt out per wavefront, without LDS or barriers:
//   single-segment rows (at most kSegLen entries)  16 consecutive entries of the tail of the gather plan's
//       segment list per wavefront.  A tail entry carries the row's first edge (seg_ebeg) and its length
//       (seg_dst = -1 - length), so one round trip yields both; on graphs whose windows share few neighbours the
//       tail is ordered by row length, so the 16 rows are alike, and the wavefront runs the variant that fits
//       the longest: G lanes per row with S entries per lane in registers, (G, S) = (4, 2) up to 8 entries,
//       (8, 2) up to 16, (16, 2) up to 32, (16, 8) up to 128.  Rows without entries are in the list too (the
//       aggregation writes their zeros) and cost nothing here.
//   split rows of up to kGiantRow entries           one wavefront each, the row in registers (8, 16 or 32
//       values per lane), first edge and length from the plan's long-row table.
//   the few longer rows                            in pieces of kGiantChunk entries, see softmax_piece().
// All values a wavefront needs are requested before its first result is stored (input and output may be the
// same array, so the compiler keeps loads behind earlier stores).
constexpr int kTailRowsPerWave = 16;             // lanes 0 .. 15 look the rows up (more rows per wavefront cost
                                                 // registers, and with them resident wavefronts: measured slower)

template <int G, int S>
__device__ __forceinline__ void softmax_tail_rows(int32_t b_l, int32_t len_l, const float *in, float *out)
{
    constexpr int RPP = kWave / G;                   // rows per pass of the wavefront
    constexpr int PASSES = kTailRowsPerWave / RPP;
    constexpr int BATCH = PASSES * S > 32 ? 32 / S : PASSES;      // passes whose values are in registers together
    const int lane = threadIdx.x & (kWave - 1);
    const int gl = lane % G;
#pragma unroll
    for (int p0 = 0; p0 < PASSES; p0 += BATCH) {
        float v[BATCH][S];
        int32_t b[BATCH], e[BATCH];
#pragma unroll
        for (int q = 0; q < BATCH; ++q) {
            const int r = (p0 + q) * RPP + lane / G;
            b[q] = __shfl(b_l, r, kWave);
            e[q] = b[q] + __shfl(len_l, r, kWave);
#pragma unroll
            for (int i = 0; i < S; ++i) {
                const int32_t k = b[q] + gl + G * i;
                v[q][i] = k < e[q] ? in[k] : -INFINITY;
            }
        }
#pragma unroll
        for (int q = 0; q < BATCH; ++q) {
            float m = -INFINITY;
#pragma unroll
            for (int i = 0; i < S; ++i) m = fmaxf(m, v[q][i]);
#pragma unroll
            for (int off = 1; off < G; off <<= 1) m = fmaxf(m, __shfl_xor(m, off, kWave));
            float sum = 0.f;
#pragma unroll
            for (int i = 0; i < S; ++i) {
                v[q][i] = b[q] + gl + G * i < e[q] ? expf(v[q][i] - m) : 0.f;
                sum += v[q][i];
            }
#pragma unroll
            for (int off = 1; off < G; off <<= 1) sum += __shfl_xor(sum, off, kWave);
            const float inv = 1.f / sum;
#pragma unroll
            for (int i = 0; i < S; ++i) {
                const int32_t k = b[q] + gl + G * i;
                if (k < e[q]) out[k] = v[q][i] * inv;
            }
        }
    }
}

template <int R>
__device__ __forceinline__ void softmax_row_wave(int32_t b, int32_t e, const float *in, float *out)
{
    const int lane = threadIdx.x & (kWave - 1);
    float v[R];
    float m = -INFINITY;
#pragma unroll
    for (int i = 0; i < R; ++i) {
        const int32_t k = b + lane + kWave * i;
        v[i] = k < e ? in[k] : -INFINITY;
        m = fmaxf(m, v[i]);
    }
    m = wave_max(m);
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < R; ++i) {
        v[i] = b + lane + kWave * i < e ? expf(v[i] - m) : 0.f;
        sum += v[i];
    }
    const float inv = 1.f / wave_sum(sum);
#pragma unroll
    for (int i = 0; i < R; ++i) {
        const int32_t k = b + lane + kWave * i;
        if (k < e) out[k] = v[i] * inv;
    }
}

// The few longer rows are cut into pieces of kGiantChunk entries (the plan lists them), one workgroup per piece
// with the piece in registers, in two launches: the first leaves the (maximum, sum of exponentials) of every piece,
// in the second the workgroup of a piece merges the figures of its row's pieces in a fixed order and writes the
// normalised values.  A hub row of tens of thousands of entries is then spread over the chip instead of being a
// chain of round trips in one workgroup that outlasts the rest of the kernel (one workgroup per row, two passes:
// 54 us on the 1M-node graph, 30 of them the longest row's; a second launch *after* the main one to combine the
// pieces: 62 us).
constexpr int kPieceVals = kGiantChunk / kBlock;
constexpr int kWavesPerBlock = kBlock / kWave;

struct RowPiece {
    int32_t b, e;            // the piece's entries
    int32_t first, count;    // the pieces of its row in the list
};

__device__ __forceinline__ RowPiece giant_piece(int32_t k, const int32_t *gchunk_li, const int32_t *gchunk_c,
                                             const int32_t *long_ebeg, const int32_t *long_len)
{
    const int32_t li = gchunk_li[k], c = gchunk_c[k];
    const int32_t rb = long_ebeg[li], len = long_len[li];
    RowPiece p;
    p.b = rb + c * kGiantChunk;
    p.e = min(rb + len, p.b + kGiantChunk);
    p.first = k - c;
    p.count = (len + kGiantChunk - 1) / kGiantChunk;
    return p;
}

// Workgroup-wide maximum / sum in a fixed order.  Every thread of the workgroup calls them.
__device__ __forceinline__ float block_max(float v, float *s_red)
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    v = wave_max(v);
    __syncthreads();                                   // s_red may still be read from an earlier call
    if (lane == 0) s_red[wave] = v;
    __syncthreads();
    float r = s_red[0];
#pragma unroll
    for (int i = 1; i < kWavesPerBlock; ++i) r = fmaxf(r, s_red[i]);
    return r;
}

__device__ __forceinline__ float block_sum(float v, float *s_red)
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    v = wave_sum(v);
    __syncthreads();
    if (lane == 0) s_red[wave] = v;
    __syncthreads();
    float r = s_red[0];
#pragma unroll
    for (int i = 1; i < kWavesPerBlock; ++i) r += s_red[i];
    return r;
}

__global__ __launch_bounds__(kBlock) void softmax_piece_stats_kernel(const int32_t *__restrict__ gchunk_li,
                                                                     const int32_t *__restrict__ gchunk_c,
                                                                     const int32_t *__restrict__ long_ebeg,
                                                                     const int32_t *__restrict__ long_len,
                                                                     const float *__restrict__ in,
                                                                     float2 *__restrict__ stats)
{
    __shared__ float s_red[kWavesPerBlock];
    const RowPiece p = giant_piece((int32_t)blockIdx.x, gchunk_li, gchunk_c, long_ebeg, long_len);
    float v[kPieceVals];
    float m = -INFINITY;
#pragma unroll
    for (int u = 0; u < kPieceVals; ++u) {
        const int32_t k = p.b + threadIdx.x + u * kBlock;
        v[u] = k < p.e ? in[k] : -INFINITY;
        m = fmaxf(m, v[u]);
    }
    const float M = block_max(m, s_red);
    float sum = 0.f;
#pragma unroll
    for (int u = 0; u < kPieceVals; ++u) sum += v[u] > -INFINITY ? expf(v[u] - M) : 0.f;
    const float S = block_sum(sum, s_red);
    if (threadIdx.x == 0) stats[blockIdx.x] = make_float2(M, S);
}

__device__ __forceinline__ void softmax_piece(const RowPiece &p, const float2 *stats, const float *in, float *out,
                                              float *s_red)
{
    float v[kPieceVals];
#pragma unroll
    for (int u = 0; u < kPieceVals; ++u) {
        const int32_t k = p.b + threadIdx.x + u * kBlock;
        v[u] = k < p.e ? in[k] : -INFINITY;
    }
    float m = -INFINITY;
    for (int32_t i = threadIdx.x; i < p.count; i += kBlock) m = fmaxf(m, stats[p.first + i].x);
    const float M = block_max(m, s_red);
    float sum = 0.f;
    for (int32_t i = threadIdx.x; i < p.count; i += kBlock) {
        const float2 t = stats[p.first + i];
        sum += t.x > -INFINITY ? t.y * expf(t.x - M) : 0.f;
    }
    const float inv = 1.f / block_sum(sum, s_red);
#pragma unroll
    for (int u = 0; u < kPieceVals; ++u) {
        const int32_t k = p.b + threadIdx.x + u * kBlock;
        if (k < p.e) out[k] = expf(v[u] - M) * inv;
    }
}

// One launch, three kinds of workgroups in the order in which they should start: the pieces of the very long rows,
// then the other split rows (four per workgroup, one per wavefront), then the single-segment rows (64 per
// workgroup, 16 per wavefront).
__global__ __launch_bounds__(kBlock) void row_softmax_kernel(
    int32_t n_gchunks, const int32_t *__restrict__ gchunk_li, const int32_t *__restrict__ gchunk_c,
    const float2 *__restrict__ stats, int32_t n_long, const int32_t *__restrict__ long_ebeg,
    const int32_t *__restrict__ long_len, int32_t tail_start, int32_t tail_count,
    const int32_t *__restrict__ seg_ebeg, const int32_t *__restrict__ seg_dst, const float *in, float *out)
{
    __shared__ float s_red[kWavesPerBlock];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    int32_t blk = blockIdx.x;
    if (blk < n_gchunks) {
        softmax_piece(giant_piece(blk, gchunk_li, gchunk_c, long_ebeg, long_len), stats, in, out, s_red);
        return;
    }
    blk -= n_gchunks;
    const int32_t n_long_blocks = (n_long + kWavesPerBlock - 1) / kWavesPerBlock;
    if (blk < n_long_blocks) {
        const int32_t li = blk * kWavesPerBlock + wave;
        if (li >= n_long) return;
        const int32_t b = long_ebeg[li], len = long_len[li];
        if (len <= 8 * kWave) softmax_row_wave<8>(b, b + len, in, out);
        else if (len <= 16 * kWave) softmax_row_wave<16>(b, b + len, in, out);
        else if (len <= kGiantRow) softmax_row_wave<kGiantRow / kWave>(b, b + len, in, out);
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
    if (longest <= 8) softmax_tail_rows<4, 2>(b, len, in, out);
    else if (longest <= 16) softmax_tail_rows<8, 2>(b, len, in, out);
    else if (longest <= 32) softmax_tail_rows<16, 2>(b, len, in, out);
    else softmax_tail_rows<16, kSegLen / 16>(b, len, in, out);
}

template <int DT, int G, int NCH, int PB = 16>
void launch_sddmm(const tcg_meta *m, const void *P, int64_t ldp, const void *X, int64_t ldx, int32_t n_chunks,
                  float *out, const uint8_t *win_path, hipStream_t s, int accumulate = 0)
{
    // A group narrower than 8 lanes reduces 8 partial products with more shuffles and stores than
    // loads; it takes as many edges per step as it has lanes.
    constexpr int UNROLL = NCH == 1 ? (G < 8 ? G : 8) : (NCH == 2 ? 4 : 2);
    const unsigned grid = (unsigned)plan_grid(m->h_lane_tab, kBlock / G);
    hipLaunchKernelGGL((sddmm_gather_kernel<DT, G, NCH, UNROLL, PB>), dim3(grid), dim3(kBlock), 0, s, m->d_lane_tab,
                       m->d_seg_row, m->d_seg_ebeg, m->d_seg_dst, m->d_row_ptr, m->d_col_idx, static_cast<const char *>(P),
                       ldp * Elem<DT>::BYTES, static_cast<const char *>(X), ldx * Elem<DT>::BYTES, n_chunks, out, win_path,
                       m->win_h, accumulate);
}

template <int DT>
bool dispatch_sddmm(const tcg_meta *m, const void *P, int64_t ldp, const void *X, int64_t ldx, int32_t n_chunks,
                    float *out, const uint8_t *win_path, hipStream_t s, int accumulate = 0)
{
    if (n_chunks <= 4) launch_sddmm<DT, 4, 1>(m, P, ldp, X, ldx, n_chunks, out, win_path, s);
    else if (n_chunks <= 8) launch_sddmm<DT, 8, 1>(m, P, ldp, X, ldx, n_chunks, out, win_path, s);
    else if (n_chunks <= 16) launch_sddmm<DT, 16, 1>(m, P, ldp, X, ldx, n_chunks, out, win_path, s, accumulate);
    else if (n_chunks <= 32) launch_sddmm<DT, 32, 1>(m, P, ldp, X, ldx, n_chunks, out, win_path, s);
    else if (n_chunks <= 64) launch_sddmm<DT, 64, 1>(m, P, ldp, X, ldx, n_chunks, out, win_path, s);
    else if (n_chunks <= 128) launch_sddmm<DT, 64, 2>(m, P, ldp, X, ldx, n_chunks, out, win_path, s);
    else if (n_chunks <= 256) launch_sddmm<DT, 64, 4>(m, P, ldp, X, ldx, n_chunks, out, win_path, s);
    else return false;
    return true;
}

// Rows read in pieces of PB < 16 bytes: up to 256 pieces per row.
template <int DT, int PB>
bool dispatch_sddmm_small(const tcg_meta *m, const void *P, int64_t ldp, const void *X, int64_t ldx, int32_t D,
                          float *out, const uint8_t *win_path, hipStream_t s)
{
    const int32_t n = D / Piece<DT, PB>::VEC;
    if (n <= 4) launch_sddmm<DT, 4, 1, PB>(m, P, ldp, X, ldx, n, out, win_path, s);
    else if (n <= 8) launch_sddmm<DT, 8, 1, PB>(m, P, ldp, X, ldx, n, out, win_path, s);
    else if (n <= 16) launch_sddmm<DT, 16, 1, PB>(m, P, ldp, X, ldx, n, out, win_path, s);
    else if (n <= 32) launch_sddmm<DT, 32, 1, PB>(m, P, ldp, X, ldx, n, out, win_path, s);
    else if (n <= 64) launch_sddmm<DT, 64, 1, PB>(m, P, ldp, X, ldx, n, out, win_path, s);
    else if (n <= 128) launch_sddmm<DT, 64, 2, PB>(m, P, ldp, X, ldx, n, out, win_path, s);
    else if (n <= 256) launch_sddmm<DT, 64, 4, PB>(m, P, ldp, X, ldx, n, out, win_path, s);
    else return false;
    return true;
}

template <int DT>
bool dispatch_sddmm_elem(const tcg_meta *m, const void *P, int64_t ldp, const void *X, int64_t ldx, int32_t D,
                         float *out, const uint8_t *win_path, hipStream_t s)
{
    if (small_piece_bytes(Elem<DT>::BYTES, D, ldp, ldx, P, X) == 4)
        return dispatch_sddmm_small<DT, 4>(m, P, ldp, X, ldx, D, out, win_path, s);
    if constexpr (DT != TCG_F32) return dispatch_sddmm_small<DT, 2>(m, P, ldp, X, ldx, D, out, win_path, s);
    return false;
}

}  // namespace

int sddmm_impl(tcg_meta *m, const void *d_P, int64_t ldp, const void *d_X, int64_t ldx, tcg_dtype x_dt, int32_t D,
               float *d_out, hipStream_t s)
{
    if (m->n_rows == 0 || m->nnz == 0) return TCG_OK;
    // fp32 rows take the tile path (six MFMAs per product) only where it was measured to pay; a forced policy
    // is taken literally
    const bool wide_enough = x_dt != TCG_F32 || m->policy == TCG_POLICY_TILE ||
                             (D >= kTileMinWidthFew && (float)m->nnz_tile >= kTileMinReuseF32Sddmm * (float)m->unique_tile);
    const bool use_tiles = m->n_tile_win > 0 && m->win_h == 16 && wide_enough &&
                           sddmm_tile_supports(x_dt, D, ldx, d_X) && sddmm_tile_supports(x_dt, D, ldp, d_P);
    const uint8_t *win_path = use_tiles ? m->d_win_path : nullptr;
    if (use_tiles) TCG_TRY(sddmm_tile_launch(m, d_P, ldp, d_X, ldx, x_dt, D, d_out, s));
    if (use_tiles && m->nnz_tile == m->nnz) return TCG_OK;

    const int es = dtype_size(x_dt);
    const bool vec_ok = ((int64_t)D * es) % 16 == 0 && (ldx * es) % 16 == 0 && ldx * es < (1ll << 32) &&
                        (ldp * es) % 16 == 0 && (reinterpret_cast<uintptr_t>(d_X) & 15) == 0 &&
                        (reinterpret_cast<uintptr_t>(d_P) & 15) == 0;
    bool done = false;
    if (vec_ok) {
        const int64_t row_bytes = (int64_t)D * es;
        // As in the aggregation, rows of 512 bytes and more are gathered in slabs of 256 bytes, one launch per
        // slab, when the operand exceeds the caches; a later slab adds its share of the dot product to what the
        // earlier ones left in d_out (read back with the column ids, ahead of the rows).  Measured on the 1M-node
        // R-MAT graph, old and new side by side: fp32 D = 128 1.18 -> 1.16 ms, D = 256 2.65 -> 2.52 ms, bf16
        // D = 512 2.63 -> 2.38 ms.
        int slabs = 1;
        if (row_bytes >= 512 && row_bytes % kSlabBytes == 0 && (int64_t)m->n_cols * row_bytes >= kSlabMinMatrixBytes)
            slabs = (int)(row_bytes / kSlabBytes);
        const int32_t n_chunks = (int32_t)(row_bytes / slabs / 16);
        done = true;
        for (int sl = 0; sl < slabs && done; ++sl) {
            const char *Ps = static_cast<const char *>(d_P) + (int64_t)sl * kSlabBytes;
            const char *Xs = static_cast<const char *>(d_X) + (int64_t)sl * kSlabBytes;
            if (x_dt == TCG_F32) done = dispatch_sddmm<TCG_F32>(m, Ps, ldp, Xs, ldx, n_chunks, d_out, win_path, s, sl > 0);
            else if (x_dt == TCG_BF16) done = dispatch_sddmm<TCG_BF16>(m, Ps, ldp, Xs, ldx, n_chunks, d_out, win_path, s, sl > 0);
            else done = dispatch_sddmm<TCG_F16>(m, Ps, ldp, Xs, ldx, n_chunks, d_out, win_path, s, sl > 0);
        }
    }
    if (!done) {
        if (x_dt == TCG_F32) done = dispatch_sddmm_elem<TCG_F32>(m, d_P, ldp, d_X, ldx, D, d_out, win_path, s);
        else if (x_dt == TCG_BF16) done = dispatch_sddmm_elem<TCG_BF16>(m, d_P, ldp, d_X, ldx, D, d_out, win_path, s);
        else done = dispatch_sddmm_elem<TCG_F16>(m, d_P, ldp, d_X, ldx, D, d_out, win_path, s);
    }
    if (!done) {
        const unsigned grid = (unsigned)plan_grid(m->h_lane_tab, kBlock / kWave);
        hipLaunchKernelGGL(sddmm_gather_generic_kernel, dim3(grid), dim3(kBlock), 0, s, m->d_lane_tab, m->d_seg_row,
                           m->d_seg_ebeg, m->d_seg_dst, m->d_row_ptr, m->d_col_idx, d_P, ldp, d_X, (int)x_dt, ldx, D, d_out, win_path,
                           m->win_h);
    }
    return launch_status("sddmm_gather_kernel");
}

int row_softmax_impl(const tcg_meta *m, const float *d_in, float *d_out, hipStream_t s)
{
    if (m->n_rows == 0 || m->nnz == 0) return TCG_OK;
    const int32_t tail_start = m->h_lane_tab[4], tail_count = m->h_lane_tab[5];
    const int64_t grid = m->n_gchunks + ceil_div(m->n_long, kWavesPerBlock) +
                         ceil_div(tail_count, kWavesPerBlock * kTailRowsPerWave);
    float2 *stats = reinterpret_cast<float2 *>(m->d_partial_ml);        // one pair per piece; pieces <= slots
    if (m->n_gchunks > 0)
        hipLaunchKernelGGL(softmax_piece_stats_kernel, dim3((unsigned)m->n_gchunks), dim3(kBlock), 0, s, m->d_gchunk_li,
                           m->d_gchunk_c, m->d_long_ebeg, m->d_long_len, d_in, stats);
    if (grid > 0) {
        hipLaunchKernelGGL(row_softmax_kernel, dim3((unsigned)grid), dim3(kBlock), 0, s, (int32_t)m->n_gchunks,
                           m->d_gchunk_li, m->d_gchunk_c, stats, (int32_t)m->n_long, m->d_long_ebeg, m->d_long_len,
                           tail_start, tail_count, m->d_seg_ebeg, m->d_seg_dst, d_in, d_out);
        TCG_TRY(launch_status("row_softmax_kernel"));
    }
    return TCG_OK;
}

}  // namespace tcg
