// Neighbour aggregation on condensed tiles (Algorithm 2 of the paper) with gfx950 MFMA.
//
// One workgroup (4 wavefronts) per row window of 16 rows that the plan assigned to this path,
// i.e. windows whose rows share enough neighbours that every gathered X row is reused several
// times.  The window's condensed columns (its sorted unique neighbour list from SGT) are walked
// in chunks of KC = 32:
//   InitSparse  the 16 x KC slice of the condensed adjacency is built in LDS in fp32 from the
//               window's edges and edge_to_col (repeated entries add up), then rounded to the
//               feature type when it is loaded as the MFMA A operand;
//   FetchDense  the KC neighbour rows named by col_to_row are copied into LDS with 16-byte
//               coalesced loads -- each unique neighbour is fetched once per window, which is
//               the traffic reduction SGT exists for;
//   TCcompute   v_mfma_f32_16x16x32 (bf16 or f16 inputs, fp32 accumulate); the feature dimension
//               is split in 16-column slices over the wavefronts, which share the A operand;
//   StoreDense  after the last chunk the accumulators are written to the window's rows of Y.
// Differences from the paper's kernel: the K extent of a tile is 32 (gfx950 bf16/f16 MFMA)
// instead of 8 (TF-32 WMMA), the column -> node map comes straight from SGT's col_to_row
// instead of being rebuilt per block, and the B operand is transposed by the LDS read itself
// (ds_read_b64_tr_b16), so the staged rows keep their row-major layout.
#include "common.h"
#include "devutil.h"

namespace tcg {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

constexpr int kTileBlock = 256;
constexpr int kWaves = kTileBlock / kWave;
constexpr int KC = 32;          // condensed columns per chunk = K of one MFMA
constexpr int kAStride = KC + 1;

// Staged X rows are padded so that consecutive rows start 32 bytes (8 LDS banks) apart modulo the
// 256-byte bank cycle: the transposing reads below then touch every bank exactly once per pass.
__host__ __device__ inline int32_t staged_row_stride(int32_t row_bytes)
{
    return row_bytes + ((32 - row_bytes % 256) + 256) % 256;
}

template <int DT>
__device__ __forceinline__ f32x4 mfma16(const uint32_t (&a)[4], const uint32_t (&b)[4], f32x4 c)
{
    if constexpr (DT == TCG_BF16) {
        bf16x8 va, vb;
        __builtin_memcpy(&va, a, 16);
        __builtin_memcpy(&vb, b, 16);
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, vb, c, 0, 0, 0);
    } else {
        f16x8 va, vb;
        __builtin_memcpy(&va, a, 16);
        __builtin_memcpy(&vb, b, 16);
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(va, vb, c, 0, 0, 0);
    }
}

// Edge values to the feature type.  Unit values (and their small integer sums for repeated
// entries) are exact in both 16-bit types, so without edge values truncation is exact.
template <int DT, bool EXACT>
__device__ __forceinline__ uint32_t pack2(float lo, float hi)
{
    if constexpr (DT == TCG_BF16) {
        if constexpr (EXACT) return (__float_as_uint(lo) >> 16) | (__float_as_uint(hi) & 0xFFFF0000u);
        else return (uint32_t)f32_to_bf16_bits(lo) | ((uint32_t)f32_to_bf16_bits(hi) << 16);
    } else {
        return (uint32_t)__half_as_ushort(__float2half_rn(lo)) | ((uint32_t)__half_as_ushort(__float2half_rn(hi)) << 16);
    }
}

typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;

// gfx950 transposing LDS read (ds_read_b64_tr_b16).  Inside each group of 16 lanes, lane i receives
// as its element e the element (i % 4) of the 8-byte chunk addressed by lane (i / 4 + 4 * e): a
// 4 x 16 block of 16-bit values stored row-major comes back with one column per lane.
__device__ __forceinline__ uint2 lds_read_tr16(const char *p)
{
    bf16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4 *)(p));
    uint2 r;
    __builtin_memcpy(&r, &v, 8);
    return r;
}

// K index of the MFMA operand element j (0..7) of lane group g (0..3) inside a 32-column chunk.  Any
// bijection works as long as A and B use the same one; this one makes the first four elements of all
// groups rows 0..15 and the last four rows 16..31, which keeps the transposing reads conflict-free.
__device__ __forceinline__ int chunk_k(int g, int j) { return (j < 4 ? 0 : 16) + 4 * g + (j & 3); }

// MAXS: 16-column slices of D per wavefront (D <= 64 * MAXS).
template <int DT, bool HAS_W, int MAXS>
__global__ __launch_bounds__(kTileBlock) void spmm_tile_kernel(
    int32_t n_rows, int64_t n_win, const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ edge_to_col,
    const int32_t *__restrict__ win_unique_ptr, const int32_t *__restrict__ col_to_row,
    const uint8_t *__restrict__ win_path, const float *__restrict__ w, const char *__restrict__ X,
    int64_t ldx_bytes, int32_t D, void *__restrict__ Y, int y_dt, int64_t ldy)
{
    extern __shared__ __align__(16) char smem[];
    // Workgroup i runs on die i % kXcds: give every die a contiguous range of windows, so that
    // neighbouring windows (which share neighbours on clustered graphs) meet in the same L2.
    const int64_t per_die = (n_win + kXcds - 1) / kXcds;
    const int64_t win = (int64_t)(blockIdx.x % kXcds) * per_die + blockIdx.x / kXcds;
    if (win >= n_win || !win_path[win]) return;

    const int32_t row_bytes = D * 2;
    const int32_t rs = staged_row_stride(row_bytes);              // staged row stride, bytes (multiple of 16)
    char *xs = smem;                                              // KC rows
    float *a32 = reinterpret_cast<float *>(smem + (size_t)KC * rs);   // 16 x kAStride
    int32_t *s_rp = reinterpret_cast<int32_t *>(a32 + 16 * kAStride);   // 17 row pointers

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid >> 6;
    const int64_t r0 = win * 16;
    if (tid < 17) {
        int64_t r = r0 + tid;
        s_rp[tid] = row_ptr[r < n_rows ? r : n_rows];
    }
    __syncthreads();
    const int32_t lo = s_rp[0], hi = s_rp[16];
    const int32_t u0 = win_unique_ptr[win];
    const int32_t U = win_unique_ptr[win + 1] - u0;
    const int32_t n_chunks16 = row_bytes / 16;
    const int32_t n_slices = (D + 15) / 16;

    f32x4 acc[MAXS];
#pragma unroll
    for (int i = 0; i < MAXS; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};

    // A window of at most 2 * kTileBlock edges keeps them in registers for all chunks (condensed
    // column, offset of its row inside the A slice, value); larger windows re-read them per chunk.
    constexpr int EPT = 2;
    const bool edges_in_regs = hi - lo <= EPT * kTileBlock;
    int32_t e_col[EPT];
    int e_aoff[EPT];
    float e_val[EPT];
#pragma unroll
    for (int q = 0; q < EPT; ++q) {
        const int32_t e = lo + tid + q * kTileBlock;
        e_col[q] = -1;
        e_aoff[q] = 0;
        e_val[q] = 0.f;
        if (edges_in_regs && e < hi) {
            e_col[q] = edge_to_col[e];
            e_val[q] = HAS_W ? w[e] : 1.f;
            int r = 0;
#pragma unroll
            for (int step = 8; step > 0; step >>= 1)
                if (s_rp[r + step] <= e) r += step;
            e_aoff[q] = r * kAStride;
        }
    }

    // FetchDense: one row is n_chunks16 16-byte pieces; a thread owns pieces idx = tid + i * kTileBlock
    // of each KC x n_chunks16 chunk (rows beyond the window's list are zero).
    int32_t p_k[MAXS], p_goff[MAXS], p_loff[MAXS];     // row in chunk, byte offset in the row, LDS offset
#pragma unroll
    for (int i = 0; i < MAXS; ++i) {
        const int32_t idx = tid + i * kTileBlock;
        const int32_t k = idx / n_chunks16, ch = idx - k * n_chunks16;
        p_k[i] = idx < KC * n_chunks16 ? k : -1;
        p_goff[i] = ch * 16;
        p_loff[i] = k * rs + ch * 16;
    }
    // MFMA operand addressing (constant over the chunks).
    const int g = lane >> 4, n_in = lane & 15;
    // A: row n_in of the slice, K elements chunk_k(g, 0..7)
    const float *a_lo = a32 + n_in * kAStride + 4 * g;            // k = 4g .. 4g+3
    const float *a_hi = a_lo + 16;                                // k = 16+4g .. 16+4g+3
    // B: lane j of a 16-lane group addresses row (4g + j / 4) [+16 for the second read], 8-byte chunk j % 4
    const int32_t b_off = (4 * g + (n_in >> 2)) * rs + (n_in & 3) * 8;

    // The chunks are processed in groups of PD whose neighbour rows are requested at once (ids first,
    // then the rows).  Measured on MI355X, deeper groups lose more through register pressure (fewer
    // resident workgroups) than they gain in memory-level parallelism: PD = 1 is fastest.
    constexpr int PD = 1;
    for (int32_t kg = 0; kg < U; kg += PD * KC) {
        uint4 pre[PD][MAXS];
        int32_t nid[PD][MAXS];
#pragma unroll
        for (int c = 0; c < PD; ++c)
#pragma unroll
            for (int i = 0; i < MAXS; ++i) {
                const int32_t k = kg + c * KC + p_k[i];
                nid[c][i] = (p_k[i] >= 0 && k < U) ? col_to_row[u0 + k] : -1;
            }
#pragma unroll
        for (int c = 0; c < PD; ++c)
#pragma unroll
            for (int i = 0; i < MAXS; ++i) {
                pre[c][i] = make_uint4(0, 0, 0, 0);
                if (nid[c][i] >= 0)
                    pre[c][i] = *reinterpret_cast<const uint4 *>(X + (int64_t)nid[c][i] * ldx_bytes + p_goff[i]);
            }
#pragma unroll
        for (int c = 0; c < PD; ++c) {
            const int32_t k0 = kg + c * KC;
            if (k0 >= U) break;
            for (int i = tid; i < 16 * kAStride; i += kTileBlock) a32[i] = 0.f;
#pragma unroll
            for (int i = 0; i < MAXS; ++i)
                if (p_k[i] >= 0) *reinterpret_cast<uint4 *>(xs + p_loff[i]) = pre[c][i];
            __syncthreads();
            // InitSparse: scatter the window's edges that fall into this chunk.
            if (edges_in_regs) {
#pragma unroll
                for (int q = 0; q < EPT; ++q) {
                    const int32_t cc = e_col[q] - k0;
                    if (cc >= 0 && cc < KC) atomicAdd(&a32[e_aoff[q] + cc], e_val[q]);
                }
            } else {
                for (int32_t e = lo + tid; e < hi; e += kTileBlock) {
                    int32_t cc = edge_to_col[e] - k0;
                    if (cc >= 0 && cc < KC) {
                        int r = 0;
#pragma unroll
                        for (int step = 8; step > 0; step >>= 1)
                            if (s_rp[r + step] <= e) r += step;
                        atomicAdd(&a32[r * kAStride + cc], HAS_W ? w[e] : 1.f);
                    }
                }
            }
            __syncthreads();
            // TCcompute.
            uint32_t af[4];
            af[0] = pack2<DT, !HAS_W>(a_lo[0], a_lo[1]);
            af[1] = pack2<DT, !HAS_W>(a_lo[2], a_lo[3]);
            af[2] = pack2<DT, !HAS_W>(a_hi[0], a_hi[1]);
            af[3] = pack2<DT, !HAS_W>(a_hi[2], a_hi[3]);
#pragma unroll
            for (int i = 0; i < MAXS; ++i) {
                const int sl = wave + kWaves * i;
                if (sl < n_slices) {  // D is a multiple of 8: columns of a half slice beyond D read padding and are never stored
                    const char *p = xs + b_off + sl * 32;
                    const uint2 b0 = lds_read_tr16(p);
                    const uint2 b1 = lds_read_tr16(p + 16 * rs);
                    const uint32_t bf[4] = {b0.x, b0.y, b1.x, b1.y};
                    acc[i] = mfma16<DT>(af, bf, acc[i]);
                }
            }
            __syncthreads();
        }
    }

    // StoreDense: lane holds rows 4 * (lane / 16) + r, column lane % 16 of each of its slices.
#pragma unroll
    for (int i = 0; i < MAXS; ++i) {
        const int sl = wave + kWaves * i;
        if (sl >= n_slices) continue;
        const int n = sl * 16 + n_in;
        if (n >= D) continue;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int64_t row = r0 + 4 * g + r;
            if (row < n_rows) {
                if (y_dt == TCG_F32) static_cast<float *>(Y)[row * ldy + n] = acc[i][r];
                else store_elem(Y, row * ldy + n, y_dt, acc[i][r]);
            }
        }
    }
}

template <int DT, bool HAS_W, int MAXS>
void launch(const tcg_meta *m, const void *X, int64_t ldx, int32_t D, const float *w, void *Y, int y_dt,
            int64_t ldy, hipStream_t s)
{
    const size_t lds = (size_t)KC * staged_row_stride(D * 2) + 16 * kAStride * sizeof(float) + 17 * sizeof(int32_t);
    hipLaunchKernelGGL((spmm_tile_kernel<DT, HAS_W, MAXS>), dim3((unsigned)(kXcds * ceil_div(m->n_win, kXcds))), dim3(kTileBlock), lds, s,
                       m->n_rows, m->n_win, m->d_row_ptr, m->d_edge_to_col, m->d_win_unique_ptr, m->d_col_to_row,
                       m->d_win_path, w, static_cast<const char *>(X), ldx * 2, D, Y, y_dt, ldy);
}

template <int DT, bool HAS_W>
void launch_s(const tcg_meta *m, const void *X, int64_t ldx, int32_t D, const float *w, void *Y, int y_dt,
              int64_t ldy, hipStream_t s)
{
    if (D <= 64) launch<DT, HAS_W, 1>(m, X, ldx, D, w, Y, y_dt, ldy, s);
    else if (D <= 128) launch<DT, HAS_W, 2>(m, X, ldx, D, w, Y, y_dt, ldy, s);
    else if (D <= 256) launch<DT, HAS_W, 4>(m, X, ldx, D, w, Y, y_dt, ldy, s);
    else launch<DT, HAS_W, 8>(m, X, ldx, D, w, Y, y_dt, ldy, s);
}

}  // namespace

bool tile_path_supports(tcg_dtype x_dt, int32_t D, int64_t ldx, const void *X)
{
    return x_dt != TCG_F32 && D % 8 == 0 && D <= 512 && ldx % 8 == 0 &&
           (reinterpret_cast<uintptr_t>(X) & 15) == 0;
}

int spmm_tile_launch(tcg_meta *m, const void *d_X, tcg_dtype x_dt, int32_t D, int64_t ldx, const float *d_w,
                     void *d_Y, tcg_dtype y_dt, int64_t ldy, hipStream_t s)
{
    if (x_dt == TCG_BF16) {
        if (d_w) launch_s<TCG_BF16, true>(m, d_X, ldx, D, d_w, d_Y, (int)y_dt, ldy, s);
        else launch_s<TCG_BF16, false>(m, d_X, ldx, D, d_w, d_Y, (int)y_dt, ldy, s);
    } else {
        if (d_w) launch_s<TCG_F16, true>(m, d_X, ldx, D, d_w, d_Y, (int)y_dt, ldy, s);
        else launch_s<TCG_F16, false>(m, d_X, ldx, D, d_w, d_Y, (int)y_dt, ldy, s);
    }
    return launch_status("spmm_tile_kernel");
}

}  // namespace tcg
