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
// instead of being rebuilt per block, and the B operand is transposed on the LDS read side.
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
constexpr int kRowPad = 8;      // bytes added to every staged X row (spreads the K-strided reads over banks)

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

template <int DT>
__device__ __forceinline__ uint32_t pack2(float lo, float hi)
{
    if constexpr (DT == TCG_BF16) return (uint32_t)f32_to_bf16_bits(lo) | ((uint32_t)f32_to_bf16_bits(hi) << 16);
    else return (uint32_t)__half_as_ushort(__float2half_rn(lo)) | ((uint32_t)__half_as_ushort(__float2half_rn(hi)) << 16);
}

// MAXS: 16-column slices of D per wavefront (D <= 64 * MAXS).
template <int DT, bool HAS_W, int MAXS>
__global__ __launch_bounds__(kTileBlock) void spmm_tile_kernel(
    int32_t n_rows, const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ edge_to_col,
    const int32_t *__restrict__ win_unique_ptr, const int32_t *__restrict__ col_to_row,
    const uint8_t *__restrict__ win_path, const float *__restrict__ w, const char *__restrict__ X,
    int64_t ldx_bytes, int32_t D, void *__restrict__ Y, int y_dt, int64_t ldy)
{
    extern __shared__ __align__(16) char smem[];
    const int64_t win = blockIdx.x;
    if (!win_path[win]) return;

    const int32_t row_bytes = D * 2;
    const int32_t rs = row_bytes + kRowPad;                       // staged row stride, bytes
    char *xs = smem;                                              // KC rows
    float *a32 = reinterpret_cast<float *>(smem + (size_t)KC * rs);   // 16 x kAStride (offset is 8-byte aligned)
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

    for (int32_t k0 = 0; k0 < U; k0 += KC) {
        for (int i = tid; i < 16 * kAStride; i += kTileBlock) a32[i] = 0.f;
        // FetchDense: KC neighbour rows -> LDS (rows beyond the window's list are zero).
        for (int32_t idx = tid; idx < KC * n_chunks16; idx += kTileBlock) {
            int32_t k = idx / n_chunks16, ch = idx - k * n_chunks16;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (k0 + k < U)
                v = *reinterpret_cast<const uint4 *>(X + (int64_t)col_to_row[u0 + k0 + k] * ldx_bytes + (int64_t)ch * 16);
            uint2 *dst = reinterpret_cast<uint2 *>(xs + (size_t)k * rs + (size_t)ch * 16);
            dst[0] = make_uint2(v.x, v.y);
            dst[1] = make_uint2(v.z, v.w);
        }
        __syncthreads();
        // InitSparse: scatter the window's edges that fall into this chunk.
        for (int32_t e = lo + tid; e < hi; e += kTileBlock) {
            int32_t c = edge_to_col[e] - k0;
            if (c >= 0 && c < KC) {
                int r = 0;
#pragma unroll
                for (int step = 8; step > 0; step >>= 1)
                    if (s_rp[r + step] <= e) r += step;
                atomicAdd(&a32[r * kAStride + c], HAS_W ? w[e] : 1.f);
            }
        }
        __syncthreads();
        // TCcompute.
        const int m = lane & 15, kb = (lane >> 4) * 8;
        uint32_t af[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            af[j] = pack2<DT>(a32[m * kAStride + kb + 2 * j], a32[m * kAStride + kb + 2 * j + 1]);
#pragma unroll
        for (int i = 0; i < MAXS; ++i) {
            const int sl = wave + kWaves * i;
            if (sl < n_slices) {
                const int n = sl * 16 + (lane & 15);
                uint32_t bf[4] = {0, 0, 0, 0};
                if (n < D) {
                    const char *p = xs + (size_t)kb * rs + (size_t)n * 2;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        uint32_t v0 = *reinterpret_cast<const uint16_t *>(p + (size_t)(2 * j) * rs);
                        uint32_t v1 = *reinterpret_cast<const uint16_t *>(p + (size_t)(2 * j + 1) * rs);
                        bf[j] = v0 | (v1 << 16);
                    }
                }
                acc[i] = mfma16<DT>(af, bf, acc[i]);
            }
        }
        __syncthreads();
    }

    // StoreDense: lane holds rows 4 * (lane / 16) + r, column lane % 16 of each of its slices.
#pragma unroll
    for (int i = 0; i < MAXS; ++i) {
        const int sl = wave + kWaves * i;
        if (sl >= n_slices) continue;
        const int n = sl * 16 + (lane & 15);
        if (n >= D) continue;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            int64_t row = r0 + 4 * (lane >> 4) + r;
            if (row < n_rows) store_elem(Y, row * ldy + n, y_dt, acc[i][r]);
        }
    }
}

template <int DT, bool HAS_W, int MAXS>
void launch(const tcg_meta *m, const void *X, int64_t ldx, int32_t D, const float *w, void *Y, int y_dt,
            int64_t ldy, hipStream_t s)
{
    const size_t lds = (size_t)KC * (D * 2 + kRowPad) + 16 * kAStride * sizeof(float) + 17 * sizeof(int32_t);
    hipLaunchKernelGGL((spmm_tile_kernel<DT, HAS_W, MAXS>), dim3((unsigned)m->n_win), dim3(kTileBlock), lds, s,
                       m->n_rows, m->d_row_ptr, m->d_edge_to_col, m->d_win_unique_ptr, m->d_col_to_row,
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
