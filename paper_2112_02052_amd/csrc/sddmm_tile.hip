// Edge feature computation on condensed tiles (Algorithm 3 of the paper) with gfx950 MFMA.
//
// One workgroup (4 wavefronts) per row window of 16 rows assigned to the tile path.  Here the
// contraction runs over the feature dimension, which is contiguous in memory for both operands,
// so the MFMA operands are loaded straight from global memory with 16-byte loads:
//   FetchDenseRow  XTile_A = the window's own 16 rows (of P; P = X in the paper's operation), kept in
//                  registers for the whole window;
//   FetchDenseCol  XTile_B = 16 neighbour rows named by col_to_row (each unique neighbour once);
//   TCcompute      v_mfma_f32_16x16x32 accumulated over all of D before anything is written
//                  (section 4.3: the result is only output after all iterations along the
//                  embedding dimension);
//   StoreSparse    the 16 x 16 output tiles of up to 256 condensed columns are parked in LDS and
//                  every edge of the window picks its value through edge_to_col, which yields
//                  the edgeList-ordered output.
#include "common.h"
#include "devutil.h"

namespace tcg {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

constexpr int kTileBlock = 256;
constexpr int kWaves = kTileBlock / kWave;
constexpr int kCols = 256;            // condensed columns per LDS pass
constexpr int kEStride = kCols + 4;   // floats; 4 * stride = 16 (mod 64 banks): the four row groups of a tile miss each other

template <int DT>
__device__ __forceinline__ f32x4 mfma16(const uint4 &a, const uint4 &b, f32x4 c)
{
    if constexpr (DT == TCG_BF16) {
        bf16x8 va, vb;
        __builtin_memcpy(&va, &a, 16);
        __builtin_memcpy(&vb, &b, 16);
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, vb, c, 0, 0, 0);
    } else {
        f16x8 va, vb;
        __builtin_memcpy(&va, &a, 16);
        __builtin_memcpy(&vb, &b, 16);
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(va, vb, c, 0, 0, 0);
    }
}

// Orders the LDS accesses of the wavefront's lanes for the compiler; the hardware already completes a
// wavefront's LDS operations in program order, so no instruction is emitted.
__device__ __forceinline__ void wave_lds_order()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// KSTEPS = ceil(D / 32) rounded up to a power of two; steps beyond D contribute zeros.
template <int DT, int KSTEPS>
__global__ __launch_bounds__(kTileBlock) void sddmm_tile_kernel(
    int32_t n_rows, int64_t n_win, const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ edge_to_col,
    const int32_t *__restrict__ win_unique_ptr, const int32_t *__restrict__ col_to_row,
    const uint8_t *__restrict__ win_path, const char *__restrict__ P, int64_t ldp_bytes,
    const char *__restrict__ X, int64_t ldx_bytes, int32_t D, float *__restrict__ out, bool skip_few)
{
    __shared__ float s_e[16 * kEStride];
    __shared__ int32_t s_rp[17];
    // Workgroup i runs on die i % kXcds: give every die a contiguous range of windows, so that
    // neighbouring windows (which share neighbours on clustered graphs) meet in the same L2.
    const int64_t per_die = (n_win + kXcds - 1) / kXcds;
    const int64_t win = (int64_t)(blockIdx.x % kXcds) * per_die + blockIdx.x / kXcds;
    if (win >= n_win || !win_path[win] || (skip_few && win_path[win] == kTileFew)) return;

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
    const int32_t cb = row_ptr[r0];             // the window's list sits at its edge offset
    const int32_t U = win_unique_ptr[win + 1] - u0;
    const int32_t row_bytes = D * 2;
    const int n = lane & 15;                    // tile row (A) / tile column (B) of this lane
    const int32_t koff = (lane >> 4) * 16;      // byte offset of the lane's 8 features inside a 64-byte K step

    uint4 a[KSTEPS];
    {
        const int64_t row = r0 + n;
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
            int32_t off = kk * 64 + koff;
            a[kk] = make_uint4(0, 0, 0, 0);
            if (row < n_rows && off < row_bytes) a[kk] = *reinterpret_cast<const uint4 *>(P + row * ldp_bytes + off);
        }
    }

    for (int32_t c0 = 0; c0 < U; c0 += kCols) {
        for (int t = wave; t < kCols / 16 && c0 + t * 16 < U; t += kWaves) {
            const int32_t col = c0 + t * 16 + n;
            const int64_t node = col < U ? col_to_row[cb + col] : -1;
            uint4 b[KSTEPS];
#pragma unroll
            for (int kk = 0; kk < KSTEPS; ++kk) {
                int32_t off = kk * 64 + koff;
                b[kk] = make_uint4(0, 0, 0, 0);
                if (node >= 0 && off < row_bytes) b[kk] = *reinterpret_cast<const uint4 *>(X + node * ldx_bytes + off);
            }
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < KSTEPS; ++kk) acc = mfma16<DT>(a[kk], b[kk], acc);
#pragma unroll
            for (int r = 0; r < 4; ++r) s_e[(4 * (lane >> 4) + r) * kEStride + t * 16 + n] = acc[r];
        }
        __syncthreads();
        // StoreSparse: dense tile -> edgeList order.
        for (int32_t e = lo + tid; e < hi; e += kTileBlock) {
            int32_t c = edge_to_col[e] - c0;
            if (c >= 0 && c < kCols) {
                int r = 0;
#pragma unroll
                for (int step = 8; step > 0; step >>= 1)
                    if (s_rp[r + step] <= e) r += step;
                out[e] = s_e[r * kEStride + c];
            }
        }
        __syncthreads();
    }
}

// ---- one wavefront per window (class kTileFew: at most kTileFewEdges edges, kept in registers) ----------
// No barrier, 1 KB of LDS per window (one 16 x 16 score tile), the B operand of the next tile column is
// requested before the current one is multiplied, and the window's edges (row, condensed column) wait in
// registers for their tile column to come by: after each tile column every lane looks its edges up in
// the tile and writes those that fall into it.
constexpr int kScoreStride = 17;

template <int DT, int KSTEPS>
__global__ __launch_bounds__(kWave) void sddmm_tile_wave_kernel(
    int32_t n_rows, int64_t n_win, const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ edge_to_col,
    const int32_t *__restrict__ win_unique_ptr, const int32_t *__restrict__ col_to_row,
    const uint8_t *__restrict__ win_path, const char *__restrict__ P, int64_t ldp_bytes,
    const char *__restrict__ X, int64_t ldx_bytes, int32_t D, float *__restrict__ out)
{
    constexpr int EPT = kTileFewEdges / kWave;
    __shared__ float s_e[16 * kScoreStride];
    __shared__ int32_t s_rp[17];
    const int64_t per_die = (n_win + kXcds - 1) / kXcds;
    const int64_t win = (int64_t)(blockIdx.x % kXcds) * per_die + blockIdx.x / kXcds;
    if (blockIdx.x / kXcds >= per_die || win >= n_win || win_path[win] != kTileFew) return;

    const int lane = threadIdx.x;
    const int n = lane & 15;                    // tile row (A) / tile column (B) of this lane
    const int kg = lane >> 4;                   // which 16 bytes of every 64-byte K step
    const int64_t r0 = win * 16;
    if (lane < 17) {
        int64_t r = r0 + lane;
        s_rp[lane] = row_ptr[r < n_rows ? r : n_rows];
    }
    const int32_t u0 = win_unique_ptr[win];
    const int32_t cb = row_ptr[r0];             // the window's list sits at its edge offset
    const int32_t U = win_unique_ptr[win + 1] - u0;
    const int32_t row_bytes = D * 2;
    int32_t nid = n < U ? col_to_row[cb + n] : -1;              // neighbour of tile column 0
    int32_t nid_nxt = 16 + n < U ? col_to_row[cb + 16 + n] : -1;

    uint4 a[KSTEPS];
    {
        const int64_t row = r0 + n;
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
            const int32_t off = kk * 64 + kg * 16;
            a[kk] = make_uint4(0, 0, 0, 0);
            if (row < n_rows && off < row_bytes) a[kk] = *reinterpret_cast<const uint4 *>(P + row * ldp_bytes + off);
        }
    }
    uint4 b[KSTEPS];
    auto fetch = [&](int32_t node) {
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
            const int32_t off = kk * 64 + kg * 16;
            b[kk] = make_uint4(0, 0, 0, 0);
            if (node >= 0 && off < row_bytes) b[kk] = *reinterpret_cast<const uint4 *>(X + (int64_t)node * ldx_bytes + off);
        }
    };
    fetch(nid);

    wave_lds_order();
    const int32_t lo = s_rp[0], hi = s_rp[16];
    // the window's edges: (score-tile row offset << 16 | condensed column); larger windows (only a forced
    // policy puts them here) re-read their edges for every tile column
    const bool edges_in_regs = hi - lo <= EPT * kWave;
    int32_t e_code[EPT];
#pragma unroll
    for (int q = 0; q < EPT; ++q) {
        const int32_t e = lo + lane + q * kWave;
        e_code[q] = -1;
        if (edges_in_regs && e < hi) {
            int r = 0;
#pragma unroll
            for (int step = 8; step > 0; step >>= 1)
                if (s_rp[r + step] <= e) r += step;
            e_code[q] = (r * kScoreStride) << 16 | edge_to_col[e];
        }
    }

    for (int32_t c0 = 0; c0 < U; c0 += 16) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) acc = mfma16<DT>(a[kk], b[kk], acc);
        // next tile column: its rows go out now, its successor's ids with them
        nid = nid_nxt;
        if (c0 + 16 < U) {
            fetch(nid);
            nid_nxt = c0 + 32 + n < U ? col_to_row[cb + c0 + 32 + n] : -1;
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) s_e[(4 * kg + r) * kScoreStride + n] = acc[r];
        wave_lds_order();
        // StoreSparse
        if (edges_in_regs) {
#pragma unroll
            for (int q = 0; q < EPT; ++q) {
                const int32_t cc = (e_code[q] & 0xFFFF) - c0;
                if (e_code[q] >= 0 && cc >= 0 && cc < 16) out[lo + lane + q * kWave] = s_e[(e_code[q] >> 16) + cc];
            }
        } else {
            for (int32_t e = lo + lane; e < hi; e += kWave) {
                const int32_t cc = edge_to_col[e] - c0;
                if (cc >= 0 && cc < 16) {
                    int r = 0;
#pragma unroll
                    for (int step = 8; step > 0; step >>= 1)
                        if (s_rp[r + step] <= e) r += step;
                    out[e] = s_e[r * kScoreStride + cc];
                }
            }
        }
        wave_lds_order();
    }
}

// ---- fp32 features -----------------------------------------------------------------------------------------
// No MFMA takes fp32 inputs on gfx950, but an fp32 value is exactly the sum of three bf16 values (its upper 16
// bits, the upper 16 bits of the remainder, and of the remainder of that: 3 x 8 significant bits, by
// truncation).  <p, x> over a K step is then computed as six bf16 MFMAs with fp32 accumulation,
//     ph xh + ph xm + pm xh + ph xl + pm xm + pl xh,
// the three dropped products being below 2^-23 of |p x| -- the size of the rounding of an fp32 product.  The
// window's own rows are split once and kept (A operands), the neighbour rows arrive as fp32 and are split
// per tile column.  MANY = false: windows of class kTileFew, edges in registers, one 16 x 16 score tile in
// LDS at a time.  MANY = true: windows with more edges park the scores of up to 256 condensed columns and
// walk their edges once per such batch.
__device__ __forceinline__ uint32_t upper_halves(float lo, float hi)
{
    return __builtin_amdgcn_perm(__float_as_uint(hi), __float_as_uint(lo), 0x07060302u);
}
__device__ __forceinline__ float below_upper_half(float v)
{
    return v - __uint_as_float(__float_as_uint(v) & 0xFFFF0000u);      // exact
}
// eight consecutive fp32 features -> the three bf16 operands (eight values each)
__device__ __forceinline__ void split8(const f32x4 &u, const f32x4 &v, uint4 &h, uint4 &m, uint4 &l)
{
    h = make_uint4(upper_halves(u[0], u[1]), upper_halves(u[2], u[3]), upper_halves(v[0], v[1]), upper_halves(v[2], v[3]));
    float s[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        s[i] = below_upper_half(u[i]);
        s[4 + i] = below_upper_half(v[i]);
    }
    m = make_uint4(upper_halves(s[0], s[1]), upper_halves(s[2], s[3]), upper_halves(s[4], s[5]), upper_halves(s[6], s[7]));
#pragma unroll
    for (int i = 0; i < 8; ++i) s[i] = below_upper_half(s[i]);
    l = make_uint4(upper_halves(s[0], s[1]), upper_halves(s[2], s[3]), upper_halves(s[4], s[5]), upper_halves(s[6], s[7]));
}

constexpr int kScoreStrideF = 17;          // floats per row of a 16-column score tile

template <int KSTEPS, bool MANY>
__global__ __launch_bounds__(kWave) __attribute__((amdgpu_waves_per_eu(KSTEPS >= 8 || MANY ? 2 : 4))) void sddmm_tile_f32_kernel(
    int32_t n_rows, int64_t n_win, const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ edge_to_col,
    const int32_t *__restrict__ win_unique_ptr, const int32_t *__restrict__ col_to_row,
    const uint8_t *__restrict__ win_path, const float *__restrict__ P, int64_t ldp, const float *__restrict__ X,
    int64_t ldx, int32_t D, float *__restrict__ out)
{
    constexpr int EPT = kTileFewEdges / kWave;
    constexpr int kBatch = MANY ? kCols : 16;                  // condensed columns parked in LDS
    constexpr int kStride = MANY ? kEStride : kScoreStrideF;
    __shared__ float s_e[16 * kStride];
    __shared__ int32_t s_rp[17];
    const int64_t per_die = (n_win + kXcds - 1) / kXcds;
    const int64_t win = (int64_t)(blockIdx.x % kXcds) * per_die + blockIdx.x / kXcds;
    if (blockIdx.x / kXcds >= per_die || win >= n_win || win_path[win] != (MANY ? kTileMany : kTileFew)) return;

    const int lane = threadIdx.x;
    const int n = lane & 15;                    // tile row (A) / tile column (B) of this lane
    const int kg = lane >> 4;                   // which 8 features of every K step of 32
    const int64_t r0 = win * 16;
    if (lane < 17) {
        int64_t r = r0 + lane;
        s_rp[lane] = row_ptr[r < n_rows ? r : n_rows];
    }
    const int32_t u0 = win_unique_ptr[win];
    const int32_t cb = row_ptr[r0];             // the window's list sits at its edge offset
    const int32_t U = win_unique_ptr[win + 1] - u0;
    int32_t nid = n < U ? col_to_row[cb + n] : -1;              // neighbour of tile column 0
    int32_t nid_nxt = 16 + n < U ? col_to_row[cb + 16 + n] : -1;

    // features kk * 32 + 8 kg .. + 7 of a row, as two 16-byte pieces (D is a multiple of 4)
    auto load8 = [&](const float *row, int kk, f32x4 &u, f32x4 &v) {
        const int32_t f = kk * 32 + kg * 8;
        u = f32x4{0.f, 0.f, 0.f, 0.f};
        v = f32x4{0.f, 0.f, 0.f, 0.f};
        if (row != nullptr && f < D) u = *reinterpret_cast<const f32x4 *>(row + f);
        if (row != nullptr && f + 4 < D) v = *reinterpret_cast<const f32x4 *>(row + f + 4);
    };
    f32x4 b[KSTEPS][2];
    auto fetch = [&](int32_t node) {
        const float *row = node >= 0 ? X + (int64_t)node * ldx : nullptr;
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) load8(row, kk, b[kk][0], b[kk][1]);
    };
    fetch(nid);

    uint4 ah[KSTEPS], am[KSTEPS], al[KSTEPS];
    {
        const float *row = r0 + n < n_rows ? P + (r0 + n) * ldp : nullptr;
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
            f32x4 u, v;
            load8(row, kk, u, v);
            split8(u, v, ah[kk], am[kk], al[kk]);
        }
    }

    wave_lds_order();
    const int32_t lo = s_rp[0], hi = s_rp[16];
    // class kTileFew: (score-tile row offset << 16 | condensed column) of the lane's edges; windows with more
    // edges that only a forced policy puts into this class re-read theirs for every tile column
    const bool edges_in_regs = !MANY && hi - lo <= EPT * kWave;
    int32_t e_code[MANY ? 1 : EPT];
    if constexpr (!MANY) {
#pragma unroll
        for (int q = 0; q < EPT; ++q) {
            const int32_t e = lo + lane + q * kWave;
            e_code[q] = -1;
            if (edges_in_regs && e < hi) {
                int r = 0;
#pragma unroll
                for (int step = 8; step > 0; step >>= 1)
                    if (s_rp[r + step] <= e) r += step;
                e_code[q] = (r * kStride) << 16 | edge_to_col[e];
            }
        }
    }
    // StoreSparse for the condensed columns [b0, b0 + width) parked in s_e, edges read from global memory
    auto store_from_global = [&](int32_t b0, int32_t width) {
        for (int32_t e = lo + lane; e < hi; e += kWave) {
            const int32_t cc = edge_to_col[e] - b0;
            if (cc >= 0 && cc < width) {
                int r = 0;
#pragma unroll
                for (int step = 8; step > 0; step >>= 1)
                    if (s_rp[r + step] <= e) r += step;
                out[e] = s_e[r * kStride + cc];
            }
        }
    };

    for (int32_t c0 = 0; c0 < U; c0 += 16) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
            uint4 bh, bm, bl;
            split8(b[kk][0], b[kk][1], bh, bm, bl);
            acc = mfma16<TCG_BF16>(ah[kk], bl, acc);            // smallest terms first
            acc = mfma16<TCG_BF16>(al[kk], bh, acc);
            acc = mfma16<TCG_BF16>(am[kk], bm, acc);
            acc = mfma16<TCG_BF16>(am[kk], bh, acc);
            acc = mfma16<TCG_BF16>(ah[kk], bm, acc);
            acc = mfma16<TCG_BF16>(ah[kk], bh, acc);
        }
        // next tile column: its rows go out now, its successor's ids with them
        nid = nid_nxt;
        if (c0 + 16 < U) {
            fetch(nid);
            nid_nxt = c0 + 32 + n < U ? col_to_row[cb + c0 + 32 + n] : -1;
        }
        const int32_t cb = MANY ? c0 % kBatch : 0;              // where this tile column sits in the parked batch
#pragma unroll
        for (int r = 0; r < 4; ++r) s_e[(4 * kg + r) * kStride + cb + n] = acc[r];
        wave_lds_order();
        if constexpr (!MANY) {
            if (edges_in_regs) {
#pragma unroll
                for (int q = 0; q < EPT; ++q) {
                    const int32_t cc = (e_code[q] & 0xFFFF) - c0;
                    if (e_code[q] >= 0 && cc >= 0 && cc < 16) out[lo + lane + q * kWave] = s_e[(e_code[q] >> 16) + cc];
                }
            } else {
                store_from_global(c0, 16);
            }
            wave_lds_order();
        } else if (cb + 16 == kBatch || c0 + 16 >= U) {
            store_from_global(c0 - cb, kBatch);
            wave_lds_order();
        }
    }
}

template <int KSTEPS>
void launch_f32(const tcg_meta *m, const float *P, int64_t ldp, const float *X, int64_t ldx, int32_t D, float *out,
                hipStream_t s)
{
    const dim3 grid((unsigned)(kXcds * ceil_div(m->n_win, kXcds)));
    if (m->n_tile_win > m->n_tile_many)
        hipLaunchKernelGGL((sddmm_tile_f32_kernel<KSTEPS, false>), grid, dim3(kWave), 0, s, m->n_rows, m->n_win,
                           m->d_row_ptr, m->d_edge_to_col, m->d_win_unique_ptr, m->d_col_to_row, m->d_win_path, P, ldp,
                           X, ldx, D, out);
    if (m->n_tile_many > 0)
        hipLaunchKernelGGL((sddmm_tile_f32_kernel<KSTEPS, true>), grid, dim3(kWave), 0, s, m->n_rows, m->n_win,
                           m->d_row_ptr, m->d_edge_to_col, m->d_win_unique_ptr, m->d_col_to_row, m->d_win_path, P, ldp,
                           X, ldx, D, out);
}

template <int DT, int KSTEPS>
void launch(const tcg_meta *m, const void *P, int64_t ldp, const void *X, int64_t ldx, int32_t D, float *out,
            hipStream_t s)
{
    const dim3 grid((unsigned)(kXcds * ceil_div(m->n_win, kXcds)));
    const bool few = m->n_tile_win > m->n_tile_many;
    if (few)
        hipLaunchKernelGGL((sddmm_tile_wave_kernel<DT, KSTEPS>), grid, dim3(kWave), 0, s, m->n_rows, m->n_win,
                           m->d_row_ptr, m->d_edge_to_col, m->d_win_unique_ptr, m->d_col_to_row, m->d_win_path,
                           static_cast<const char *>(P), ldp * 2, static_cast<const char *>(X), ldx * 2, D, out);
    if (m->n_tile_many > 0)
        hipLaunchKernelGGL((sddmm_tile_kernel<DT, KSTEPS>), grid, dim3(kTileBlock), 0, s, m->n_rows, m->n_win,
                           m->d_row_ptr, m->d_edge_to_col, m->d_win_unique_ptr, m->d_col_to_row, m->d_win_path,
                           static_cast<const char *>(P), ldp * 2, static_cast<const char *>(X), ldx * 2, D, out, true);
}

template <int DT>
void launch_k(const tcg_meta *m, const void *P, int64_t ldp, const void *X, int64_t ldx, int32_t D, float *out,
              hipStream_t s)
{
    const int ks = (D + 31) / 32;
    if (ks <= 1) launch<DT, 1>(m, P, ldp, X, ldx, D, out, s);
    else if (ks <= 2) launch<DT, 2>(m, P, ldp, X, ldx, D, out, s);
    else if (ks <= 4) launch<DT, 4>(m, P, ldp, X, ldx, D, out, s);
    else if (ks <= 8) launch<DT, 8>(m, P, ldp, X, ldx, D, out, s);
    else launch<DT, 16>(m, P, ldp, X, ldx, D, out, s);
}

}  // namespace

bool sddmm_tile_supports(tcg_dtype x_dt, int32_t D, int64_t ld, const void *ptr)
{
    if (x_dt == TCG_F32)       // the kernel that splits fp32 operands into bf16 triples
        return D % 4 == 0 && D <= 256 && ld % 4 == 0 && (reinterpret_cast<uintptr_t>(ptr) & 15) == 0;
    return tile_path_supports(x_dt, D, ld, ptr);
}

int sddmm_tile_launch(tcg_meta *m, const void *d_P, int64_t ldp, const void *d_X, int64_t ldx, tcg_dtype x_dt,
                      int32_t D, float *d_out, hipStream_t s)
{
    if (x_dt == TCG_F32) {
        const float *P = static_cast<const float *>(d_P), *X = static_cast<const float *>(d_X);
        if (D <= 64) launch_f32<2>(m, P, ldp, X, ldx, D, d_out, s);
        else if (D <= 128) launch_f32<4>(m, P, ldp, X, ldx, D, d_out, s);
        else launch_f32<8>(m, P, ldp, X, ldx, D, d_out, s);
    } else if (x_dt == TCG_BF16) launch_k<TCG_BF16>(m, d_P, ldp, d_X, ldx, D, d_out, s);
    else launch_k<TCG_F16>(m, d_P, ldp, d_X, ldx, D, d_out, s);
    return launch_status("sddmm_tile kernels");
}

}  // namespace tcg
