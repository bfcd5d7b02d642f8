// Neighbour aggregation on condensed tiles (Algorithm 2 of the paper) with gfx950 MFMA.
//
// One wavefront per row window of 16 rows that the plan assigned to this path, i.e. windows whose
// rows share enough neighbours that every gathered X row is reused several times.  The window's
// condensed columns (its sorted unique neighbour list from SGT) are walked in chunks of KW = 16:
//   InitSparse  the 16 x KW slice of the condensed adjacency is built in LDS in fp32 from the
//               window's edges and edge_to_col (repeated entries add up), then rounded to the
//               feature type when it is loaded as the MFMA A operand;
//   FetchDense  the KW neighbour rows named by col_to_row are fetched with coalesced loads -- each
//               unique neighbour once per window, which is the traffic reduction SGT exists for;
//   TCcompute   v_mfma_f32_16x16x16 (bf16 or f16 inputs, fp32 accumulate), all sharing the A operand;
//   StoreDense  after the last chunk the accumulators are written to the window's rows of Y in
//               16-byte pieces, as streaming stores.
// Two kernels implement this.  spmm_tile_direct_kernel (rows of more than 64 features) loads the
// neighbour rows straight into the B operand registers and stores straight from the accumulators;
// spmm_tile_wave_kernel (narrow rows, 32-row windows) stages the rows and the finished tile in LDS.
// Differences from the paper's kernel: the K extent of a tile is 16 (bf16/f16 MFMA) instead of 8
// (TF-32 WMMA); the column -> node map comes straight from SGT's col_to_row instead of being
// rebuilt per block; no transposition through shared memory is needed for the B operand (a permuted
// assignment of features to MFMA columns in the direct kernel, the transposing LDS read
// ds_read_b64_tr_b16 in the other); and a window belongs to one wavefront instead of a block of
// warps that split the feature dimension.  A wavefront's LDS operations complete in program
// order, so the kernels have no barrier at all, and a compute unit keeps twelve to sixteen windows
// in flight, which is what hides the chain of dependent loads of a window (row pointers -> edge
// list and neighbour ids -> neighbour rows).  The neighbour rows of chunk c + 1 are requested as
// soon as chunk c has been consumed, their ids one chunk earlier still.  The counters show the path
// bound by the memory side (row fetches through L2, result stores), not by the matrix cores.
#include "common.h"
#include "devutil.h"

namespace tcg {

namespace {

typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 h16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;

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

constexpr int KW = 16;
constexpr int kAStrideW = 20;     // floats; 16 x 20 = 5 x 64: five stores per lane clear the slice

// Orders the LDS accesses of the wavefront's lanes for the compiler; the hardware already completes a
// wavefront's LDS operations in program order, so no instruction is emitted.
__device__ __forceinline__ void wave_lds_order()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int DT>
__device__ __forceinline__ f32x4 mfma16k16(const uint2 &a, const uint2 &b, f32x4 c)
{
    if constexpr (DT == TCG_BF16) {
        s16x4 va, vb;
        __builtin_memcpy(&va, &a, 8);
        __builtin_memcpy(&vb, &b, 8);
        return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(va, vb, c, 0, 0, 0);
    } else {
        h16x4 va, vb;
        __builtin_memcpy(&va, &a, 8);
        __builtin_memcpy(&vb, &b, 8);
        return __builtin_amdgcn_mfma_f32_16x16x16f16(va, vb, c, 0, 0, 0);
    }
}

// NS: 16-column slices of D per wavefront; a window with D > 16 * NS is shared by n_dparts wavefronts.
// FULL_A = false serves the windows of class kTileFew (at most kTileFewEdges edges, kept in registers;
// the 16 x KW slice of the condensed adjacency is rebuilt for every chunk).  FULL_A = true serves class
// kTileMany: the whole 16 x U_w condensed adjacency of the window is built once in (dynamic) LDS with a
// single pass over the window's edges -- dense windows would otherwise walk thousands of edges per chunk --
// and every chunk reads its slice from there; a_stride = its row stride in floats.
// HB: 16-row blocks per window (1: windows of 16 rows, 2: windows of 32 rows, class kTileFew only).  A taller
// window fetches a neighbour shared by its rows once instead of once per 16 rows, and every B fragment read
// from LDS feeds HB MFMAs.
template <int DT, bool HAS_W, int NS, bool FULL_A, int HB>
__global__ __launch_bounds__(kWave) __attribute__((amdgpu_waves_per_eu(3))) void spmm_tile_wave_kernel(
    int32_t n_rows, int64_t n_win, const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ edge_to_col,
    const int32_t *__restrict__ win_unique_ptr, const int32_t *__restrict__ col_to_row,
    const uint8_t *__restrict__ win_path, const float *__restrict__ w, const char *__restrict__ X,
    int64_t ldx_bytes, int32_t D, int32_t n_dparts, void *__restrict__ Y, int y_dt, int64_t ldy, bool y_vec,
    int32_t a_stride, bool skip_small)
{
    static_assert(!(FULL_A && HB != 1), "the whole-window adjacency variant handles 16-row windows");
    constexpr int H = 16 * HB;
    extern __shared__ __align__(16) float a_full[];              // FULL_A: 16 x a_stride
    constexpr int PP = NS / 2;                                    // 16-byte pieces of a chunk per lane
    // Staged row stride: an odd multiple of 32 bytes, so the 8 rows that half a wavefront touches in
    // a transposing read start in 8 different groups of 8 LDS banks.
    constexpr int32_t rs = NS * 32 + 32;
    __shared__ __align__(16) char xs[KW * rs];
    __shared__ __align__(16) float a_slice[FULL_A ? 4 : H * kAStrideW];
    __shared__ int32_t s_rp[H + 1];
    float *a32 = FULL_A ? a_full : a_slice;
    const int32_t as = FULL_A ? a_stride : kAStrideW;

    // Workgroup i runs on die i % kXcds: every die gets a contiguous range of windows.
    const int64_t per_die = (n_win + kXcds - 1) / kXcds;
    const int64_t j = blockIdx.x / kXcds;
    const int64_t win = (int64_t)(blockIdx.x % kXcds) * per_die + j / n_dparts;
    if (j / n_dparts >= per_die || win >= n_win || win_path[win] != (FULL_A ? kTileMany : kTileFew)) return;
    const int32_t d0 = (int32_t)(j % n_dparts) * (NS * 16);       // first feature column of this part
    const int32_t Dp = min(NS * 16, D - d0);

    const int lane = threadIdx.x;
    const int64_t r0 = win * H;
    if (lane < H + 1) {
        int64_t r = r0 + lane;
        s_rp[lane] = row_ptr[r < n_rows ? r : n_rows];
    }
    wave_lds_order();
    const int32_t u0 = win_unique_ptr[win];
    const int32_t cb = row_ptr[r0];             // the window's list sits at its edge offset
    const int32_t U = win_unique_ptr[win + 1] - u0;
    // ids of the neighbours of chunks 0 and 1 (lane k < 16 holds row k of the chunk)
    const int kk = lane & 15;
    int32_t nid_cur = kk < U ? col_to_row[cb + kk] : -1;
    int32_t nid_nxt = KW + kk < U ? col_to_row[cb + KW + kk] : -1;
    const int32_t lo = s_rp[0], hi = s_rp[H];
    if (skip_small && hi - lo <= kTileFewEdges) return;        // taken by the direct kernel
    const int32_t n_slices = (Dp + 15) / 16;

    // FetchDense mapping: 2 * NS lanes cover one row part with 16-byte pieces, so one pass of the
    // wavefront loads RPP rows and PP passes load the chunk; piece i of a lane is row i * RPP + sub.
    constexpr int LPR = 2 * NS, RPP = kWave / LPR;
    const int sub = lane / LPR;
    const int32_t goff = (lane % LPR) * 16;
    const bool piece_ok = goff < Dp * 2;
    const char *Xp = X + (int64_t)d0 * 2 + goff;
    char *xs_dst = xs + sub * rs + goff;
    uint4 pre[PP];
    auto fetch = [&](int32_t nid) {
#pragma unroll
        for (int i = 0; i < PP; ++i) {
            const int32_t node = __shfl(nid, i * RPP + sub);
            pre[i] = make_uint4(0, 0, 0, 0);
            if (piece_ok && node >= 0) pre[i] = *reinterpret_cast<const uint4 *>(Xp + (int64_t)node * ldx_bytes);
        }
    };
    fetch(nid_cur);

    // !FULL_A: a window of at most EPT * 64 edges keeps them in registers: (A-slice row offset << 16 |
    // condensed column) and the value.  (Windows forced onto this path with more edges re-read them for
    // every chunk.)
    constexpr int EPT = FULL_A ? 1 : HB * kTileFewEdges / kWave;
    const bool edges_in_regs = hi - lo <= EPT * kWave;
    int32_t e_code[EPT];
    float e_val[EPT];
    if constexpr (!FULL_A) {
#pragma unroll
        for (int q = 0; q < EPT; ++q) {
            const int32_t e = lo + lane + q * kWave;
            e_code[q] = -1;
            e_val[q] = 0.f;
            if (edges_in_regs && e < hi) {
                int r = 0;
#pragma unroll
                for (int step = H / 2; step > 0; step >>= 1)
                    if (s_rp[r + step] <= e) r += step;
                e_code[q] = (r * kAStrideW) << 16 | edge_to_col[e];     // condensed column < kTileMaxUnique
                if (HAS_W) e_val[q] = w[e];
            }
        }
    } else {
        // InitSparse for the whole window: clear 16 x a_stride floats, then one pass over the edges.
        for (int32_t i = lane * 4; i < 16 * as; i += kWave * 4)
            *reinterpret_cast<float4 *>(a32 + i) = make_float4(0.f, 0.f, 0.f, 0.f);
        wave_lds_order();
        // batches of 8 edges per lane: the loads of a batch are issued together (clamped, always valid)
        for (int32_t e0 = lo; e0 < hi; e0 += 8 * kWave) {
            int32_t cc[8];
            float vv[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int32_t e = min(e0 + lane + q * kWave, hi - 1);
                cc[q] = edge_to_col[e];
                vv[q] = HAS_W ? w[e] : 1.f;
            }
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int32_t e = e0 + lane + q * kWave;
                if (e < hi) {
                    int r = 0;
#pragma unroll
                    for (int step = H / 2; step > 0; step >>= 1)
                        if (s_rp[r + step] <= e) r += step;
                    atomicAdd(&a32[r * as + cc[q]], vv[q]);
                }
            }
        }
        wave_lds_order();
    }

    f32x4 acc[HB][NS];
#pragma unroll
    for (int hb = 0; hb < HB; ++hb)
#pragma unroll
        for (int i = 0; i < NS; ++i) acc[hb][i] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int g = lane >> 4, n_in = lane & 15;
    const float *a_src = a32 + n_in * as + 4 * g;                 // A: row n_in, k = 4g .. 4g+3 (+ k0 if FULL_A)
    // B: lane j of a 16-lane group addresses row 4g + j / 4, 8-byte chunk j % 4 of a slice
    const char *b_src = xs + (4 * g + (n_in >> 2)) * rs + (n_in & 3) * 8;

    for (int32_t k0 = 0; k0 < U; k0 += KW) {
        // chunk k0: registers -> LDS, then request chunk k0 + KW and the ids of chunk k0 + 2 KW
#pragma unroll
        for (int i = 0; i < PP; ++i)
            if (piece_ok) *reinterpret_cast<uint4 *>(xs_dst + i * RPP * rs) = pre[i];
        nid_cur = nid_nxt;
        if (k0 + KW < U) {
            fetch(nid_cur);
            nid_nxt = k0 + 2 * KW + kk < U ? col_to_row[cb + k0 + 2 * KW + kk] : -1;
        }
        if constexpr (!FULL_A) {
            // InitSparse
#pragma unroll
            for (int i = 0; i < 5 * HB; ++i) a32[lane + i * kWave] = 0.f;
            wave_lds_order();
            if (edges_in_regs) {
#pragma unroll
                for (int q = 0; q < EPT; ++q) {
                    const int32_t cc = (e_code[q] & 0xFFFF) - k0;
                    if (e_code[q] >= 0 && cc >= 0 && cc < KW) atomicAdd(&a32[(e_code[q] >> 16) + cc], HAS_W ? e_val[q] : 1.f);
                }
            } else {
                for (int32_t e = lo + lane; e < hi; e += kWave) {
                    int32_t cc = edge_to_col[e] - k0;
                    if (cc >= 0 && cc < KW) {
                        int r = 0;
#pragma unroll
                        for (int step = H / 2; step > 0; step >>= 1)
                            if (s_rp[r + step] <= e) r += step;
                        atomicAdd(&a32[r * kAStrideW + cc], HAS_W ? w[e] : 1.f);
                    }
                }
            }
            wave_lds_order();
        }
        // TCcompute
        uint2 af[HB];
#pragma unroll
        for (int hb = 0; hb < HB; ++hb) {
            const float4 av = *reinterpret_cast<const float4 *>(a_src + hb * 16 * as + (FULL_A ? k0 : 0));
            af[hb].x = pack2<DT, !HAS_W>(av.x, av.y);
            af[hb].y = pack2<DT, !HAS_W>(av.z, av.w);
        }
#pragma unroll
        for (int i = 0; i < NS; ++i)
            if (i < n_slices) {   // columns of a half slice beyond D read padding and are never stored
                const uint2 bf = lds_read_tr16(b_src + i * 32);
#pragma unroll
                for (int hb = 0; hb < HB; ++hb) acc[hb][i] = mfma16k16<DT>(af[hb], bf, acc[hb][i]);
            }
        wave_lds_order();
    }

    // StoreDense.  A lane holds rows 4g .. 4g+3 of one column per slice; the tile goes through LDS (the
    // staging area is free now), half of the slices at a time, and leaves as whole 16-byte pieces of
    // consecutive lanes: every store instruction writes RPP complete row parts.
    constexpr int SP = NS / 2, YS = 8 * NS + 4;                   // slices per pass; LDS row stride in floats
    float *ys = reinterpret_cast<float *>(xs);
#pragma unroll
    for (int hh = 0; hh < 2 * HB; ++hh) {
        const int hb = hh / 2, h = hh % 2;
        if (h * SP >= n_slices) continue;
#pragma unroll
        for (int i = 0; i < SP; ++i)
#pragma unroll
            for (int r = 0; r < 4; ++r) ys[(4 * g + r) * YS + i * 16 + n_in] = acc[hb][h * SP + i][r];
        wave_lds_order();
        const int32_t col = h * SP * 16 + (lane % LPR) * 4;       // first of the lane's 4 columns inside the part
#pragma unroll
        for (int i = 0; i < PP; ++i) {
            const int64_t row = r0 + hb * 16 + i * RPP + sub;
            if (row >= n_rows || col >= Dp) continue;
            const float4 v = *reinterpret_cast<const float4 *>(ys + (i * RPP + sub) * YS + (lane % LPR) * 4);
            const int64_t o = row * ldy + d0 + col;
            if (y_dt == TCG_F32) {
                float *y = static_cast<float *>(Y) + o;
                if (y_vec) stream_store(y, v.x, v.y, v.z, v.w);
                else { y[0] = v.x; y[1] = v.y; y[2] = v.z; y[3] = v.w; }
            } else {
                uint16_t *y = static_cast<uint16_t *>(Y) + o;
                uint2 pk;
                if (y_dt == TCG_BF16) {
                    pk.x = (uint32_t)f32_to_bf16_bits(v.x) | ((uint32_t)f32_to_bf16_bits(v.y) << 16);
                    pk.y = (uint32_t)f32_to_bf16_bits(v.z) | ((uint32_t)f32_to_bf16_bits(v.w) << 16);
                } else {
                    pk.x = (uint32_t)__half_as_ushort(__float2half_rn(v.x)) | ((uint32_t)__half_as_ushort(__float2half_rn(v.y)) << 16);
                    pk.y = (uint32_t)__half_as_ushort(__float2half_rn(v.z)) | ((uint32_t)__half_as_ushort(__float2half_rn(v.w)) << 16);
                }
                if (y_vec) stream_store(y, pk.x, pk.y);
                else { y[0] = (uint16_t)pk.x; y[1] = (uint16_t)(pk.x >> 16); y[2] = (uint16_t)pk.y; y[3] = (uint16_t)(pk.y >> 16); }
            }
        }
        wave_lds_order();
    }
}

// ---- neighbour rows straight into the MFMA operand registers (16-row windows, both tile classes) ---------
// The B operand of v_mfma_f32_16x16x16 wants, per lane (n = lane % 16, q = lane / 16), the four values
// B[4q .. 4q+3][n]: four NEIGHBOURS, one feature.  Memory has the features of a neighbour contiguous, which
// is why the kernel above stages the rows in LDS and reads them back transposed.  But nothing says that
// column n of the tile must be feature n: here lane (n, q) loads 8 bytes = the 4 features 4n .. 4n+3 of
// each of its four neighbour rows 4q .. 4q+3 (16 lanes cover 128 contiguous bytes of a row) and issues four
// MFMAs, the m-th of which takes element m of the four loaded pieces (two byte-permute instructions
// assemble the operand).  MFMA m then computes, in its column n, feature 4n + m: across the four
// accumulators a lane ends up with 4 CONSECUTIVE features of its four output rows, one 16-byte store per
// row with 16 lanes writing 256 contiguous bytes -- no LDS staging on the way in, none on the way out,
// no barrier.  A second set of pieces, 64 features further on, fills a block of 128 features.  LDS
// only holds the A operand and the row pointers: for a window of class kTileFew the window's edges (as row /
// condensed-column codes) and the 16 x 16 slice of the condensed adjacency rebuilt from them per chunk,
// for class kTileMany (FULL_A) the whole 16 x U_w adjacency, built once.
// NFB: blocks of 128 features per wavefront (a wider D is split over n_dparts wavefronts).
template <int DT, bool HAS_W, int NFB, bool FULL_A>
__global__ __launch_bounds__(kWave) __attribute__((amdgpu_waves_per_eu(4))) void spmm_tile_direct_kernel(
    int32_t n_rows, int64_t n_win, const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ edge_to_col,
    const int32_t *__restrict__ win_unique_ptr, const int32_t *__restrict__ col_to_row,
    const uint8_t *__restrict__ win_path, const float *__restrict__ w, const char *__restrict__ X,
    int64_t ldx_bytes, int32_t D, int32_t n_dparts, void *__restrict__ Y, int y_dt, int64_t ldy, bool y_vec,
    int32_t a_stride)
{
    constexpr int EPT = kTileFewEdges / kWave;
    extern __shared__ __align__(16) float a_full[];                    // FULL_A: 16 x a_stride
    __shared__ __align__(16) float a_slice[FULL_A ? 4 : 16 * kAStrideW];
    __shared__ int32_t s_rp[17];
    __shared__ int32_t s_code[FULL_A ? 1 : kTileFewEdges];             // per edge: slice row offset << 16 | condensed column
    __shared__ float s_val[HAS_W && !FULL_A ? kTileFewEdges : 1];      // per edge: its value
    float *a32 = FULL_A ? a_full : a_slice;
    const int32_t as = FULL_A ? a_stride : kAStrideW;

    const int64_t per_die = (n_win + kXcds - 1) / kXcds;
    const int64_t j = blockIdx.x / kXcds;
    const int64_t win = (int64_t)(blockIdx.x % kXcds) * per_die + j / n_dparts;
    if (j / n_dparts >= per_die || win >= n_win || win_path[win] != (FULL_A ? kTileMany : kTileFew)) return;
    const int32_t d0 = (int32_t)(j % n_dparts) * (NFB * 128);     // first feature column of this part
    const int32_t Dp = min(NFB * 128, D - d0);

    const int lane = threadIdx.x;
    const int n = lane & 15, q = lane >> 4;
    const int64_t r0 = win * 16;
    if (lane < 17) {
        int64_t r = r0 + lane;
        s_rp[lane] = row_ptr[r < n_rows ? r : n_rows];
    }
    wave_lds_order();
    const int32_t u0 = win_unique_ptr[win];
    const int32_t cb = row_ptr[r0];             // the window's list sits at its edge offset
    const int32_t U = win_unique_ptr[win + 1] - u0;
    // ids of the neighbours of chunks 0 and 1 (lane k < 16 holds row k of the chunk)
    int32_t nid_cur = n < U ? col_to_row[cb + n] : -1;
    int32_t nid_nxt = KW + n < U ? col_to_row[cb + KW + n] : -1;
    const int32_t lo = s_rp[0], hi = s_rp[16];
    if (!FULL_A && hi - lo > kTileFewEdges) return;    // only a forced policy puts such a window into this class

    // FetchDense: chunk rows 4q .. 4q+3; of every block of 128 features the two 8-byte pieces
    // 4n .. 4n+3 and 64 + 4n .. 64 + 4n+3 (16 lanes cover 128 contiguous bytes of a row per load)
    const char *Xp = X + (int64_t)d0 * 2 + n * 8;
    uint2 xr[NFB][2][4];
    auto fetch = [&](int32_t nid) {
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const int32_t node = __shfl(nid, 4 * q + jj);
#pragma unroll
            for (int fb = 0; fb < NFB; ++fb)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    xr[fb][h][jj] = make_uint2(0, 0);
                    if (node >= 0 && fb * 128 + h * 64 + 4 * n < Dp)
                        xr[fb][h][jj] =
                            *reinterpret_cast<const uint2 *>(Xp + (int64_t)node * ldx_bytes + fb * 256 + h * 128);
                }
        }
    };
    fetch(nid_cur);

    if constexpr (!FULL_A) {
        // the window's edges go to LDS (registers are the scarce resource here: they bound the wavefronts,
        // and so the bytes in flight, per CU); each lane writes and later reads only its own slots
#pragma unroll
        for (int e_i = 0; e_i < EPT; ++e_i) {
            const int32_t e = lo + lane + e_i * kWave;
            int32_t code = -1;
            if (e < hi) {
                int r = 0;
#pragma unroll
                for (int step = 8; step > 0; step >>= 1)
                    if (s_rp[r + step] <= e) r += step;
                code = (r * kAStrideW) << 16 | edge_to_col[e];     // condensed column < kTileFewEdges
                if (HAS_W) s_val[lane + e_i * kWave] = w[e];
            }
            s_code[lane + e_i * kWave] = code;
        }
    } else {
        // InitSparse for the whole window: clear 16 x a_stride floats, then one pass over the edges in
        // batches of 8 per lane whose loads are issued together (clamped, always valid)
        for (int32_t i = lane * 4; i < 16 * as; i += kWave * 4)
            *reinterpret_cast<float4 *>(a32 + i) = make_float4(0.f, 0.f, 0.f, 0.f);
        wave_lds_order();
        for (int32_t e0 = lo; e0 < hi; e0 += 8 * kWave) {
            int32_t cc[8];
            float vv[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int32_t e = min(e0 + lane + i * kWave, hi - 1);
                cc[i] = edge_to_col[e];
                vv[i] = HAS_W ? w[e] : 1.f;
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int32_t e = e0 + lane + i * kWave;
                if (e < hi) {
                    int r = 0;
#pragma unroll
                    for (int step = 8; step > 0; step >>= 1)
                        if (s_rp[r + step] <= e) r += step;
                    atomicAdd(&a32[r * as + cc[i]], vv[i]);
                }
            }
        }
        wave_lds_order();
    }

    f32x4 acc[NFB][8];
#pragma unroll
    for (int fb = 0; fb < NFB; ++fb)
#pragma unroll
        for (int m = 0; m < 8; ++m) acc[fb][m] = f32x4{0.f, 0.f, 0.f, 0.f};
    const float *a_src = a32 + n * as + 4 * q;                    // A: row n, k = 4q .. 4q+3

    for (int32_t k0 = 0; k0 < U; k0 += KW) {
        if constexpr (!FULL_A) {
            // InitSparse (the rows of this chunk are still on their way)
#pragma unroll
            for (int i = 0; i < 5; ++i) a32[lane + i * kWave] = 0.f;
            wave_lds_order();
#pragma unroll
            for (int e_i = 0; e_i < EPT; ++e_i) {
                const int32_t code = s_code[lane + e_i * kWave];
                const int32_t cc = (code & 0xFFFF) - k0;
                if (code >= 0 && cc >= 0 && cc < KW)
                    atomicAdd(&a32[(code >> 16) + cc], HAS_W ? s_val[lane + e_i * kWave] : 1.f);
            }
            wave_lds_order();
        }
        const float4 av = *reinterpret_cast<const float4 *>(a_src + (FULL_A ? k0 : 0));
        uint2 af;
        af.x = pack2<DT, !HAS_W>(av.x, av.y);
        af.y = pack2<DT, !HAS_W>(av.z, av.w);
        wave_lds_order();
        // TCcompute: element m of the four pieces -> B operand of MFMA (h, m)
#pragma unroll
        for (int fb = 0; fb < NFB; ++fb)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const uint32_t wd[4][2] = {{xr[fb][h][0].x, xr[fb][h][0].y},
                                           {xr[fb][h][1].x, xr[fb][h][1].y},
                                           {xr[fb][h][2].x, xr[fb][h][2].y},
                                           {xr[fb][h][3].x, xr[fb][h][3].y}};
#pragma unroll
                for (int m = 0; m < 4; ++m) {
                    const uint32_t sel = (m & 1) ? 0x07060302u : 0x05040100u;   // high / low halves of two words
                    uint2 bf;
                    bf.x = __builtin_amdgcn_perm(wd[1][m >> 1], wd[0][m >> 1], sel);
                    bf.y = __builtin_amdgcn_perm(wd[3][m >> 1], wd[2][m >> 1], sel);
                    acc[fb][h * 4 + m] = mfma16k16<DT>(af, bf, acc[fb][h * 4 + m]);
                }
            }
        // next chunk's rows into the registers just consumed; the ids of the one after
        nid_cur = nid_nxt;
        if (k0 + KW < U) {
            fetch(nid_cur);
            nid_nxt = k0 + 2 * KW + n < U ? col_to_row[cb + k0 + 2 * KW + n] : -1;
        }
    }

    // StoreDense: acc[fb][4h + m][r] = Y[r0 + 4q + r][d0 + 128 fb + 64 h + 4n + m]: 16 lanes write 256
    // contiguous bytes of a row per store
#pragma unroll
    for (int fb = 0; fb < NFB; ++fb)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int32_t col = fb * 128 + h * 64 + 4 * n;
            if (col >= Dp) continue;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int64_t row = r0 + 4 * q + r;
                if (row < n_rows)
                    store4(Y, y_dt, row * ldy + d0 + col,
                           make_float4(acc[fb][4 * h][r], acc[fb][4 * h + 1][r], acc[fb][4 * h + 2][r],
                                       acc[fb][4 * h + 3][r]), y_vec);
            }
        }
}

// ---- fp32 features ---------------------------------------------------------------------------------------
// gfx950 has no MFMA that takes fp32 inputs, and on the vector ALUs the dense 16 x U_w x D product of a window
// (mostly zeros of the condensed adjacency) costs more than the memory traffic it saves.  An fp32 value is,
// however, EXACTLY the sum of three bf16 values: its upper 16 bits, the upper 16 bits of what is left, and the
// upper 16 bits of what is left after that (8 significant bits each, 24 in all; truncation, so nothing rounds
// and nothing overflows).  So the kernel is the direct kernel above with every fp32 operand split in three:
//     w x  =  (wh + wm + wl)(xh + xm + xl)  ~  wh xh + wh xm + wm xh + wh xl + wm xm + wl xh,
// six bf16 MFMAs with fp32 accumulation; the three dropped terms are below 2^-23 |w x|, the size of the
// rounding of the fp32 result itself.  With unit edge values the adjacency entries are small integers (the
// multiplicity of an edge; exact in bf16 up to 256) and three MFMAs suffice.  Lane (n, q) loads the 16-byte
// piece "features 4n .. 4n+3" of a block of 64 features from its four neighbour rows; MFMA m of the block takes
// element m, so its column n is feature 4n + m and a lane ends up with four consecutive features of its four
// output rows: one 16-byte streaming store per row.  NB blocks of 64 features per wavefront.
// (A non-finite feature becomes NaN in every row of its window that has an edge to it or not -- inf - inf in
// the split, NaN x 0 in the MFMA -- where the gather path propagates it only along edges.)
__device__ __forceinline__ uint32_t upper_halves(float lo, float hi)
{
    return __builtin_amdgcn_perm(__float_as_uint(hi), __float_as_uint(lo), 0x07060302u);
}
__device__ __forceinline__ float below_upper_half(float v)
{
    return v - __uint_as_float(__float_as_uint(v) & 0xFFFF0000u);      // exact
}

template <bool HAS_W, int NB, bool FULL_A>
__global__ __launch_bounds__(kWave) __attribute__((amdgpu_waves_per_eu(NB >= 4 ? 2 : 4))) void spmm_tile_f32_kernel(
    int32_t n_rows, int64_t n_win, const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ edge_to_col,
    const int32_t *__restrict__ win_unique_ptr, const int32_t *__restrict__ col_to_row,
    const uint8_t *__restrict__ win_path, const float *__restrict__ w, const float *__restrict__ X, int64_t ldx,
    int32_t D, int32_t n_dparts, void *__restrict__ Y, int y_dt, int64_t ldy, bool y_vec, int32_t a_stride)
{
    constexpr int EPT = kTileFewEdges / kWave;
    extern __shared__ __align__(16) float a_full[];                    // FULL_A: 16 x a_stride
    __shared__ __align__(16) float a_slice[FULL_A ? 4 : 16 * kAStrideW];
    __shared__ int32_t s_rp[17];
    __shared__ int32_t s_code[FULL_A ? 1 : kTileFewEdges];             // per edge: slice row offset << 16 | condensed column
    __shared__ float s_val[HAS_W && !FULL_A ? kTileFewEdges : 1];      // per edge: its value
    float *a32 = FULL_A ? a_full : a_slice;
    const int32_t as = FULL_A ? a_stride : kAStrideW;

    const int64_t per_die = (n_win + kXcds - 1) / kXcds;
    const int64_t j = blockIdx.x / kXcds;
    const int64_t win = (int64_t)(blockIdx.x % kXcds) * per_die + j / n_dparts;
    if (j / n_dparts >= per_die || win >= n_win || win_path[win] != (FULL_A ? kTileMany : kTileFew)) return;
    const int32_t d0 = (int32_t)(j % n_dparts) * (NB * 64);       // first feature column of this part
    const int32_t Dp = min(NB * 64, D - d0);

    const int lane = threadIdx.x;
    const int n = lane & 15, q = lane >> 4;
    const int64_t r0 = win * 16;
    if (lane < 17) {
        int64_t r = r0 + lane;
        s_rp[lane] = row_ptr[r < n_rows ? r : n_rows];
    }
    wave_lds_order();
    const int32_t u0 = win_unique_ptr[win];
    const int32_t cb = row_ptr[r0];             // the window's list sits at its edge offset
    const int32_t U = win_unique_ptr[win + 1] - u0;
    // ids of the neighbours of chunks 0 and 1 (lane k < 16 holds row k of the chunk)
    int32_t nid_cur = n < U ? col_to_row[cb + n] : -1;
    int32_t nid_nxt = KW + n < U ? col_to_row[cb + KW + n] : -1;
    const int32_t lo = s_rp[0], hi = s_rp[16];
    // only a forced policy puts a window with more edges into class kTileFew: its edges are then read from
    // global memory for every chunk
    const bool edges_in_lds = hi - lo <= kTileFewEdges;

    // FetchDense: chunk rows 4q .. 4q+3, features 4n .. 4n+3 of every block of 64
    const float *Xp = X + d0 + 4 * n;
    f32x4 xr[NB][4];
    auto fetch = [&](int32_t nid) {
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const int32_t node = __shfl(nid, 4 * q + jj);
#pragma unroll
            for (int fb = 0; fb < NB; ++fb) {
                xr[fb][jj] = f32x4{0.f, 0.f, 0.f, 0.f};
                if (node >= 0 && fb * 64 + 4 * n < Dp)
                    xr[fb][jj] = *reinterpret_cast<const f32x4 *>(Xp + (int64_t)node * ldx + fb * 64);
            }
        }
    };
    fetch(nid_cur);

    if constexpr (!FULL_A) {
        // the window's edges go to LDS; each lane writes and later reads only its own slots
#pragma unroll
        for (int e_i = 0; e_i < EPT; ++e_i) {
            const int32_t e = lo + lane + e_i * kWave;
            int32_t code = -1;
            if (edges_in_lds && e < hi) {
                int r = 0;
#pragma unroll
                for (int step = 8; step > 0; step >>= 1)
                    if (s_rp[r + step] <= e) r += step;
                code = (r * kAStrideW) << 16 | edge_to_col[e];     // condensed column < kTileFewEdges
                if (HAS_W) s_val[lane + e_i * kWave] = w[e];
            }
            s_code[lane + e_i * kWave] = code;
        }
    } else {
        // InitSparse for the whole window
        for (int32_t i = lane * 4; i < 16 * as; i += kWave * 4)
            *reinterpret_cast<float4 *>(a32 + i) = make_float4(0.f, 0.f, 0.f, 0.f);
        wave_lds_order();
        for (int32_t e0 = lo; e0 < hi; e0 += 8 * kWave) {
            int32_t cc[8];
            float vv[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int32_t e = min(e0 + lane + i * kWave, hi - 1);
                cc[i] = edge_to_col[e];
                vv[i] = HAS_W ? w[e] : 1.f;
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int32_t e = e0 + lane + i * kWave;
                if (e < hi) {
                    int r = 0;
#pragma unroll
                    for (int step = 8; step > 0; step >>= 1)
                        if (s_rp[r + step] <= e) r += step;
                    atomicAdd(&a32[r * as + cc[i]], vv[i]);
                }
            }
        }
        wave_lds_order();
    }

    f32x4 acc[NB][4];
#pragma unroll
    for (int fb = 0; fb < NB; ++fb)
#pragma unroll
        for (int m = 0; m < 4; ++m) acc[fb][m] = f32x4{0.f, 0.f, 0.f, 0.f};
    const float *a_src = a32 + n * as + 4 * q;                    // A: row n, k = 4q .. 4q+3

    for (int32_t k0 = 0; k0 < U; k0 += KW) {
        if constexpr (!FULL_A) {
            // InitSparse (the rows of this chunk are still on their way)
#pragma unroll
            for (int i = 0; i < 5; ++i) a32[lane + i * kWave] = 0.f;
            wave_lds_order();
            if (edges_in_lds) {
#pragma unroll
                for (int e_i = 0; e_i < EPT; ++e_i) {
                    const int32_t code = s_code[lane + e_i * kWave];
                    const int32_t cc = (code & 0xFFFF) - k0;
                    if (code >= 0 && cc >= 0 && cc < KW)
                        atomicAdd(&a32[(code >> 16) + cc], HAS_W ? s_val[lane + e_i * kWave] : 1.f);
                }
            } else {
                for (int32_t e = lo + lane; e < hi; e += kWave) {
                    const int32_t cc = edge_to_col[e] - k0;
                    if (cc >= 0 && cc < KW) {
                        int r = 0;
#pragma unroll
                        for (int step = 8; step > 0; step >>= 1)
                            if (s_rp[r + step] <= e) r += step;
                        atomicAdd(&a32[r * kAStrideW + cc], HAS_W ? w[e] : 1.f);
                    }
                }
            }
            wave_lds_order();
        }
        const float4 av = *reinterpret_cast<const float4 *>(a_src + (FULL_A ? k0 : 0));
        wave_lds_order();
        // A operand: the upper halves; with edge values also the two remainders
        uint2 ah, am, al;
        ah.x = upper_halves(av.x, av.y);
        ah.y = upper_halves(av.z, av.w);
        if (HAS_W) {
            const float r0x = below_upper_half(av.x), r0y = below_upper_half(av.y), r0z = below_upper_half(av.z),
                        r0w = below_upper_half(av.w);
            am.x = upper_halves(r0x, r0y);
            am.y = upper_halves(r0z, r0w);
            al.x = upper_halves(below_upper_half(r0x), below_upper_half(r0y));
            al.y = upper_halves(below_upper_half(r0z), below_upper_half(r0w));
        }
        // TCcompute: element m of the four pieces, split in three -> B operands of the MFMAs of (fb, m)
#pragma unroll
        for (int fb = 0; fb < NB; ++fb)
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const float v0 = xr[fb][0][m], v1 = xr[fb][1][m], v2 = xr[fb][2][m], v3 = xr[fb][3][m];
                const float s0 = below_upper_half(v0), s1 = below_upper_half(v1), s2 = below_upper_half(v2),
                            s3 = below_upper_half(v3);
                uint2 bh, bm, bl;
                bh.x = upper_halves(v0, v1);
                bh.y = upper_halves(v2, v3);
                bm.x = upper_halves(s0, s1);
                bm.y = upper_halves(s2, s3);
                bl.x = upper_halves(below_upper_half(s0), below_upper_half(s1));
                bl.y = upper_halves(below_upper_half(s2), below_upper_half(s3));
                f32x4 c = acc[fb][m];
                c = mfma16k16<TCG_BF16>(ah, bl, c);             // smallest terms first
                if (HAS_W) {
                    c = mfma16k16<TCG_BF16>(al, bh, c);
                    c = mfma16k16<TCG_BF16>(am, bm, c);
                    c = mfma16k16<TCG_BF16>(am, bh, c);
                }
                c = mfma16k16<TCG_BF16>(ah, bm, c);
                c = mfma16k16<TCG_BF16>(ah, bh, c);
                acc[fb][m] = c;
            }
        // next chunk's rows into the registers just consumed; the ids of the one after
        nid_cur = nid_nxt;
        if (k0 + KW < U) {
            fetch(nid_cur);
            nid_nxt = k0 + 2 * KW + n < U ? col_to_row[cb + k0 + 2 * KW + n] : -1;
        }
    }

    // StoreDense: acc[fb][m][r] = Y[r0 + 4q + r][d0 + 64 fb + 4n + m]: 16 lanes write 256 contiguous bytes of a row
#pragma unroll
    for (int fb = 0; fb < NB; ++fb) {
        const int32_t col = fb * 64 + 4 * n;
        if (col >= Dp) continue;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int64_t row = r0 + 4 * q + r;
            if (row < n_rows)
                store4(Y, y_dt, row * ldy + d0 + col,
                       make_float4(acc[fb][0][r], acc[fb][1][r], acc[fb][2][r], acc[fb][3][r]), y_vec);
        }
    }
}

template <bool HAS_W, int NB>
void launch_tile_f32(const tcg_meta *m, const float *X, int64_t ldx, int32_t D, const float *w, void *Y, int y_dt,
                     int64_t ldy, int tile_mask, hipStream_t s)
{
    const int32_t parts = (D + NB * 64 - 1) / (NB * 64);
    const bool y_vec = ldy % 4 == 0 && reinterpret_cast<uintptr_t>(Y) % (y_dt == TCG_F32 ? 16 : 8) == 0;
    const dim3 grid((unsigned)(kXcds * ceil_div(m->n_win, kXcds) * parts));
    if ((tile_mask >> kTileFew) & 1)
        hipLaunchKernelGGL((spmm_tile_f32_kernel<HAS_W, NB, false>), grid, dim3(kWave), 0, s, m->n_rows, m->n_win,
                           m->d_row_ptr, m->d_edge_to_col, m->d_win_unique_ptr, m->d_col_to_row, m->d_win_path, w, X,
                           ldx, D, parts, Y, y_dt, ldy, y_vec, 0);
    if ((tile_mask >> kTileMany) & 1) {
        const int32_t a_stride = (int32_t)((m->max_unique_many + KW - 1) / KW * KW + 4);
        hipLaunchKernelGGL((spmm_tile_f32_kernel<HAS_W, NB, true>), grid, dim3(kWave),
                           (size_t)16 * a_stride * sizeof(float), s, m->n_rows, m->n_win, m->d_row_ptr,
                           m->d_edge_to_col, m->d_win_unique_ptr, m->d_col_to_row, m->d_win_path, w, X, ldx, D, parts,
                           Y, y_dt, ldy, y_vec, a_stride);
    }
}

template <bool HAS_W>
void launch_tile_f32_s(const tcg_meta *m, const float *X, int64_t ldx, int32_t D, const float *w, void *Y,
                       int y_dt, int64_t ldy, int tile_mask, hipStream_t s)
{
    if (D <= 64) launch_tile_f32<HAS_W, 1>(m, X, ldx, D, w, Y, y_dt, ldy, tile_mask, s);
    else if (D <= 128) launch_tile_f32<HAS_W, 2>(m, X, ldx, D, w, Y, y_dt, ldy, tile_mask, s);
    else launch_tile_f32<HAS_W, 4>(m, X, ldx, D, w, Y, y_dt, ldy, tile_mask, s);
}

template <int DT, bool HAS_W, int NS, int HB>
void launch_wave(const tcg_meta *m, const void *X, int64_t ldx, int32_t D, const float *w, void *Y, int y_dt,
                 int64_t ldy, int tile_mask, hipStream_t s)
{
    const int32_t n_dparts = (D + NS * 16 - 1) / (NS * 16);
    // 4 outputs of a row leave in one store if every such group is aligned to its own size
    const bool y_vec = ldy % 4 == 0 && reinterpret_cast<uintptr_t>(Y) % (y_dt == TCG_F32 ? 16 : 8) == 0;
    const dim3 grid((unsigned)(kXcds * ceil_div(m->n_win, kXcds) * n_dparts));
    // Rows of more than 64 features in 16-row windows go to the kernel that loads them straight into the MFMA
    // operands; narrower rows would leave most of its lanes without a piece to load.
    constexpr bool kDirect = HB == 1 && NS >= 8;
    constexpr int NFB = NS >= 16 ? 2 : 1;                          // 128-feature blocks per wavefront
    const int32_t parts = (D + NFB * 128 - 1) / (NFB * 128);
    const dim3 grid_direct((unsigned)(kXcds * ceil_div(m->n_win, kXcds) * parts));
    if ((tile_mask >> kTileFew) & 1) {
        bool rest = true;        // windows of the class left for the LDS-staging kernel
        if constexpr (kDirect) {
            hipLaunchKernelGGL((spmm_tile_direct_kernel<DT, HAS_W, NFB, false>), grid_direct, dim3(kWave), 0, s,
                               m->n_rows, m->n_win, m->d_row_ptr, m->d_edge_to_col, m->d_win_unique_ptr,
                               m->d_col_to_row, m->d_win_path, w, static_cast<const char *>(X), ldx * 2, D, parts, Y,
                               y_dt, ldy, y_vec, 0);
            rest = m->policy == TCG_POLICY_TILE;       // only a forced policy puts larger windows into this class
        }
        if (rest)
            hipLaunchKernelGGL((spmm_tile_wave_kernel<DT, HAS_W, NS, false, HB>), grid, dim3(kWave), 0, s, m->n_rows,
                               m->n_win, m->d_row_ptr, m->d_edge_to_col, m->d_win_unique_ptr, m->d_col_to_row,
                               m->d_win_path, w, static_cast<const char *>(X), ldx * 2, D, n_dparts, Y, y_dt, ldy, y_vec,
                               0, kDirect);
    }
    if constexpr (HB == 1) {
        if ((tile_mask >> kTileMany) & 1) {
            // row stride of the window's condensed adjacency: its widest window rounded up to whole chunks,
            // plus 4 floats so that consecutive rows start in different banks
            const int32_t a_stride = (int32_t)((m->max_unique_many + KW - 1) / KW * KW + 4);
            const size_t a_bytes = (size_t)16 * a_stride * sizeof(float);
            if constexpr (kDirect)
                hipLaunchKernelGGL((spmm_tile_direct_kernel<DT, HAS_W, NFB, true>), grid_direct, dim3(kWave), a_bytes, s,
                                   m->n_rows, m->n_win, m->d_row_ptr, m->d_edge_to_col, m->d_win_unique_ptr,
                                   m->d_col_to_row, m->d_win_path, w, static_cast<const char *>(X), ldx * 2, D, parts,
                                   Y, y_dt, ldy, y_vec, a_stride);
            else
                hipLaunchKernelGGL((spmm_tile_wave_kernel<DT, HAS_W, NS, true, 1>), grid, dim3(kWave), a_bytes, s,
                                   m->n_rows, m->n_win, m->d_row_ptr, m->d_edge_to_col, m->d_win_unique_ptr,
                                   m->d_col_to_row, m->d_win_path, w, static_cast<const char *>(X), ldx * 2, D,
                                   n_dparts, Y, y_dt, ldy, y_vec, a_stride, false);
        }
    }
}

template <int DT, bool HAS_W>
void launch_wave_s(const tcg_meta *m, const void *X, int64_t ldx, int32_t D, const float *w, void *Y, int y_dt,
                   int64_t ldy, int tile_mask, hipStream_t s)
{
    if (m->win_h == 32) {      // two row blocks per wavefront: half as many feature slices each
        if (D <= 64) launch_wave<DT, HAS_W, 4, 2>(m, X, ldx, D, w, Y, y_dt, ldy, tile_mask, s);
        else launch_wave<DT, HAS_W, 8, 2>(m, X, ldx, D, w, Y, y_dt, ldy, tile_mask, s);
    } else if (D <= 64) launch_wave<DT, HAS_W, 4, 1>(m, X, ldx, D, w, Y, y_dt, ldy, tile_mask, s);
    else if (D <= 128) launch_wave<DT, HAS_W, 8, 1>(m, X, ldx, D, w, Y, y_dt, ldy, tile_mask, s);
    else launch_wave<DT, HAS_W, 16, 1>(m, X, ldx, D, w, Y, y_dt, ldy, tile_mask, s);
}

}  // namespace

bool tile_path_supports(tcg_dtype x_dt, int32_t D, int64_t ldx, const void *X)
{
    return x_dt != TCG_F32 && D % 8 == 0 && D <= 512 && ldx % 8 == 0 &&
           (reinterpret_cast<uintptr_t>(X) & 15) == 0;
}

bool spmm_tile_supports(tcg_dtype x_dt, int32_t D, int64_t ldx, const void *X, int32_t win_h)
{
    if (x_dt == TCG_F32)       // the kernel that splits fp32 operands into bf16 triples
        return win_h == 16 && D % 4 == 0 && D <= 1024 && ldx % 4 == 0 && (reinterpret_cast<uintptr_t>(X) & 15) == 0;
    return (win_h == 16 || win_h == 32) && tile_path_supports(x_dt, D, ldx, X);
}

int spmm_tile_launch(tcg_meta *m, const void *d_X, tcg_dtype x_dt, int32_t D, int64_t ldx, const float *d_w,
                     void *d_Y, tcg_dtype y_dt, int64_t ldy, int tile_mask, hipStream_t s)
{
    if (x_dt == TCG_F32) {
        const float *X = static_cast<const float *>(d_X);
        if (d_w) launch_tile_f32_s<true>(m, X, ldx, D, d_w, d_Y, (int)y_dt, ldy, tile_mask, s);
        else launch_tile_f32_s<false>(m, X, ldx, D, d_w, d_Y, (int)y_dt, ldy, tile_mask, s);
    } else if (x_dt == TCG_BF16) {
        if (d_w) launch_wave_s<TCG_BF16, true>(m, d_X, ldx, D, d_w, d_Y, (int)y_dt, ldy, tile_mask, s);
        else launch_wave_s<TCG_BF16, false>(m, d_X, ldx, D, d_w, d_Y, (int)y_dt, ldy, tile_mask, s);
    } else {
        if (d_w) launch_wave_s<TCG_F16, true>(m, d_X, ldx, D, d_w, d_Y, (int)y_dt, ldy, tile_mask, s);
        else launch_wave_s<TCG_F16, false>(m, d_X, ldx, D, d_w, d_Y, (int)y_dt, ldy, tile_mask, s);
    }
    return launch_status("spmm_tile kernels");
}

}  // namespace tcg
