// Neighbour aggregation Y = (w (.) A) X (Equation 1 / Algorithm 2 of the paper), gather path.
//
// The paper maps one row window to one thread block and multiplies condensed tiles on tensor
// cores.  On MI355X the operation is bound by the HBM gathers of X rows, and on graphs without
// much neighbour sharing inside a window a dense tile is mostly zeros, so windows that are not
// assigned to the condensed-tile path run here:
//   - every row is cut into segments of at most kSegLen edges (hub rows of power-law graphs
//     would otherwise serialise on one wavefront);
//   - a group of G lanes (G * 16 bytes >= one feature row) owns a segment; each lane keeps its
//     16-byte slice of the row sum in registers, so every gathered X row is one fully coalesced
//     request of the group and a 64-wide wavefront has 64 / G rows in flight per instruction;
//   - neighbour ids (and edge values) of the next iteration are fetched before the current
//     iteration's rows are consumed, so the id -> row dependency is off the critical path;
//   - segments of one row window sit in the same workgroup, so neighbours shared inside the
//     window are served by the CU's cache rather than HBM;
//   - a row with a single segment is written straight to Y; a longer row writes one fp32
//     partial per segment and a second kernel adds them in segment order (deterministic).
#include "common.h"
#include "devutil.h"

#include <stdio.h>

#include <mutex>

namespace tcg {

// spmm_tile.hip
int spmm_tile_launch(tcg_meta *m, const void *d_X, tcg_dtype x_dt, int32_t D, int64_t ldx, const float *d_w,
                     void *d_Y, tcg_dtype y_dt, int64_t ldy, int tile_mask, hipStream_t s);

namespace {

constexpr int kBlock = 256;
constexpr int64_t kSlabBytes = 256;                       // see spmm_impl
constexpr int64_t kSlabMinMatrixBytes = (int64_t)64 << 20;

template <int DT, int G, int NCH, bool HAS_W, int UNROLL>
__global__ __launch_bounds__(kBlock) void spmm_gather_kernel(
    const int32_t *__restrict__ lane_tab, const int32_t *__restrict__ seg_row, const int32_t *__restrict__ seg_ebeg,
    const int32_t *__restrict__ seg_dst, const int32_t *__restrict__ row_ptr,
    const int32_t *__restrict__ col_idx, const float *__restrict__ w, const char *__restrict__ X,
    int64_t ldx_bytes, int32_t n_chunks, int32_t D, void *__restrict__ Y, int y_dt, int64_t ldy,
    float *__restrict__ partial, int64_t partial_ld, const uint8_t *__restrict__ win_path, int32_t win_h,
    int tile_mask, int y_vec)
{
    constexpr int VEC = Elem<DT>::VEC;
    const int lane = threadIdx.x % G;
    const int64_t seg = plan_segment(lane_tab, kBlock / G, threadIdx.x / G);
    if (seg < 0) return;
    const int32_t row = seg_row[seg];
    if (win_path != nullptr && ((tile_mask >> win_path[row / win_h]) & 1)) return;
    const int32_t eb = seg_ebeg[seg];
    const int32_t dst = seg_dst[seg];
    const int32_t ee = segment_end(eb, dst, row, row_ptr);

    float acc[NCH][VEC];
#pragma unroll
    for (int c = 0; c < NCH; ++c)
#pragma unroll
        for (int k = 0; k < VEC; ++k) acc[c][k] = 0.f;

    if (eb < ee) {
        // Ids (and edge values) are always read from a clamped, valid position, so these loads carry
        // no predicate and are issued back to back; only the row loads of a ragged tail are masked.
        const int32_t last = ee - 1;
        const uint32_t ldx32 = (uint32_t)ldx_bytes;
        // Ids (and edge values) are loaded a block of IDB entries at a time, once per lane group -- lane l takes
        // entries l, l + G, ... of the block -- and handed round inside the group: every lane loading all of
        // its step's ids costs more load instructions than narrow rows do themselves.  A block is a whole cache
        // line of ids requested in one go: asked for eight at a time, step by step, the line had left the L2
        // again between two steps (the gathered rows turn the cache over every few microseconds) and was fetched
        // up to four times -- 0.3 GB read per launch for the 76 MB of either array on the 1M-node graph.
        // (Four-lane groups keep half a line when there are edge values too: the registers of a whole one cost more.)
        constexpr int IDB = G <= 4 ? (HAS_W ? 16 : 32) : (UNROLL * 8 < (G > 32 ? 64 : 32) ? UNROLL * 8 : (G > 32 ? 64 : 32));
        constexpr int PER = (IDB + G - 1) / G;
        constexpr int STEPS = IDB / UNROLL;
        auto request = [&](int32_t e0, int32_t (&mc)[PER], float (&mw)[PER]) {
#pragma unroll
            for (int k = 0; k < PER; ++k) {
                const int32_t en = min(e0 + lane + k * G, last);
                mc[k] = col_idx[en];
                mw[k] = HAS_W ? w[en] : 1.f;
            }
        };
        int32_t mc[PER];
        float mw[PER];
        request(eb, mc, mw);
        for (int32_t e = eb; e < ee; e += IDB) {
            // The next block's ids go out first: they are older than the row loads below, so a wait for rows
            // also covers them and their latency hides under the rows'.
            int32_t mc_next[PER];
            float mw_next[PER];
            request(e + IDB, mc_next, mw_next);
            static_for<STEPS>([&](auto step) {
                constexpr int S = decltype(step)::value;
                const int32_t es = e + S * UNROLL;
                if (es < ee) {
                    int32_t cn[UNROLL];
                    float wc[UNROLL];
                    block_ids<G, UNROLL, PER, S>(mc, cn);
                    if constexpr (HAS_W) block_ids<G, UNROLL, PER, S>(mw, wc);
                    uint4 raw[UNROLL][NCH];
#pragma unroll
                    for (int u = 0; u < UNROLL; ++u) {
                        if (!HAS_W || es + u >= ee) wc[u] = 0.f;
                        const char *xr = X + (uint64_t)(uint32_t)cn[u] * ldx32;
#pragma unroll
                        for (int c = 0; c < NCH; ++c) {
                            const int chunk = lane + c * G;
                            raw[u][c] = make_uint4(0, 0, 0, 0);
                            if (es + u < ee && chunk < n_chunks)
                                raw[u][c] = *reinterpret_cast<const uint4 *>(xr + (uint32_t)chunk * 16u);
                        }
                    }
#pragma unroll
                    for (int u = 0; u < UNROLL; ++u) {
#pragma unroll
                        for (int c = 0; c < NCH; ++c) {
                            float v[VEC];
                            unpack16<DT>(raw[u][c], v);   // masked-off loads left zeros: they add nothing
#pragma unroll
                            for (int k = 0; k < VEC; ++k) {
                                if (HAS_W) acc[c][k] = fmaf(wc[u], v[k], acc[c][k]);
                                else acc[c][k] += v[k];
                            }
                        }
                    }
                }
            });
#pragma unroll
            for (int k = 0; k < PER; ++k) {
                mc[k] = mc_next[k];
                mw[k] = mw_next[k];
            }
        }
    }

#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        int chunk = lane + c * G;
        if (chunk >= n_chunks) continue;
        int64_t d0 = (int64_t)chunk * VEC;
        if (dst >= 0) {
            float *p = partial + (int64_t)segment_slot(dst) * partial_ld + d0;
#pragma unroll
            for (int k = 0; k < VEC; k += 4)
                stream_store(p + k, acc[c][k], acc[c][k + 1], acc[c][k + 2], acc[c][k + 3]);   // like Y: not in L2's way
        } else if (y_dt == TCG_F32 && y_vec) {
            // the branch stays outside the loop: the 16-byte stores of a lane then leave back to back and meet in
            // the same write (apart, they reach memory as two partial ones: +0.27 GB written per call on the
            // 1M-node graph with bf16 features)
            float *p = static_cast<float *>(Y) + (int64_t)row * ldy + d0;
#pragma unroll
            for (int k = 0; k < VEC; k += 4) stream_store(p + k, acc[c][k], acc[c][k + 1], acc[c][k + 2], acc[c][k + 3]);
        } else {
            bool stored = false;
            if constexpr (VEC == 8) {
                if (y_vec == 2) {
                    store8_16bit(static_cast<uint16_t *>(Y) + (int64_t)row * ldy + d0, y_dt, acc[c]);
                    stored = true;
                }
            }
            if (!stored) {
#pragma unroll
                for (int k = 0; k < VEC; k += 4)
                    store4(Y, y_dt, (int64_t)row * ldy + d0 + k,
                           make_float4(acc[c][k], acc[c][k + 1], acc[c][k + 2], acc[c][k + 3]), y_vec != 0);
            }
        }
    }
}

// Rows that cannot be read in 16-byte pieces (width or leading dimension not a multiple of 16 bytes,
// or a misaligned base): the same segment / group / prefetch structure with pieces of PB = 4 bytes (one
// fp32, two 16-bit elements) or one 16-bit element per lane and pass; G lanes per segment, n_pieces <=
// G * NCH.  Narrow outputs of a layer (a handful of classes) land here.
template <int DT, int PB, int G, int NCH, bool HAS_W, int UNROLL>
__global__ __launch_bounds__(kBlock) void spmm_gather_small_kernel(
    const int32_t *__restrict__ lane_tab, const int32_t *__restrict__ seg_row, const int32_t *__restrict__ seg_ebeg,
    const int32_t *__restrict__ seg_dst, const int32_t *__restrict__ row_ptr,
    const int32_t *__restrict__ col_idx, const float *__restrict__ w, const char *__restrict__ X,
    int64_t ldx_bytes, int32_t n_pieces, void *__restrict__ Y, int y_dt, int64_t ldy, float *__restrict__ partial,
    int64_t partial_ld, const uint8_t *__restrict__ win_path, int32_t win_h, int tile_mask)
{
    using Pc = Piece<DT, PB>;
    constexpr int VEC = Pc::VEC;
    const int lane = threadIdx.x % G;
    const int64_t seg = plan_segment(lane_tab, kBlock / G, threadIdx.x / G);
    if (seg < 0) return;
    const int32_t row = seg_row[seg];
    if (win_path != nullptr && ((tile_mask >> win_path[row / win_h]) & 1)) return;
    const int32_t eb = seg_ebeg[seg];
    const int32_t dst = seg_dst[seg];
    const int32_t ee = segment_end(eb, dst, row, row_ptr);

    float acc[NCH][VEC];
#pragma unroll
    for (int c = 0; c < NCH; ++c)
#pragma unroll
        for (int k = 0; k < VEC; ++k) acc[c][k] = 0.f;

    if (eb < ee) {
        const int32_t last = ee - 1;
        int32_t cn[UNROLL];
        float wn[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int32_t en = min(eb + u, last);
            cn[u] = col_idx[en];
            wn[u] = HAS_W ? w[en] : 1.f;
        }
        for (int32_t e = eb; e < ee; e += UNROLL) {
            int32_t cnext[UNROLL];
            float wnext[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const int32_t en = min(e + UNROLL + u, last);
                cnext[u] = col_idx[en];
                wnext[u] = HAS_W ? w[en] : 1.f;
            }
            float v[UNROLL][NCH][VEC];
            float wc[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                wc[u] = (e + u < ee) ? wn[u] : 0.f;
                const char *xr = X + (int64_t)cn[u] * ldx_bytes;
#pragma unroll
                for (int c = 0; c < NCH; ++c) {
                    const int piece = lane + c * G;
#pragma unroll
                    for (int k = 0; k < VEC; ++k) v[u][c][k] = 0.f;
                    if (e + u < ee && piece < n_pieces) Pc::load(xr + piece * PB, v[u][c]);
                }
            }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                cn[u] = cnext[u];
                wn[u] = wnext[u];
            }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u)
#pragma unroll
                for (int c = 0; c < NCH; ++c)
#pragma unroll
                    for (int k = 0; k < VEC; ++k) {
                        if (HAS_W) acc[c][k] = fmaf(wc[u], v[u][c][k], acc[c][k]);
                        else acc[c][k] += v[u][c][k];
                    }
        }
    }

#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int piece = lane + c * G;
        if (piece >= n_pieces) continue;
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            const int d = piece * VEC + k;
            if (dst >= 0) partial[(int64_t)segment_slot(dst) * partial_ld + d] = acc[c][k];
            else store_elem(Y, (int64_t)row * ldy + d, y_dt, acc[c][k]);
        }
    }
}

// Any D, any alignment: one wavefront per segment, one lane per feature element (D > 256 only).
template <bool HAS_W>
__global__ __launch_bounds__(kBlock) void spmm_gather_generic_kernel(
    const int32_t *__restrict__ lane_tab, const int32_t *__restrict__ seg_row, const int32_t *__restrict__ seg_ebeg,
    const int32_t *__restrict__ seg_dst, const int32_t *__restrict__ row_ptr,
    const int32_t *__restrict__ col_idx, const float *__restrict__ w, const void *__restrict__ X, int x_dt,
    int64_t ldx, int32_t D, void *__restrict__ Y, int y_dt, int64_t ldy, float *__restrict__ partial,
    int64_t partial_ld, const uint8_t *__restrict__ win_path, int32_t win_h, int tile_mask)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t seg = plan_segment(lane_tab, kBlock / kWave, threadIdx.x >> 6);
    if (seg < 0) return;
    const int32_t row = seg_row[seg];
    if (win_path != nullptr && ((tile_mask >> win_path[row / win_h]) & 1)) return;
    const int32_t eb = seg_ebeg[seg];
    const int32_t dst = seg_dst[seg];
    const int32_t ee = segment_end(eb, dst, row, row_ptr);
    for (int32_t d = lane; d < D; d += kWave) {
        float acc = 0.f;
        for (int32_t e = eb; e < ee; ++e) {
            float x = load_elem(X, (int64_t)col_idx[e] * ldx + d, x_dt);
            acc = HAS_W ? fmaf(w[e], x, acc) : acc + x;
        }
        if (dst >= 0) partial[(int64_t)segment_slot(dst) * partial_ld + d] = acc;
        else store_elem(Y, (int64_t)row * ldy + d, y_dt, acc);
    }
}

// Adds the per-segment partials of every long row: one workgroup per row.  When D is a multiple of 4 (and
// at most 4 * kBlock) a thread takes four columns, so D / 4 threads cover a partial row and the kBlock /
// (D / 4) thread groups each add every such-and-such partial (four loads in flight); the groups' sums
// meet in LDS and are added in group order.  The order of the additions is fixed by the sizes alone, so
// results repeat from run to run.  A hub row of a power-law graph has hundreds of partials:
// adding them one after the other in a single thread per column set the duration of the whole kernel.
__global__ __launch_bounds__(kBlock) void spmm_reduce_long_kernel(
    int64_t n_long, const int32_t *__restrict__ long_row, const int32_t *__restrict__ long_slot_ptr,
    const float *__restrict__ partial, int64_t partial_ld, int32_t D, void *__restrict__ Y, int y_dt,
    int64_t ldy, const uint8_t *__restrict__ win_path, int32_t win_h, int tile_mask, int y_vec)
{
    __shared__ float4 s_part[kBlock];
    const int64_t li = blockIdx.x;
    const int32_t row = long_row[li];
    if (win_path != nullptr && ((tile_mask >> win_path[row / win_h]) & 1)) return;
    const int32_t s0 = long_slot_ptr[li], s1 = long_slot_ptr[li + 1];
    const int32_t c4 = D / 4;                                  // threads per partial row
    const int32_t n_threads = blockDim.x;                      // kBlock, or half of it for rows of up to 64 columns
    if (D % 4 == 0 && c4 <= n_threads) {
        const int32_t nsg = n_threads / c4;                       // groups of threads, each on its own partials
        const int32_t c = threadIdx.x % c4, sg = threadIdx.x / c4;
        float4 a[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) a[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (sg < nsg) {
            const float *base = partial + 4 * c;
            int32_t s = s0 + sg;
            for (; s + 3 * nsg < s1; s += 4 * nsg) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const float4 v = *reinterpret_cast<const float4 *>(base + (int64_t)(s + u * nsg) * partial_ld);
                    a[u].x += v.x;
                    a[u].y += v.y;
                    a[u].z += v.z;
                    a[u].w += v.w;
                }
            }
            for (; s < s1; s += nsg) {
                const float4 v = *reinterpret_cast<const float4 *>(base + (int64_t)s * partial_ld);
                a[0].x += v.x;
                a[0].y += v.y;
                a[0].z += v.z;
                a[0].w += v.w;
            }
        }
        s_part[threadIdx.x] = make_float4((a[0].x + a[1].x) + (a[2].x + a[3].x), (a[0].y + a[1].y) + (a[2].y + a[3].y),
                                          (a[0].z + a[1].z) + (a[2].z + a[3].z), (a[0].w + a[1].w) + (a[2].w + a[3].w));
        __syncthreads();
        if (sg == 0) {
            float4 t = s_part[c];
            for (int32_t g = 1; g < nsg; ++g) {
                const float4 v = s_part[g * c4 + c];
                t.x += v.x;
                t.y += v.y;
                t.z += v.z;
                t.w += v.w;
            }
            store4(Y, y_dt, (int64_t)row * ldy + 4 * c, t, y_vec);
        }
        return;
    }
    for (int32_t d = threadIdx.x; d < D; d += n_threads) {
        float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
        int32_t s = s0;
        for (; s + 4 <= s1; s += 4) {
            a0 += partial[(int64_t)(s + 0) * partial_ld + d];
            a1 += partial[(int64_t)(s + 1) * partial_ld + d];
            a2 += partial[(int64_t)(s + 2) * partial_ld + d];
            a3 += partial[(int64_t)(s + 3) * partial_ld + d];
        }
        for (; s < s1; ++s) a0 += partial[(int64_t)s * partial_ld + d];
        store_elem(Y, (int64_t)row * ldy + d, y_dt, (a0 + a1) + (a2 + a3));
    }
}

// Narrow results (4, 8 or 16 columns): one wavefront per split row and four rows per
// workgroup, no LDS and no barrier.  A lane takes four columns of every n-th partial (n = 64 / (D / 4) groups of
// lanes, two loads in flight each), the groups meet in a butterfly of shuffles whose order is fixed by the sizes.
// With one workgroup per row the 2 * 10^4 split rows of the 1M-node graph took 24 us at 16 columns, where the
// partials are 12 MB.  (From 32 columns on a wavefront has too few groups for a hub row's hundreds of partials and
// the workgroup-per-row kernel above is quicker.)
__global__ __launch_bounds__(kBlock) void spmm_reduce_long_wave_kernel(
    int64_t n_long, const int32_t *__restrict__ long_row, const int32_t *__restrict__ long_slot_ptr,
    const float *__restrict__ partial, int64_t partial_ld, int c4_log2, void *__restrict__ Y, int y_dt, int64_t ldy,
    const uint8_t *__restrict__ win_path, int32_t win_h, int tile_mask, int y_vec)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t li = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / kWave;
    if (li >= n_long) return;                            // whole wavefronts leave together
    const int32_t row = long_row[li];
    if (win_path != nullptr && ((tile_mask >> win_path[row / win_h]) & 1)) return;
    const int32_t s0 = long_slot_ptr[li], s1 = long_slot_ptr[li + 1];
    const int c = lane & ((1 << c4_log2) - 1), sg = lane >> c4_log2, nsg = kWave >> c4_log2;
    const float *base = partial + 4 * c;
    float4 a0 = make_float4(0.f, 0.f, 0.f, 0.f), a1 = a0;
    int32_t sl = s0 + sg;
    for (; sl + nsg < s1; sl += 2 * nsg) {
        const float4 v0 = *reinterpret_cast<const float4 *>(base + (int64_t)sl * partial_ld);
        const float4 v1 = *reinterpret_cast<const float4 *>(base + (int64_t)(sl + nsg) * partial_ld);
        a0.x += v0.x; a0.y += v0.y; a0.z += v0.z; a0.w += v0.w;
        a1.x += v1.x; a1.y += v1.y; a1.z += v1.z; a1.w += v1.w;
    }
    if (sl < s1) {
        const float4 v0 = *reinterpret_cast<const float4 *>(base + (int64_t)sl * partial_ld);
        a0.x += v0.x; a0.y += v0.y; a0.z += v0.z; a0.w += v0.w;
    }
    float4 t = make_float4(a0.x + a1.x, a0.y + a1.y, a0.z + a1.z, a0.w + a1.w);
    for (int off = 1 << c4_log2; off < kWave; off <<= 1) {
        t.x += __shfl_xor(t.x, off, kWave);
        t.y += __shfl_xor(t.y, off, kWave);
        t.z += __shfl_xor(t.z, off, kWave);
        t.w += __shfl_xor(t.w, off, kWave);
    }
    if (sg == 0) store4(Y, y_dt, (int64_t)row * ldy + 4 * c, t, y_vec);
}

struct GatherArgs {
    const tcg_meta *m;
    float *partial;     // partial sums of split rows: the plan's buffer or the library's static one
    const void *X;
    int64_t ldx;
    int32_t D;
    const float *w;
    void *Y;
    int y_dt;
    int64_t ldy;
    const uint8_t *win_path;
    int tile_mask;      // bit c set: windows of path class c are handled by the tile kernels
    hipStream_t s;
};

template <int DT, int G, int NCH, bool HAS_W>
void launch_gather(const GatherArgs &a, int32_t n_chunks)
{
    constexpr int UNROLL = NCH == 1 ? 8 : (NCH == 2 ? 4 : 2);
    const tcg_meta *m = a.m;
    const int gpb = kBlock / G;
    const unsigned grid = (unsigned)plan_grid(m->h_lane_tab, gpb);
    // 0: scalar stores; 1: four results per store; 2: a 16-bit result whose rows are 16-byte aligned (eight per store)
    int y_vec = (a.ldy & 3) == 0 && reinterpret_cast<uintptr_t>(a.Y) % (a.y_dt == TCG_F32 ? 16 : 8) == 0;
    if (y_vec && a.y_dt != TCG_F32 && (a.ldy & 7) == 0 && (reinterpret_cast<uintptr_t>(a.Y) & 15) == 0) y_vec = 2;
    hipLaunchKernelGGL((spmm_gather_kernel<DT, G, NCH, HAS_W, UNROLL>), dim3(grid), dim3(kBlock), 0, a.s,
                       m->d_lane_tab, m->d_seg_row, m->d_seg_ebeg, m->d_seg_dst, m->d_row_ptr, m->d_col_idx, a.w,
                       static_cast<const char *>(a.X), a.ldx * Elem<DT>::BYTES, n_chunks, a.D, a.Y, a.y_dt,
                       a.ldy, a.partial, (int64_t)a.D, a.win_path, m->win_h, a.tile_mask, y_vec);
}

template <int DT, bool HAS_W>
bool dispatch_gather(const GatherArgs &a, int32_t n_chunks)
{
    if (n_chunks <= 4) launch_gather<DT, 4, 1, HAS_W>(a, n_chunks);
    else if (n_chunks <= 8) launch_gather<DT, 8, 1, HAS_W>(a, n_chunks);
    else if (n_chunks <= 16) launch_gather<DT, 16, 1, HAS_W>(a, n_chunks);
    else if (n_chunks <= 32) launch_gather<DT, 32, 1, HAS_W>(a, n_chunks);
    else if (n_chunks <= 64) launch_gather<DT, 64, 1, HAS_W>(a, n_chunks);
    else if (n_chunks <= 128) launch_gather<DT, 64, 2, HAS_W>(a, n_chunks);
    else if (n_chunks <= 256) launch_gather<DT, 64, 4, HAS_W>(a, n_chunks);
    else return false;
    return true;
}

template <int DT>
bool dispatch_gather_w(const GatherArgs &a, int32_t n_chunks)
{
    return a.w ? dispatch_gather<DT, true>(a, n_chunks) : dispatch_gather<DT, false>(a, n_chunks);
}

template <int DT, int PB, int G, int NCH, bool HAS_W>
void launch_small(const GatherArgs &a, int32_t n_pieces)
{
    constexpr int UNROLL = NCH == 1 ? 8 : (NCH == 2 ? 4 : 2);
    const tcg_meta *m = a.m;
    const unsigned grid = (unsigned)plan_grid(m->h_lane_tab, kBlock / G);
    hipLaunchKernelGGL((spmm_gather_small_kernel<DT, PB, G, NCH, HAS_W, UNROLL>), dim3(grid), dim3(kBlock), 0, a.s,
                       m->d_lane_tab, m->d_seg_row, m->d_seg_ebeg, m->d_seg_dst, m->d_row_ptr, m->d_col_idx, a.w,
                       static_cast<const char *>(a.X), a.ldx * Elem<DT>::BYTES, n_pieces, a.Y, a.y_dt, a.ldy,
                       a.partial, (int64_t)a.D, a.win_path, m->win_h, a.tile_mask);
}

template <int DT, int PB, bool HAS_W>
bool dispatch_small(const GatherArgs &a)
{
    const int32_t n = a.D / Piece<DT, PB>::VEC;
    if (n <= 4) launch_small<DT, PB, 4, 1, HAS_W>(a, n);
    else if (n <= 8) launch_small<DT, PB, 8, 1, HAS_W>(a, n);
    else if (n <= 16) launch_small<DT, PB, 16, 1, HAS_W>(a, n);
    else if (n <= 32) launch_small<DT, PB, 32, 1, HAS_W>(a, n);
    else if (n <= 64) launch_small<DT, PB, 64, 1, HAS_W>(a, n);
    else if (n <= 128) launch_small<DT, PB, 64, 2, HAS_W>(a, n);
    else if (n <= 256) launch_small<DT, PB, 64, 4, HAS_W>(a, n);
    else return false;
    return true;
}

template <int DT>
bool dispatch_elem_w(const GatherArgs &a)
{
    if (small_piece_bytes(Elem<DT>::BYTES, a.D, a.ldx, a.ldx, a.X, a.X) == 4)
        return a.w ? dispatch_small<DT, 4, true>(a) : dispatch_small<DT, 4, false>(a);
    if constexpr (DT != TCG_F32) return a.w ? dispatch_small<DT, 2, true>(a) : dispatch_small<DT, 2, false>(a);
    return false;
}

}  // namespace

// Scratch of tcg_spmm_noalloc: the partial sums of split rows, for callers that must not allocate.  Every
// GPU the library runs on holds its own copy of the array until the process ends.  In host code the
// array's name is only a handle for hipGetSymbolAddress; kernels get the address that call returned.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mu;
static void *g_scratch_ptr[kMaxDevices] = {nullptr};

int static_scratch(float **ptr, int64_t *capacity_elems)
{
    int dev = 0;
    TCG_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return TCG_EINVAL;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        TCG_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));      // this device's copy of the array
        g_scratch_ptr[dev] = p;
    }
    if (ptr) *ptr = static_cast<float *>(g_scratch_ptr[dev]);
    if (capacity_elems) *capacity_elems = (int64_t)(kStaticScratchBytes / sizeof(float));
    return TCG_OK;
}

int reserve_partial(tcg_meta *m, int32_t D, hipStream_t s)
{
    const int64_t need = m->n_slots * (int64_t)D;
    if (need <= m->partial_elems) return TCG_OK;
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &cap) == hipSuccess && cap != hipStreamCaptureStatusNone) {
        set_message("the partial-sum scratch of this plan is too small for this feature width and cannot be "
                    "regrown while the stream is being captured: call tcg_sgt_reserve first");
        return TCG_ESCRATCH;
    }
    float *fresh = nullptr;
    TCG_TRY(dev_alloc(&fresh, need));        // on failure the plan keeps the scratch it has
    if (m->partial_owned) {
        TCG_HIP(hipStreamSynchronize(s));
        pool_free(m->d_partial);
    }
    m->d_partial = fresh;
    m->partial_elems = need;
    m->partial_owned = true;
    return TCG_OK;
}

int spmm_impl(tcg_meta *m, const void *d_X, tcg_dtype x_dt, int32_t D, int64_t ldx, const float *d_w,
              void *d_Y, tcg_dtype y_dt, int64_t ldy, bool no_alloc, hipStream_t s)
{
    if (m->n_rows == 0) return TCG_OK;

    // Scratch for the partial sums of rows that span several segments: the plan's own buffer (regrown for
    // a wider D than it was reserved for), or the library's static array for callers that cannot allocate.
    const int64_t need = m->n_slots * (int64_t)D;
    float *partial = nullptr;
    if (no_alloc) {
        int64_t cap = 0;
        TCG_TRY(static_scratch(&partial, &cap));
        if (need > cap) {
            char msg[200];
            snprintf(msg, sizeof(msg), "tcg_spmm_noalloc: %lld split-row segments x D = %d need %lld bytes of scratch, "
                     "the static buffer holds %lld", (long long)m->n_slots, (int)D, (long long)(need * 4),
                     (long long)kStaticScratchBytes);
            set_message(msg);
            return TCG_ESCRATCH;
        }
    } else {
        TCG_TRY(reserve_partial(m, D, s));
        partial = m->d_partial;
    }

    // Which classes of tile-path windows really go to the MFMA kernels depends on the feature width, which
    // the plan does not know: measured on MI355X (the calibration tool's sweeps), narrow rows are gathered
    // faster than they are staged through LDS, and building a window's whole condensed adjacency in LDS
    // pays only for wider rows still.  A forced tile policy is taken literally.
    int tile_mask = 0;
    if (m->n_tile_win > 0 && spmm_tile_supports(x_dt, D, ldx, d_X, m->win_h)) {
        const bool forced = m->policy == TCG_POLICY_TILE;
        if (forced || D >= kTileMinWidthFew) tile_mask |= 1 << kTileFew;
        if (forced || D >= kTileMinWidthMany) tile_mask |= 1 << kTileMany;
    }
    const int64_t n_few = m->n_tile_win - m->n_tile_many;
    const bool few = ((tile_mask >> kTileFew) & 1) || n_few == 0;            // class handled, or empty
    const bool many = ((tile_mask >> kTileMany) & 1) || m->n_tile_many == 0;
    if (n_few == 0) tile_mask &= ~(1 << kTileFew);
    if (m->n_tile_many == 0) tile_mask &= ~(1 << kTileMany);
    const bool use_tiles = tile_mask != 0;
    const uint8_t *win_path = use_tiles ? m->d_win_path : nullptr;
    if (use_tiles) TCG_TRY(spmm_tile_launch(m, d_X, x_dt, D, ldx, d_w, d_Y, y_dt, ldy, tile_mask, s));
    if (few && many && m->nnz_tile == m->nnz && m->n_tile_win == m->n_win) return TCG_OK;  // nothing left

    GatherArgs a{m, partial, d_X, ldx, D, d_w, d_Y, (int)y_dt, ldy, win_path, tile_mask, s};
    const int es = dtype_size(x_dt);
    const bool vec_ok = ((int64_t)D * es) % 16 == 0 && (ldx * es) % 16 == 0 && ldx * es < (1ll << 32) &&
                        (reinterpret_cast<uintptr_t>(d_X) & 15) == 0;
    bool done = false;
    if (vec_ok) {
        // Rows of 512 bytes and more are gathered in slabs of 256 bytes, one launch per slab, when X is too big
        // for the caches: each launch then keeps twice (or four times) as many rows per megabyte of L2, and the
        // hub columns of a skewed graph are re-read from memory less often.  Measured on the 1M-node R-MAT graph,
        // fp32 D = 128: 5.55 GB read in one launch, 2 x 2.35 GB in two, 1.15 -> 1.06 ms; narrower slabs or rows
        // that are 256 bytes to begin with (bf16 D = 128) gain nothing.  Every slab writes its own columns of Y
        // and of the split rows' partial sums, so nothing is added up across launches.
        const int64_t row_bytes = (int64_t)D * es;
        int slabs = 1;
        if (row_bytes >= 512 && row_bytes % kSlabBytes == 0 && (int64_t)m->n_cols * row_bytes >= kSlabMinMatrixBytes)
            slabs = (int)(row_bytes / kSlabBytes);
        const int32_t n_chunks = (int32_t)(row_bytes / slabs / 16);
        const int32_t slab_feats = D / slabs;
        done = true;
        for (int sl = 0; sl < slabs && done; ++sl) {
            GatherArgs b = a;
            b.X = static_cast<const char *>(d_X) + (int64_t)sl * slab_feats * es;
            b.Y = static_cast<char *>(d_Y) + (int64_t)sl * slab_feats * dtype_size(y_dt);
            b.partial = partial + (int64_t)sl * slab_feats;
            if (x_dt == TCG_F32) done = dispatch_gather_w<TCG_F32>(b, n_chunks);
            else if (x_dt == TCG_BF16) done = dispatch_gather_w<TCG_BF16>(b, n_chunks);
            else done = dispatch_gather_w<TCG_F16>(b, n_chunks);
        }
    }
    if (!done) {
        if (x_dt == TCG_F32) done = dispatch_elem_w<TCG_F32>(a);
        else if (x_dt == TCG_BF16) done = dispatch_elem_w<TCG_BF16>(a);
        else done = dispatch_elem_w<TCG_F16>(a);
    }
    if (!done) {
        const unsigned grid = (unsigned)plan_grid(m->h_lane_tab, kBlock / kWave);
        if (d_w)
            hipLaunchKernelGGL(spmm_gather_generic_kernel<true>, dim3(grid), dim3(kBlock), 0, s, m->d_lane_tab,
                               m->d_seg_row, m->d_seg_ebeg, m->d_seg_dst, m->d_row_ptr, m->d_col_idx, d_w, d_X,
                               (int)x_dt, ldx, D, d_Y, (int)y_dt, ldy, partial, (int64_t)D, win_path,
                               m->win_h, tile_mask);
        else
            hipLaunchKernelGGL(spmm_gather_generic_kernel<false>, dim3(grid), dim3(kBlock), 0, s, m->d_lane_tab,
                               m->d_seg_row, m->d_seg_ebeg, m->d_seg_dst, m->d_row_ptr, m->d_col_idx, d_w, d_X,
                               (int)x_dt, ldx, D, d_Y, (int)y_dt, ldy, partial, (int64_t)D, win_path,
                               m->win_h, tile_mask);
    }
    TCG_TRY(launch_status("spmm_gather_kernel"));
    if (m->n_long > 0) {
        const int y_vec = (ldy & 3) == 0 && reinterpret_cast<uintptr_t>(d_Y) % (y_dt == TCG_F32 ? 16 : 8) == 0;
        const int32_t c4 = D / 4;
        if (D % 4 == 0 && c4 <= 4 && (c4 & (c4 - 1)) == 0) {   // measured: 164 -> 156 us at 16 columns, slower from 32 on
            int c4_log2 = 0;
            while ((1 << c4_log2) < c4) ++c4_log2;
            hipLaunchKernelGGL(spmm_reduce_long_wave_kernel, dim3((unsigned)ceil_div(m->n_long, kBlock / kWave)), dim3(kBlock),
                               0, s, m->n_long, m->d_long_row, m->d_long_slot_ptr, partial, (int64_t)D, c4_log2, d_Y,
                               (int)y_dt, ldy, win_path, m->win_h, tile_mask, y_vec);
        } else {
            hipLaunchKernelGGL(spmm_reduce_long_kernel, dim3((unsigned)m->n_long), dim3(D <= 64 ? kBlock / 2 : kBlock), 0, s, m->n_long,
                               m->d_long_row, m->d_long_slot_ptr, partial, (int64_t)D, D, d_Y, (int)y_dt, ldy, win_path,
                               m->win_h, tile_mask, y_vec);
        }
        TCG_TRY(launch_status("spmm_reduce_long_kernel"));
    }
    return TCG_OK;
}

}  // namespace tcg
