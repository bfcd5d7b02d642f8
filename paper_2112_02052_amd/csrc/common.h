// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>

#include "tcgnn.h"

namespace tcg {

constexpr int kWave = 64;            // gfx950 wavefront width
constexpr int kSegLen = 128;         // a row with more entries is split; the others are one segment
// Entries per segment ("slot") of a split row: half a kSegLen when X has so many rows that it cannot stay in the
// caches -- shorter slots cover narrower column ranges, which is what the column bands live on (1M-node graph:
// SpMM -6 %, SDDMM -4 %) -- and a whole one otherwise, where more slots only mean more partial rows (100k-node
// graph: +6 % the other way).
constexpr int kSlotShort = 64;
constexpr int64_t kSlotShortFromCols = 1 << 18;
inline int slot_length(int64_t n_cols) { return n_cols >= kSlotShortFromCols ? kSlotShort : kSegLen; }
constexpr int kGiantRow = 2048;      // up to this length a row fits one wavefront's registers; longer rows are listed
constexpr int kGiantChunk = 4096;    // apart in the plan, in pieces of this many entries (one workgroup per piece in
                                     // the row-wise kernels)
// Largest nnz the library takes: the kernels form entry positions up to a few thousand past the end of a row
// (look-ahead of the unrolled loops) before comparing them with it, and those must still fit int32.
constexpr int64_t kIndexLimit = (int64_t)INT32_MAX - (1 << 16);
constexpr float kDefaultMinReuse = 2.0f;
constexpr int kXcds = 8;              // accelerator dies of an MI355X; workgroup i is dispatched to die i % 8
constexpr int kPartialInitD = 128;   // the build reserves partial-sum scratch for feature widths up to this
constexpr int kTileMaxUnique = 512;  // AUTO never sends a window with more unique columns to the tile path
// Values of the per-window path flag: 0 = gather path; tile path with the window's edges kept in
// registers (at most kTileFewEdges of them, or more unique columns than kTileMaxUnique under a forced
// tile policy); tile path with the window's whole condensed adjacency built once in LDS.
constexpr uint8_t kTileFew = 1, kTileMany = 2;
constexpr int kTileFewEdges = 512;
// SpMM sends a class to the MFMA kernels only from this feature width on (measured crossovers).
constexpr int kTileMinWidthFew = 64, kTileMinWidthMany = 128;
// fp32 features on the tile path cost six MFMAs per product: SDDMM takes it from this mean reuse (stored
// entries per distinct column over the tile-path windows) on; measured crossover 2.5 - 3.5.
constexpr float kTileMinReuseF32Sddmm = 3.0f;

// Records the text of a failing HIP call for tcg_strerror (thread local).
void set_hip_error(hipError_t e, const char *what);
// Records the detail text that tcg_strerror appends to TCG_ESCRATCH (thread local).
void set_message(const char *text);

#define TCG_HIP(call)                                   \
    do {                                                \
        hipError_t e_ = (call);                         \
        if (e_ != hipSuccess) {                         \
            ::tcg::set_hip_error(e_, #call);            \
            return TCG_EHIP;                            \
        }                                               \
    } while (0)

#define TCG_TRY(call)                                   \
    do {                                                \
        int s_ = (call);                                \
        if (s_ != TCG_OK) return s_;                    \
    } while (0)

inline int launch_status(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_hip_error(e, what);
        return TCG_EHIP;
    }
    return TCG_OK;
}

// pool.hip: caching device allocator (blocks are reused across graph translations).
int pool_alloc(void **p, size_t bytes);
void pool_free(void *p);
void pool_release_all();

template <typename T>
int dev_alloc(T **p, int64_t count)
{
    if (count <= 0) count = 1;       // keep pointers valid for empty graphs
    void *q = nullptr;
    int st = pool_alloc(&q, static_cast<size_t>(count) * sizeof(T));
    *p = static_cast<T *>(q);
    return st;
}

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Gather-plan lookup: the segment that group `group` of workgroup blockIdx.x works on, or -1.
// The segment list is ordered by column band (see sgt.hip).  Workgroup i belongs to dispatch lane
// i % kXcds (the accelerator die it runs on).  lane_tab[kLaneTabStride * lane] holds {start, count} of
// the lane's first band, {start, count} of its second band, and {start, count} of the whole unbanded
// tail of the list (the same for all lanes).  A lane walks its two bands in workgroup-sized blocks,
// one band after the other, then takes every kXcds-th run of the unbanded tail.
constexpr int kLaneTabStride = 6;
constexpr int kTailRun = 32;         // segments per contiguous run of the unbanded tail (16 .. 64 measure alike,
                                     // 128 and more 2-5 % slower: shorter runs spread a stretch of long rows over the dies)
__device__ __forceinline__ int64_t plan_segment(const int32_t *__restrict__ lane_tab, int groups_per_block,
                                                int group)
{
    const int lane = blockIdx.x % kXcds;
    const int32_t *t = lane_tab + kLaneTabStride * lane;
    int64_t blk = blockIdx.x / kXcds;
    // One band after the other: interleaving them lets the rarely used columns evict the popular ones.
#pragma unroll
    for (int part = 0; part < 2; ++part) {
        const int64_t nb = ((int64_t)t[2 * part + 1] + groups_per_block - 1) / groups_per_block;
        if (blk < nb) {
            const int64_t i = blk * groups_per_block + group;
            return i < t[2 * part + 1] ? (int64_t)t[2 * part] + i : -1;
        }
        blk -= nb;
    }
    // Unbanded tail: runs of kTailRun consecutive segments (a few row windows, whose rows tend to share
    // neighbours) stay on one die; the runs are dealt out round-robin.
    const int run_blocks = kTailRun / groups_per_block > 0 ? kTailRun / groups_per_block : 1;
    const int64_t tb = ((blk / run_blocks) * kXcds + lane) * run_blocks + blk % run_blocks;
    const int64_t i = tb * groups_per_block + group;
    return i < t[5] ? (int64_t)t[4] + i : -1;
}

// seg_dst of a segment.  Below zero: a single-segment row, written straight to the result, and -1 - seg_dst is its
// length.  Otherwise a segment of a split row: the low kSegSlotBits bits are its slot (where its partial result
// goes), and the three bits above say how long it is when it is not the last segment of its row: 0 = the last
// one, else 16 << code entries (64 or 128).  The end of a segment's entries therefore needs a look at row_ptr
// only for the last segment of a split row -- one round trip less in the chain segment record -> column ids ->
// rows, which is most of a short row's time.
constexpr int kSegSlotBits = 28;
__host__ __device__ __forceinline__ int32_t segment_full_code(int slot_len) { return slot_len == 64 ? 2 : 3; }
__device__ __forceinline__ int32_t segment_slot(int32_t dst) { return dst & ((1 << kSegSlotBits) - 1); }
__device__ __forceinline__ int32_t segment_end(int32_t eb, int32_t dst, int32_t row, const int32_t *__restrict__ row_ptr)
{
    if (dst < 0) return eb - 1 - dst;
    const int32_t code = dst >> kSegSlotBits;
    return code ? eb + (16 << code) : row_ptr[row + 1];
}

// Host side of the same mapping: number of workgroups to launch for `groups_per_block`.
inline int64_t plan_grid(const int32_t *h_lane_tab, int groups_per_block)
{
    int64_t band_blocks = 0;
    for (int l = 0; l < kXcds; ++l) {
        const int32_t *t = h_lane_tab + kLaneTabStride * l;
        const int64_t nb = ((int64_t)t[1] + groups_per_block - 1) / groups_per_block +
                           ((int64_t)t[3] + groups_per_block - 1) / groups_per_block;
        band_blocks = nb > band_blocks ? nb : band_blocks;
    }
    const int64_t run_blocks = kTailRun / groups_per_block > 0 ? kTailRun / groups_per_block : 1;
    const int64_t tail_blocks = ((int64_t)h_lane_tab[5] + groups_per_block - 1) / groups_per_block;
    const int64_t tail_runs = (tail_blocks + run_blocks - 1) / run_blocks;
    return kXcds * (band_blocks + (tail_runs + kXcds - 1) / kXcds * run_blocks);
}

// Exclusive prefix sum of n int32 values on the device; out may alias in.  out has n + 1
// entries: out[n] is the total (sums are computed in int32; callers bound the total beforehand).
// A pooled device buffer that goes back to the pool when the scope ends.  The stream that used it is
// drained first (a no-op on the normal paths, which synchronise themselves; it matters when an error
// return leaves kernels in flight).
struct PoolBuf {
    void *p = nullptr;
    hipStream_t s = nullptr;
    ~PoolBuf()
    {
        if (!p) return;
        (void)hipStreamSynchronize(s);
        pool_free(p);
    }
};

// d_work: device scratch of scan_workspace_elems(n) int32.
int64_t scan_workspace_elems(int64_t n);
int exclusive_scan_i32(const int32_t *d_in, int32_t *d_out, int64_t n, int32_t *d_work, hipStream_t s);

}  // namespace tcg

struct tcg_meta;

namespace tcg {

// sgt.hip
int sgt_build_impl(tcg_meta *m, int validate, hipStream_t s);
int choose_paths(tcg_meta *m, tcg_policy policy, float min_reuse, hipStream_t s);
// Writes the per-window unique lists back to back (the exported col_to_row) into d_packed[total_unique].
int export_col_to_row(const tcg_meta *m, int32_t *d_packed, hipStream_t s);
int tile_stats(const tcg_meta *m, int32_t tile_w, int64_t *translated, int64_t *untranslated, hipStream_t s);

// spmm.hip / sddmm.hip / softmax.hip
int spmm_impl(tcg_meta *m, const void *d_X, tcg_dtype x_dt, int32_t D, int64_t ldx, const float *d_w,
              void *d_Y, tcg_dtype y_dt, int64_t ldy, bool no_alloc, hipStream_t s);
// Makes the plan's partial-sum scratch large enough for feature width D (allocates; an error while the
// stream is being captured).
int reserve_partial(tcg_meta *m, int32_t D, hipStream_t s);
// The library's static scratch array on the current device (resolved once per device).
int static_scratch(float **ptr, int64_t *capacity_elems);
int sddmm_impl(tcg_meta *m, const void *d_P, int64_t ldp, const void *d_X, int64_t ldx, tcg_dtype x_dt, int32_t D,
               float *d_out, hipStream_t s);

// attn.hip
int attention_impl(tcg_meta *m, const void *d_X, tcg_dtype x_dt, int32_t D, int64_t ldx, const float *d_rnorm, float beta,
                   float *d_scores, void *d_Y, tcg_dtype y_dt, int64_t ldy, hipStream_t s);
int row_rnorm_impl(int64_t n, const void *d_X, tcg_dtype x_dt, int32_t D, int64_t ldx, float eps, float *d_out,
                   hipStream_t s);
int row_unit_grad_impl(int64_t n, const void *d_X, tcg_dtype x_dt, int32_t D, int64_t ldx, const float *d_rnorm,
                       float scale, const float *d_G, int64_t ldg, float *d_dX, int64_t ldd, hipStream_t s);

// backward.hip
int row_softmax_backward_impl(const tcg_meta *m, const float *d_p, const float *d_dp, float *d_dv, hipStream_t s);
int csr_transpose_impl(int32_t n_rows, int32_t n_cols, int64_t nnz, const int32_t *d_row_ptr,
                       const int32_t *d_col_idx, int32_t *d_out_row_ptr, int32_t *d_out_col_idx, int32_t *d_perm,
                       hipStream_t s);
int edge_gather_impl(int64_t n, const int32_t *d_perm, const float *d_in, float *d_out, hipStream_t s);
// radix.hip: stable least-significant-digit radix sort (8 bits per pass) of (key, value) pairs by key, keys in
// [0, 2^bits) (never negative).  d_vals_in == nullptr stands for the values 0 .. n-1.  The number of pairs is
// n_max, or, when d_n is given, the smaller of n_max and the int32 at d_n (device memory; buffers and grids
// are sized by n_max).  The outputs must not overlap the inputs.  d_scratch: device memory of
// radix_sort_scratch_bytes(n_max) bytes (0 = n_max too large).  Asynchronous on s.
size_t radix_sort_scratch_bytes(int64_t n_max);
int radix_sort_pairs(const int32_t *d_keys_in, const int32_t *d_vals_in, int64_t n_max, const int32_t *d_n, int bits,
                     int32_t *d_keys_out, int32_t *d_vals_out, void *d_scratch, hipStream_t s);

// reorder.hip
int reorder_rows_impl(int32_t n, int64_t nnz, const int32_t *d_row_ptr, const int32_t *d_col_idx, uint64_t seed,
                      int32_t refine, int32_t *d_perm, hipStream_t s);
int csr_permute_impl(int32_t n, int64_t nnz, const int32_t *d_row_ptr, const int32_t *d_col_idx,
                     const int32_t *d_perm, int32_t *d_out_row_ptr, int32_t *d_out_col_idx, int32_t *d_edge_perm,
                     hipStream_t s);
int row_softmax_impl(const tcg_meta *m, const float *d_in, float *d_out, hipStream_t s);

// spmm_tile.hip: can the condensed-tile kernels take this operand?
bool tile_path_supports(tcg_dtype x_dt, int32_t D, int64_t ldx, const void *X);
bool spmm_tile_supports(tcg_dtype x_dt, int32_t D, int64_t ldx, const void *X, int32_t win_h);
bool sddmm_tile_supports(tcg_dtype x_dt, int32_t D, int64_t ld, const void *ptr);

inline int dtype_size(tcg_dtype t) { return t == TCG_F32 ? 4 : 2; }

}  // namespace tcg

// The metadata object behind the opaque C handle.
struct tcg_meta {
    int device = 0;
    int32_t n_rows = 0, n_cols = 0, win_h = 0, tile_w = 0;
    int64_t nnz = 0, n_win = 0, total_unique = 0, total_tiles = 0;

    const int32_t *d_row_ptr = nullptr;  // borrowed
    const int32_t *d_col_idx = nullptr;  // borrowed

    // Translated graph (Algorithm 1 outputs and the per-window unique lists).
    int32_t *d_win_partition = nullptr;   // [n_win]
    int32_t *d_win_unique_ptr = nullptr;  // [n_win + 1]
    int32_t *d_edge_to_col = nullptr;     // [nnz]
    int32_t *d_col_to_row = nullptr;      // [nnz] window w's list at offset row_ptr[w * win_h], U_w entries

    // Gather plan: every row is cut into segments of at most kSegLen edges.
    int64_t n_seg = 0, n_long = 0, n_slots = 0;
    int32_t *d_seg_row = nullptr;         // [n_seg] row of the segment
    int32_t *d_seg_ebeg = nullptr;        // [n_seg] first edge
    int32_t *d_seg_dst = nullptr;         // [n_seg] see segment_end(): partial-sum slot (+ kSegFull), or below zero: write
                                          //         the row directly (-1 - the row's length: a single-segment row)
    int32_t *d_long_row = nullptr;        // [n_long] rows with more than one segment
    int32_t *d_long_slot_ptr = nullptr;   // [n_long + 1] their slot ranges
    int32_t *d_long_ebeg = nullptr;       // [n_long] their first edge
    int32_t *d_long_len = nullptr;        // [n_long] their number of entries
    int32_t *d_gchunk_li = nullptr;       // [n_gchunks] the kGiantChunk-entry pieces of the rows beyond kGiantRow: position
    int32_t *d_gchunk_c = nullptr;        //             of the row in the four arrays above, and number of the piece
    int64_t n_gchunks = 0;                //             in its row (a row's pieces are consecutive)
    int32_t *d_lane_tab = nullptr;        // [kXcds x kLaneTabStride] see plan_segment() (inside the build's result block)
    int32_t h_lane_tab[6 * 8] = {0};      // host copy (sizes the gather grids, see plan_grid())
    float *d_partial = nullptr;           // [n_slots x D] scratch; reserved for D <= kPartialInitD, regrown on demand
    int64_t partial_elems = 0;
    float *d_partial_ml = nullptr;        // [n_slots x 2] (maximum, denominator) per split-row segment (tcg_attention);
                                          //               per piece of a very long row in the row softmax and its gradient
    bool partial_owned = false;          // true once regrown by tcg_spmm for a wider D (separate allocation)

    // Device allocations owned by this object (the pointers above and below are carved from them).
    void *owned[8] = {nullptr};
    int n_owned = 0;
    unsigned long long *d_counters = nullptr;   // [0] tiles, [1] tile-path windows, [2] their edges

    // Per-window path choice.
    tcg_policy policy = TCG_POLICY_AUTO;
    float min_reuse = 0.f;
    uint8_t *d_win_path = nullptr;        // [n_win] 1 = condensed-tile path
    int64_t n_tile_win = 0, nnz_tile = 0;   // windows on the tile path (both classes) and their edges
    int64_t n_tile_many = 0, max_unique_many = 0;   // class kTileMany: count, widest window
    int64_t unique_tile = 0;                        // distinct columns summed over the tile-path windows
};
