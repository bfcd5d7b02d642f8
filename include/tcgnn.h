/*
 * tcgnn.h -- C ABI of the MI355X (gfx950) neighbour-aggregation library.
 *
 * The library implements the hot path of TC-GNN (arxiv 2112.02052): the sparse graph
 * translation (SGT) of a CSR adjacency into per-row-window condensed column tiles, the
 * SpMM-like neighbour aggregation over the translated graph and the SDDMM-like edge feature
 * computation, plus the row-wise softmax that an attention-style layer puts between the two.
 *
 * General conventions
 *   - Every pointer whose name starts with d_ is DEVICE memory on the GPU that is current when
 *     the call is made; every pointer whose name starts with h_ is HOST memory.
 *   - Every function returns TCG_OK (0) or a negative tcg_status.  No C++ exception crosses
 *     this boundary.  tcg_strerror() describes a status; after TCG_EHIP it also carries the
 *     text of the failing HIP call (per thread).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All kernels are
 *     enqueued on it and the call returns without waiting, except tcg_sgt_build and
 *     tcg_sgt_set_policy, which wait for the stream because sizes must reach the host, and
 *     tcg_sgt_export to host memory; the calls that wait say so below and return TCG_ECAPTURE when the
 *     stream is being captured into a HIP graph.
 *   - Indices are int32; nnz (and with it the sum of window-unique columns) must be below 2^31 - 2^16
 *     (TCG_ERANGE otherwise, decided before any device work).
 *   - The caller owns every array it passes in.  The CSR arrays are BORROWED by the metadata
 *     object: they must stay alive and unchanged until tcg_sgt_free().
 *   - A tcg_meta may be used by one call at a time (calls on one stream are ordered and fine;
 *     concurrent calls on different streams with the same meta race on its scratch buffers).
 */
#ifndef TCGNN_H
#define TCGNN_H

#include <stdint.h>

#if defined(__GNUC__)
#define TCG_API __attribute__((visibility("default")))
#else
#define TCG_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tcg_meta tcg_meta; /* opaque; created by tcg_sgt_build, destroyed by tcg_sgt_free */

typedef enum { TCG_F32 = 0, TCG_BF16 = 1, TCG_F16 = 2 } tcg_dtype;

typedef enum {
    TCG_OK = 0,
    TCG_EINVAL = -1, /* null pointer, non-positive size, unsupported dtype, ld < D, misalignment */
    TCG_ECSR = -2,   /* CSR malformed: row_ptr[0] != 0, row_ptr not monotone, row_ptr[n] != nnz,
                        or a column index outside [0, n_cols)                                  */
    TCG_ERANGE = -3, /* a size does not fit the int32 index space                               */
    TCG_ENOMEM = -4, /* host or device allocation failed                                        */
    TCG_EHIP = -5,   /* a HIP runtime call or kernel launch failed                              */
    TCG_ESCRATCH = -6, /* a scratch buffer is too small and may not be (re)allocated in this call: the
                        static buffer of tcg_spmm_noalloc, or a plan's buffer while the stream is
                        being captured (tcg_strerror says which and by how much)                */
    TCG_ECAPTURE = -7 /* the call waits for the stream (sizes or data travel to the host) and the stream
                        is being captured into a HIP graph; refused before the stream is touched, so
                        the capture stays intact                                                */
} tcg_status;

/* Which kernel family a row window is executed by (see tcg_sgt_set_policy). */
typedef enum {
    TCG_POLICY_AUTO = 0,   /* per window: condensed-tile MFMA path when it pays, else row gather */
    TCG_POLICY_GATHER = 1, /* every window on the wavefront row-gather path                      */
    TCG_POLICY_TILE = 2    /* every non-empty window on the condensed-tile path (needs win_h 16) */
} tcg_policy;

/*
 * Sparse Graph Translation -- Algorithm 1 and section 4.1 of the paper.
 *
 * Splits the rows into windows of `window_h` consecutive rows (the last one may be shorter).
 * For each window: the ascending, duplicate-free list of the column ids of its edges
 * (col_to_row, the text's colToRow); win_partition[w] = ceil(U_w / tile_w) where U_w is that
 * list's length (0 for a window without edges); edge_to_col[e] = 0-based position of
 * col_idx[e] in its window's list.  Column ids inside a CSR row may come in any order and may
 * repeat (repeats share a condensed column and their values add up in tcg_spmm).
 *
 * The result is deterministic and equals the sequential algorithm bit for bit.  Alongside it
 * the call prepares the execution plan used by tcg_spmm / tcg_sddmm (row segments for the
 * gather path, the per-window path choice of TCG_POLICY_AUTO).
 *
 *   n_rows, n_cols  matrix shape (the paper's adjacency is square; nothing here requires it)
 *   nnz             number of stored entries
 *   d_row_ptr       device int32[n_rows + 1]   (nodePointer)  borrowed
 *   d_col_idx       device int32[nnz]          (edgeList)     borrowed
 *   window_h        rows per window  (TC_BLK_H; the paper uses 16)            >= 1
 *   tile_w          condensed columns per tile (TC_BLK_W; paper: 8 / 16)      >= 1
 *   validate        non-zero: check the CSR on the device first (TCG_ECSR on failure);
 *                   zero: the caller guarantees a well-formed CSR
 *   out             receives the metadata object; untouched on error
 * Blocks until the stream has finished the build.  For graphs of 2^20 stored entries and more, part of the work
 * runs on two streams of the library's own (default priority, ordered against `stream` by events), and in every
 * case sizes travel to the host: `stream` must not be
 * under HIP graph capture.  Builds that run at the same time on one device share those two streams and are
 * ordered against each other there.
 */
TCG_API int tcg_sgt_build(int32_t n_rows, int32_t n_cols, int64_t nnz,
                  const int32_t *d_row_ptr, const int32_t *d_col_idx,
                  int32_t window_h, int32_t tile_w, int validate,
                  void *stream, tcg_meta **out);

/* Sizes of the translated graph.  Any output pointer may be NULL.
 *   n_windows     ceil(n_rows / window_h)
 *   total_unique  U = sum over windows of U_w            (length of col_to_row)
 *   total_tiles   sum of win_partition
 *   nnz           as given to tcg_sgt_build                                                    */
TCG_API int tcg_sgt_sizes(const tcg_meta *meta, int64_t *n_windows, int64_t *total_unique,
                  int64_t *total_tiles, int64_t *nnz);

/*
 * How many tiles a window-by-window tiled kernel visits with and without the translation -- the quantity of
 * the paper's SGT-effectiveness study (section 5.2, the figure on the reduction of traversed blocks) -- for any
 * tile width (the paper: 8 for the aggregation, 16 for the edge features; section 4.3 recounts the blocks
 * for the second width from the same translated graph):
 *   tiles_translated    sum over windows of ceil(U_w / tile_w)
 *   tiles_untranslated  sum over windows of the number of tile_w-wide column blocks of the original matrix,
 *                       aligned at multiples of tile_w, that hold at least one stored entry of the window
 * Either output may be NULL.  Blocks until the stream has finished.
 */
TCG_API int tcg_sgt_tile_stats(tcg_meta *meta, int32_t tile_w, int64_t *tiles_translated,
                       int64_t *tiles_untranslated, void *stream);

/*
 * Copies the canonical metadata into caller-owned buffers (any of them may be NULL to skip):
 *   win_partition   int32[n_windows]
 *   win_unique_ptr  int32[n_windows + 1]   offsets of each window's list inside col_to_row
 *   edge_to_col     int32[nnz]             positionally aligned with col_idx
 *   col_to_row      int32[total_unique]
 * dst_on_device != 0: the four pointers are device memory and the copies are asynchronous on
 * `stream`; otherwise they are host memory and the call returns after the copies completed.
 */
TCG_API int tcg_sgt_export(const tcg_meta *meta, int32_t *win_partition, int32_t *win_unique_ptr,
                   int32_t *edge_to_col, int32_t *col_to_row, int dst_on_device, void *stream);

/*
 * Chooses which windows run on the condensed-tile (MFMA) path.  TCG_POLICY_AUTO (the state
 * after tcg_sgt_build) sends a window there when window_h == 16, it has at most 512 unique
 * columns and its neighbour reuse nnz_w / U_w is at least `min_reuse` (<= 0 selects the library
 * default, 2); when such windows hold less than 2 % of the stored entries, none is sent there (a
 * launch that visits every window would cost more than it saves).  The flag says where a window
 * may go; a call takes the tile path only when its
 * operands can be read in 16-byte pieces (else it gathers), and under TCG_POLICY_AUTO narrow
 * features are gathered as well: tcg_spmm sends windows of at most 512 entries to the tile kernels
 * from D >= 64 and windows with more entries from D >= 128, tcg_sddmm uses them at every width for
 * bf16/f16 and, for fp32, from D >= 64 when the tile-path windows hold at least 3 entries per distinct
 * column on average (measured crossovers).  bf16/f16 features feed the MFMA units
 * directly (products of rounded edge values: the 1e-2 tolerance class); fp32 features are split
 * exactly into three bf16 values each and the six leading partial products are accumulated in fp32,
 * which keeps fp32 accuracy (D a multiple of 4, at most 1024 for tcg_spmm and 256 for tcg_sddmm).
 * TCG_POLICY_TILE sends every non-empty window to the tile kernels at any width they support.
 * Blocks until the stream has finished.  Returns TCG_EINVAL for TCG_POLICY_TILE when
 * window_h != 16.
 */
TCG_API int tcg_sgt_set_policy(tcg_meta *meta, tcg_policy policy, float min_reuse, void *stream);

/* Plan statistics.  Any output pointer may be NULL.
 *   n_tile_windows  windows currently assigned to the condensed-tile path
 *   nnz_tile        stored entries inside those windows
 *   n_segments      row segments of the gather plan
 *   n_long_rows     rows split over several segments                                           */
TCG_API int tcg_sgt_plan_stats(const tcg_meta *meta, int64_t *n_tile_windows, int64_t *nnz_tile,
                       int64_t *n_segments, int64_t *n_long_rows);

/*
 * Neighbour aggregation -- Equation 1 and Algorithm 2 of the paper:  Y = (w (.) A) X.
 *   Y[i][d] = sum over the stored entries e of row i of  w[e] * X[col_idx[e]][d],  fp32
 *   accumulation, Y overwritten (rows without entries become 0).
 *   d_X    device, row-major [n_cols x D], leading dimension ldx (elements), type x_dt
 *   d_w    device float[nnz] edge values in CSR order, or NULL for all ones
 *   d_Y    device, row-major [n_rows x D], leading dimension ldy (elements), type y_dt
 * D >= 1; ldx, ldy >= D.  Any D works; rows whose byte length and stride are multiples of 16
 * (and a 16-byte aligned base) take the vectorised kernels.  X and Y must not overlap.
 * The partial sums of rows split over several segments go to a scratch buffer reserved by
 * tcg_sgt_build for D <= 128; the first call with a wider D waits for the stream and reallocates (and
 * keeps) it -- while the stream is being captured into a HIP graph that is refused with TCG_ESCRATCH:
 * call tcg_sgt_reserve beforehand.  Apart from that the call neither allocates nor synchronises.
 * Non-finite features: on the row-gather path a NaN or infinity in X[j] reaches exactly the rows with
 * an entry in column j.  On the condensed-tile path it reaches every row of every window whose column
 * list contains j (0 x inf inside the matrix unit; inf - inf in the exact split of fp32 features), and
 * an entry (i, j) stored more than 256 times with unit values is rounded to bf16 there.
 * TCG_POLICY_GATHER gives the strict behaviour for all windows.
 */
TCG_API int tcg_spmm(tcg_meta *meta, const void *d_X, tcg_dtype x_dt, int32_t D, int64_t ldx,
             const float *d_w, void *d_Y, tcg_dtype y_dt, int64_t ldy, void *stream);

/*
 * tcg_spmm for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc).  Same arguments, same kernels and bit-identical results; the
 * partial sums of split rows go to a 64 MiB device array that is part of the library's code object
 * (one copy per GPU, held until the process ends) instead of the plan's buffer.  The call allocates
 * nothing and does not synchronise.  Limit: (number of segments of split rows) x D x 4 bytes <= 64 MiB;
 * beyond it the call does nothing and returns TCG_ESCRATCH (tcg_strerror gives both sizes).  All calls
 * on one GPU share the array: calls that overlap in time on one GPU (different streams or threads) race,
 * also with different plans.  Nothing in it needs clearing between calls (every partial row is
 * written in full before it is read).
 */
TCG_API int tcg_spmm_noalloc(tcg_meta *meta, const void *d_X, tcg_dtype x_dt, int32_t D, int64_t ldx,
                     const float *d_w, void *d_Y, tcg_dtype y_dt, int64_t ldy, void *stream);

/*
 * Grows the plan's partial-sum scratch for feature widths up to max_D now, so that later tcg_spmm /
 * tcg_attention calls with D <= max_D never allocate (needed before capturing them with D > 128).
 * May wait for the stream.
 */
TCG_API int tcg_sgt_reserve(tcg_meta *meta, int32_t max_D, void *stream);

/*
 * Edge feature computation -- Equation 2 and Algorithm 3 of the paper:
 *   d_out[e] = < X[i], X[col_idx[e]] >  for every stored entry e of row i, fp32 accumulation,
 *   written in CSR (edgeList) order.  Needs a row of X for every row and every column id:
 *   X is [max(n_rows, n_cols) x D].
 */
TCG_API int tcg_sddmm(tcg_meta *meta, const void *d_X, tcg_dtype x_dt, int32_t D, int64_t ldx,
              float *d_out, void *stream);

/*
 * Equation 2 with two dense operands:  d_out[e] = < P[i], Q[col_idx[e]] >  for every stored entry e of
 * row i.  tcg_sddmm is the case P = Q = X.  This is the edge-value gradient of tcg_spmm
 * (dw = tcg_sddmm_pq(P = dY, Q = X)).  P is [n_rows x D] with leading dimension ldp, Q is [n_cols x D]
 * with leading dimension ldq; both have type x_dt.
 */
TCG_API int tcg_sddmm_pq(tcg_meta *meta, const void *d_P, int64_t ldp, const void *d_Q, int64_t ldq,
                 tcg_dtype x_dt, int32_t D, float *d_out, void *stream);

/*
 * Row-wise softmax over the stored entries of each row (the normalisation of the
 * attention-style workload; not part of the paper's method):
 *   d_out[e] = exp(d_in[e] - m_i) / sum_{e' in row i} exp(d_in[e'] - m_i),  m_i = row maximum.
 * In-place (d_out == d_in) is allowed.  Rows of more than 2,048 entries are worked on in pieces whose partial
 * results pass through the metadata object's scratch (one call at a time per object, see the conventions above).
 */
TCG_API int tcg_row_softmax(const tcg_meta *meta, const float *d_in, float *d_out, void *stream);

/*
 * Fused attention-style aggregation (the SDDMM -> row softmax -> SpMM chain of the paper's AGNN
 * workload in one pass over the graph):
 *   Y[i] = sum over the stored entries e of row i of  softmax_i(< X[i], X[col_idx[.]] >)_e * X[col_idx[e]]
 * Every neighbour row is gathered once; the scores stay in registers (online softmax).  Rows without
 * entries give 0.  d_scores: NULL, or device float[nnz] that receives the raw scores <x_i, x_j> in CSR
 * order (what tcg_sddmm would return; the backward pass needs them).  Needs rows of X whose byte
 * length and stride are multiples of 16 bytes, a 16-byte aligned base and D * sizeof(element) <= 2048
 * (TCG_EINVAL otherwise).  Always runs on the gather path.  X: [max(n_rows, n_cols) x D].
 */
TCG_API int tcg_attention(tcg_meta *meta, const void *d_X, tcg_dtype x_dt, int32_t D, int64_t ldx,
                  float *d_scores, void *d_Y, tcg_dtype y_dt, int64_t ldy, void *stream);

/*
 * The fused aggregation with cosine-style scores, as the attention layer of the paper's AGNN model uses them
 * (the evaluation section names the model, 4 layers of 32 hidden features; the paper leaves its normalisation
 * open -- this is the published AGNN propagation):
 *   c_e = d_rnorm[i] * d_rnorm[j] * < X[i], X[j] >      for the stored entry e = (i, j)
 *   Y[i] = sum over the stored entries e of row i of  softmax_i(beta * c)_e * X[j]
 * With d_rnorm[v] = 1 / |X[v]| (tcg_row_rnorm) c_e is the cosine of the two feature rows; X itself, not a
 * normalised copy, is gathered once per entry for score and aggregation alike.  d_scores: NULL, or device
 * float[nnz] that receives c (without beta) in CSR order.  d_rnorm: device float[max(n_rows, n_cols)].
 * Same operand requirements as tcg_attention.
 */
TCG_API int tcg_attention_cos(tcg_meta *meta, const void *d_X, tcg_dtype x_dt, int32_t D, int64_t ldx,
                      const float *d_rnorm, float beta, float *d_scores, void *d_Y, tcg_dtype y_dt, int64_t ldy,
                      void *stream);

/* d_out[i] = 1 / max(|X[i]|_2, eps) for the n rows of X (row-major, leading dimension ldx, type x_dt); eps > 0. */
TCG_API int tcg_row_rnorm(int64_t n, const void *d_X, tcg_dtype x_dt, int32_t D, int64_t ldx, float eps,
                  float *d_out, void *stream);

/*
 * The way back through the row normalisation xn[i] = d_rnorm[i] * X[i] of the scaled-cosine scores (the attention
 * layer of the paper's second benchmark model, evaluation section): with d_G the gradient with respect to xn,
 *   d_dX[i] += scale * d_rnorm[i] * (d_G[i] - xn[i] * <d_G[i], xn[i]>)        for the n rows,
 * which is scale times the derivative of x / |x| applied to d_G[i] when d_rnorm[i] = 1 / |X[i]| (tcg_row_rnorm);
 * for a row clamped by eps there the second term fades with xn[i].  d_G and d_dX are fp32, row-major with leading
 * dimensions ldg, ldd >= D; d_dX is accumulated into and must not overlap d_G.  Errors: TCG_EINVAL.
 */
TCG_API int tcg_row_unit_grad(int64_t n, const void *d_X, tcg_dtype x_dt, int32_t D, int64_t ldx, const float *d_rnorm,
                      float scale, const float *d_G, int64_t ldg, float *d_dX, int64_t ldd, void *stream);

/*
 * Gradient of tcg_row_softmax:  d_dv[e] = d_p[e] * (d_dp[e] - sum over the row of d_p * d_dp), where d_p is
 * the softmax output and d_dp the gradient with respect to it.  In-place (d_dv == d_dp) is allowed.
 */
TCG_API int tcg_row_softmax_backward(const tcg_meta *meta, const float *d_p, const float *d_dp, float *d_dv,
                             void *stream);

/*
 * CSR structure of the transpose (needed for dX = (w (.) A)^T dY when A is not symmetric: translate the
 * transpose with tcg_sgt_build and run tcg_spmm on it with the permuted edge values).
 *   d_out_row_ptr  device int32[n_cols + 1]
 *   d_out_col_idx  device int32[nnz]   ascending inside every row of the transpose when the input has no
 *                                      repeated entries (entries keep the input's row-major order)
 *   d_perm         device int32[nnz]   entry k of the transpose is entry d_perm[k] of the input
 * The result is unique and deterministic (stable sort by column).  Needs a well-formed CSR.
 * Blocks until the stream has finished (temporary buffers are released on return).
 */
TCG_API int tcg_csr_transpose(int32_t n_rows, int32_t n_cols, int64_t nnz, const int32_t *d_row_ptr,
                      const int32_t *d_col_idx, int32_t *d_out_row_ptr, int32_t *d_out_col_idx,
                      int32_t *d_perm, void *stream);

/* d_out[k] = d_in[d_perm[k]] for k < n: edge values in the order of the transposed structure.
 * d_out must not overlap d_in.                                                                        */
TCG_API int tcg_edge_gather(int64_t n, const int32_t *d_perm, const float *d_in, float *d_out, void *stream);

/* Row clustering before SGT.  The paper's related-work section calls row reordering orthogonal and
 * complementary to SGT and names no algorithm; this is a cheap deterministic heuristic for graphs whose
 * labelling scatters the members of a community (SGT only pays off when the rows of a window share
 * neighbours).  For a square n x n pattern (nodes = rows = columns):
 *   hash(v) = splitmix64 of (seed, v), nodes compared by (hash, id);
 *   parent(v) = the smallest node of {v} + N(v);  root(v) = the fixed point of v -> parent(v);
 *   label = root, then `refine` synchronous rounds of "most frequent label among the first 128 stored
 *   neighbours" (ties to the smallest label id, rows without entries keep theirs);
 *   d_perm[new] = old: the nodes sorted by (label, parent, id).
 *   d_row_ptr   device int32[n + 1], d_col_idx device int32[nnz]   the pattern (borrowed)
 *   refine      >= 0                   number of refinement rounds (2 is a good default)
 *   d_perm      device int32[n]        result
 * The result is deterministic.  Returns TCG_ECSR for a malformed pattern or a column outside [0, n).
 * Blocks until the stream has finished (temporary buffers are released on return).                   */
TCG_API int tcg_reorder_rows(int32_t n, int64_t nnz, const int32_t *d_row_ptr, const int32_t *d_col_idx,
                     uint64_t seed, int32_t refine, int32_t *d_perm, void *stream);

/* Symmetric permutation of a square CSR pattern: row i of the result is row d_perm[i] of the input and
 * every column id c becomes the new position of node c.  Entries keep their order inside a row.
 *   d_perm          device int32[n]       new -> old, a permutation of 0 .. n-1 (checked: TCG_EINVAL)
 *   d_out_row_ptr   device int32[n + 1], d_out_col_idx device int32[nnz]   the result
 *   d_edge_perm     device int32[nnz] or NULL   entry k of the result is entry d_edge_perm[k] of the input
 *                                               (edge values follow with tcg_edge_gather)
 * Features and outputs follow the same relabelling: X'[i] = X[d_perm[i]], Y'[i] = Y[d_perm[i]].
 * Blocks until the stream has finished.                                                               */
TCG_API int tcg_csr_permute(int32_t n, int64_t nnz, const int32_t *d_row_ptr, const int32_t *d_col_idx,
                    const int32_t *d_perm, int32_t *d_out_row_ptr, int32_t *d_out_col_idx,
                    int32_t *d_edge_perm, void *stream);

/*
 * Row clustering, relabelling and translation in one call, for graphs whose labelling scatters the members of
 * a community (the paper's related-work section calls row reordering orthogonal and complementary to SGT):
 * tcg_reorder_rows -> tcg_csr_permute -> tcg_sgt_build on a square n x n pattern.
 *   d_perm          device int32[n]      out: new -> old, the relabelling
 *   d_out_row_ptr   device int32[n + 1]  out: the relabelled pattern; BORROWED by the metadata object like the
 *   d_out_col_idx   device int32[nnz]         CSR arrays of tcg_sgt_build (keep them alive until tcg_sgt_free)
 *   d_edge_perm     device int32[nnz] or NULL  out: entry k of the relabelled pattern is entry d_edge_perm[k] of
 *                                              the input (edge values follow with tcg_edge_gather)
 * The metadata object describes the relabelled graph: features go in as X'[i] = X[d_perm[i]], results come out
 * as Y'[i] = Y[d_perm[i]], edge outputs in the relabelled entry order.  Returns TCG_ECSR for a malformed pattern.
 * Blocks until the stream has finished.
 */
TCG_API int tcg_sgt_build_clustered(int32_t n, int64_t nnz, const int32_t *d_row_ptr, const int32_t *d_col_idx,
                            int32_t window_h, int32_t tile_w, uint64_t seed, int32_t refine, void *stream,
                            int32_t *d_perm, int32_t *d_out_row_ptr, int32_t *d_out_col_idx,
                            int32_t *d_edge_perm, tcg_meta **out);

/* Releases the metadata object and every device buffer it owns (NULL is a no-op).  The caller
 * must make sure no kernel using it is still running (its buffers go back to the library's cache
 * and may be handed to the next tcg_sgt_build).                                         */
TCG_API void tcg_sgt_free(tcg_meta *meta);

/* The library keeps device blocks it no longer needs (temporaries of tcg_sgt_build, buffers of freed
 * metadata objects) and reuses them for later calls, because allocating them costs more than the
 * translation itself.  This call hands every cached block back to the driver; blocks of live
 * metadata objects are not touched.                                                            */
TCG_API void tcg_release_cached_memory(void);

/* Text for a status code; valid until the calling thread's next library call.                  */
TCG_API const char *tcg_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* TCGNN_H */
