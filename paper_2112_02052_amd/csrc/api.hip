// The C ABI (include/tcgnn.h): argument checks, object lifetime, export, error text.
#include "common.h"

#include <stdio.h>
#include <string.h>

#include <new>

namespace tcg {

static thread_local char g_hip_msg[256] = "";
static thread_local char g_msg[320] = "";

static thread_local char g_detail[320] = "";

void set_message(const char *text) { snprintf(g_detail, sizeof(g_detail), "%s", text); }

void set_hip_error(hipError_t e, const char *what)
{
    snprintf(g_hip_msg, sizeof(g_hip_msg), "%s: %s", what, hipGetErrorString(e));
}

// The calls that wait for the stream cannot run while it is being captured into a graph: they say so before
// they touch it, which leaves the capture intact.
static int refuse_capture(void *stream, const char *name)
{
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(static_cast<hipStream_t>(stream), &cap) != hipSuccess) {
        (void)hipGetLastError();
        return TCG_OK;
    }
    if (cap == hipStreamCaptureStatusNone) return TCG_OK;
    char msg[200];
    snprintf(msg, sizeof(msg), "%s waits for the stream, which is being captured into a HIP graph", name);
    set_message(msg);
    return TCG_ECAPTURE;
}

static void free_meta(tcg_meta *m)
{
    if (!m) return;
    for (int i = 0; i < m->n_owned; ++i)
        if (m->owned[i]) pool_free(m->owned[i]);
    if (m->partial_owned && m->d_partial) pool_free(m->d_partial);
    delete m;
}

}  // namespace tcg

using namespace tcg;

extern "C" {

int tcg_sgt_build(int32_t n_rows, int32_t n_cols, int64_t nnz, const int32_t *d_row_ptr,
                  const int32_t *d_col_idx, int32_t window_h, int32_t tile_w, int validate, void *stream,
                  tcg_meta **out)
{
    if (!out || !d_row_ptr || n_rows < 0 || n_cols < 0 || nnz < 0 || window_h < 1 || tile_w < 1)
        return TCG_EINVAL;
    if (nnz > 0 && !d_col_idx) return TCG_EINVAL;
    if (nnz >= kIndexLimit || (int64_t)n_rows + 1 >= (int64_t)INT32_MAX) return TCG_ERANGE;
    TCG_TRY(refuse_capture(stream, "tcg_sgt_build"));
    tcg_meta *m = new (std::nothrow) tcg_meta();
    if (!m) return TCG_ENOMEM;
    if (hipGetDevice(&m->device) != hipSuccess) {
        delete m;
        set_hip_error(hipGetLastError(), "hipGetDevice");
        return TCG_EHIP;
    }
    // Set-up for tcg_spmm_noalloc: this device's address of the static scratch array is looked up here,
    // so that the call itself has nothing left to resolve.
    if (int st = static_scratch(nullptr, nullptr); st != TCG_OK) {
        delete m;
        return st;
    }
    m->n_rows = n_rows;
    m->n_cols = n_cols;
    m->nnz = nnz;
    m->win_h = window_h;
    m->tile_w = tile_w;
    m->n_win = ceil_div(n_rows, window_h);
    m->d_row_ptr = d_row_ptr;
    m->d_col_idx = d_col_idx;
    int st = sgt_build_impl(m, validate, static_cast<hipStream_t>(stream));
    if (st != TCG_OK) {
        (void)hipStreamSynchronize(static_cast<hipStream_t>(stream));
        free_meta(m);
        return st;
    }
    *out = m;
    return TCG_OK;
}

int tcg_sgt_build_clustered(int32_t n, int64_t nnz, const int32_t *d_row_ptr, const int32_t *d_col_idx,
                            int32_t window_h, int32_t tile_w, uint64_t seed, int32_t refine, void *stream,
                            int32_t *d_perm, int32_t *d_out_row_ptr, int32_t *d_out_col_idx, int32_t *d_edge_perm,
                            tcg_meta **out)
{
    if (!out || !d_row_ptr || !d_out_row_ptr || n < 0 || nnz < 0 || refine < 0 || window_h < 1 || tile_w < 1)
        return TCG_EINVAL;
    if (n > 0 && !d_perm) return TCG_EINVAL;
    if (nnz > 0 && (!d_col_idx || !d_out_col_idx)) return TCG_EINVAL;
    if (nnz >= kIndexLimit || (int64_t)n + 1 >= (int64_t)INT32_MAX) return TCG_ERANGE;
    TCG_TRY(refuse_capture(stream, "tcg_sgt_build_clustered"));
    hipStream_t s = static_cast<hipStream_t>(stream);
    // the clustering validates the pattern (TCG_ECSR), so the translation need not do it again
    TCG_TRY(reorder_rows_impl(n, nnz, d_row_ptr, d_col_idx, seed, refine, d_perm, s));
    TCG_TRY(csr_permute_impl(n, nnz, d_row_ptr, d_col_idx, d_perm, d_out_row_ptr, d_out_col_idx, d_edge_perm, s));
    return tcg_sgt_build(n, n, nnz, d_out_row_ptr, d_out_col_idx, window_h, tile_w, 0, stream, out);
}

int tcg_sgt_sizes(const tcg_meta *meta, int64_t *n_windows, int64_t *total_unique, int64_t *total_tiles,
                  int64_t *nnz)
{
    if (!meta) return TCG_EINVAL;
    if (n_windows) *n_windows = meta->n_win;
    if (total_unique) *total_unique = meta->total_unique;
    if (total_tiles) *total_tiles = meta->total_tiles;
    if (nnz) *nnz = meta->nnz;
    return TCG_OK;
}

int tcg_sgt_export(const tcg_meta *meta, int32_t *win_partition, int32_t *win_unique_ptr, int32_t *edge_to_col,
                   int32_t *col_to_row, int dst_on_device, void *stream)
{
    if (!meta) return TCG_EINVAL;
    if (!dst_on_device) TCG_TRY(refuse_capture(stream, "tcg_sgt_export to host memory"));
    hipStream_t s = static_cast<hipStream_t>(stream);
    const hipMemcpyKind kind = dst_on_device ? hipMemcpyDeviceToDevice : hipMemcpyDeviceToHost;
    struct Item { void *dst; const void *src; int64_t count; };
    const Item items[] = {{win_partition, meta->d_win_partition, meta->n_win},
                          {win_unique_ptr, meta->d_win_unique_ptr, meta->n_win + 1},
                          {edge_to_col, meta->d_edge_to_col, meta->nnz}};
    for (const Item &it : items)
        if (it.dst && it.count > 0)
            TCG_HIP(hipMemcpyAsync(it.dst, it.src, (size_t)it.count * sizeof(int32_t), kind, s));
    // The library keeps every window's list at the window's edge offset; the exported form is packed.
    PoolBuf staging;
    staging.s = s;
    if (col_to_row && meta->total_unique > 0) {
        int32_t *packed = col_to_row;
        if (!dst_on_device) {
            TCG_TRY(pool_alloc(&staging.p, (size_t)meta->total_unique * sizeof(int32_t)));
            packed = static_cast<int32_t *>(staging.p);
        }
        TCG_TRY(export_col_to_row(meta, packed, s));
        if (!dst_on_device)
            TCG_HIP(hipMemcpyAsync(col_to_row, packed, (size_t)meta->total_unique * sizeof(int32_t), kind, s));
    }
    if (!dst_on_device) TCG_HIP(hipStreamSynchronize(s));
    return TCG_OK;
}

int tcg_sgt_tile_stats(tcg_meta *meta, int32_t tile_w, int64_t *tiles_translated, int64_t *tiles_untranslated,
                       void *stream)
{
    if (!meta || tile_w < 1) return TCG_EINVAL;
    TCG_TRY(refuse_capture(stream, "tcg_sgt_tile_stats"));
    return tile_stats(meta, tile_w, tiles_translated, tiles_untranslated, static_cast<hipStream_t>(stream));
}

int tcg_sgt_set_policy(tcg_meta *meta, tcg_policy policy, float min_reuse, void *stream)
{
    if (!meta) return TCG_EINVAL;
    if (policy != TCG_POLICY_AUTO && policy != TCG_POLICY_GATHER && policy != TCG_POLICY_TILE) return TCG_EINVAL;
    TCG_TRY(refuse_capture(stream, "tcg_sgt_set_policy"));
    return choose_paths(meta, policy, min_reuse, static_cast<hipStream_t>(stream));
}

int tcg_sgt_plan_stats(const tcg_meta *meta, int64_t *n_tile_windows, int64_t *nnz_tile, int64_t *n_segments,
                       int64_t *n_long_rows)
{
    if (!meta) return TCG_EINVAL;
    if (n_tile_windows) *n_tile_windows = meta->n_tile_win;
    if (nnz_tile) *nnz_tile = meta->nnz_tile;
    if (n_segments) *n_segments = meta->n_seg;
    if (n_long_rows) *n_long_rows = meta->n_long;
    return TCG_OK;
}

static bool dtype_ok(int dt) { return dt == TCG_F32 || dt == TCG_BF16 || dt == TCG_F16; }

int tcg_spmm(tcg_meta *meta, const void *d_X, tcg_dtype x_dt, int32_t D, int64_t ldx, const float *d_w,
             void *d_Y, tcg_dtype y_dt, int64_t ldy, void *stream)
{
    if (!meta || D < 1 || ldx < D || ldy < D || !dtype_ok(x_dt) || !dtype_ok(y_dt)) return TCG_EINVAL;
    if ((!d_X && meta->nnz > 0) || (!d_Y && meta->n_rows > 0)) return TCG_EINVAL;
    if ((reinterpret_cast<uintptr_t>(d_X) % dtype_size(x_dt)) || (reinterpret_cast<uintptr_t>(d_Y) % dtype_size(y_dt)))
        return TCG_EINVAL;
    return spmm_impl(meta, d_X, x_dt, D, ldx, d_w, d_Y, y_dt, ldy, false, static_cast<hipStream_t>(stream));
}

int tcg_spmm_noalloc(tcg_meta *meta, const void *d_X, tcg_dtype x_dt, int32_t D, int64_t ldx, const float *d_w,
                     void *d_Y, tcg_dtype y_dt, int64_t ldy, void *stream)
{
    if (!meta || D < 1 || ldx < D || ldy < D || !dtype_ok(x_dt) || !dtype_ok(y_dt)) return TCG_EINVAL;
    if ((!d_X && meta->nnz > 0) || (!d_Y && meta->n_rows > 0)) return TCG_EINVAL;
    if ((reinterpret_cast<uintptr_t>(d_X) % dtype_size(x_dt)) || (reinterpret_cast<uintptr_t>(d_Y) % dtype_size(y_dt)))
        return TCG_EINVAL;
    return spmm_impl(meta, d_X, x_dt, D, ldx, d_w, d_Y, y_dt, ldy, true, static_cast<hipStream_t>(stream));
}

int tcg_sgt_reserve(tcg_meta *meta, int32_t max_D, void *stream)
{
    if (!meta || max_D < 1) return TCG_EINVAL;
    return reserve_partial(meta, max_D, static_cast<hipStream_t>(stream));
}

int tcg_sddmm(tcg_meta *meta, const void *d_X, tcg_dtype x_dt, int32_t D, int64_t ldx, float *d_out,
              void *stream)
{
    if (!meta || D < 1 || ldx < D || !dtype_ok(x_dt)) return TCG_EINVAL;
    if (meta->nnz > 0 && (!d_X || !d_out)) return TCG_EINVAL;
    if (reinterpret_cast<uintptr_t>(d_X) % dtype_size(x_dt)) return TCG_EINVAL;
    return sddmm_impl(meta, d_X, ldx, d_X, ldx, x_dt, D, d_out, static_cast<hipStream_t>(stream));
}

int tcg_sddmm_pq(tcg_meta *meta, const void *d_P, int64_t ldp, const void *d_Q, int64_t ldq, tcg_dtype x_dt,
                 int32_t D, float *d_out, void *stream)
{
    if (!meta || D < 1 || ldp < D || ldq < D || !dtype_ok(x_dt)) return TCG_EINVAL;
    if (meta->nnz > 0 && (!d_P || !d_Q || !d_out)) return TCG_EINVAL;
    if ((reinterpret_cast<uintptr_t>(d_P) % dtype_size(x_dt)) || (reinterpret_cast<uintptr_t>(d_Q) % dtype_size(x_dt)))
        return TCG_EINVAL;
    return sddmm_impl(meta, d_P, ldp, d_Q, ldq, x_dt, D, d_out, static_cast<hipStream_t>(stream));
}

int tcg_attention(tcg_meta *meta, const void *d_X, tcg_dtype x_dt, int32_t D, int64_t ldx, float *d_scores, void *d_Y,
                  tcg_dtype y_dt, int64_t ldy, void *stream)
{
    if (!meta || D < 1 || ldx < D || ldy < D || !dtype_ok(x_dt) || !dtype_ok(y_dt)) return TCG_EINVAL;
    if ((!d_X && meta->nnz > 0) || (!d_Y && meta->n_rows > 0)) return TCG_EINVAL;
    if ((reinterpret_cast<uintptr_t>(d_Y) % dtype_size(y_dt))) return TCG_EINVAL;
    return attention_impl(meta, d_X, x_dt, D, ldx, nullptr, 1.f, d_scores, d_Y, y_dt, ldy, static_cast<hipStream_t>(stream));
}

int tcg_attention_cos(tcg_meta *meta, const void *d_X, tcg_dtype x_dt, int32_t D, int64_t ldx, const float *d_rnorm,
                      float beta, float *d_scores, void *d_Y, tcg_dtype y_dt, int64_t ldy, void *stream)
{
    if (!meta || D < 1 || ldx < D || ldy < D || !dtype_ok(x_dt) || !dtype_ok(y_dt)) return TCG_EINVAL;
    if ((!d_X && meta->nnz > 0) || (!d_Y && meta->n_rows > 0) || (!d_rnorm && meta->n_rows > 0)) return TCG_EINVAL;
    if ((reinterpret_cast<uintptr_t>(d_Y) % dtype_size(y_dt))) return TCG_EINVAL;
    return attention_impl(meta, d_X, x_dt, D, ldx, d_rnorm, beta, d_scores, d_Y, y_dt, ldy,
                          static_cast<hipStream_t>(stream));
}

int tcg_row_rnorm(int64_t n, const void *d_X, tcg_dtype x_dt, int32_t D, int64_t ldx, float eps, float *d_out, void *stream)
{
    if (n < 0 || D < 1 || ldx < D || !dtype_ok(x_dt) || !(eps > 0.f)) return TCG_EINVAL;
    if (n > 0 && (!d_X || !d_out)) return TCG_EINVAL;
    if (reinterpret_cast<uintptr_t>(d_X) % dtype_size(x_dt)) return TCG_EINVAL;
    return row_rnorm_impl(n, d_X, x_dt, D, ldx, eps, d_out, static_cast<hipStream_t>(stream));
}

int tcg_row_unit_grad(int64_t n, const void *d_X, tcg_dtype x_dt, int32_t D, int64_t ldx, const float *d_rnorm,
                      float scale, const float *d_G, int64_t ldg, float *d_dX, int64_t ldd, void *stream)
{
    if (n < 0 || D < 1 || ldx < D || ldg < D || ldd < D || !dtype_ok(x_dt)) return TCG_EINVAL;
    if (n > 0 && (!d_X || !d_rnorm || !d_G || !d_dX)) return TCG_EINVAL;
    if (reinterpret_cast<uintptr_t>(d_X) % dtype_size(x_dt)) return TCG_EINVAL;
    return row_unit_grad_impl(n, d_X, x_dt, D, ldx, d_rnorm, scale, d_G, ldg, d_dX, ldd, static_cast<hipStream_t>(stream));
}

int tcg_row_softmax_backward(const tcg_meta *meta, const float *d_p, const float *d_dp, float *d_dv, void *stream)
{
    if (!meta) return TCG_EINVAL;
    if (meta->nnz > 0 && (!d_p || !d_dp || !d_dv)) return TCG_EINVAL;
    return row_softmax_backward_impl(meta, d_p, d_dp, d_dv, static_cast<hipStream_t>(stream));
}

int tcg_csr_transpose(int32_t n_rows, int32_t n_cols, int64_t nnz, const int32_t *d_row_ptr,
                      const int32_t *d_col_idx, int32_t *d_out_row_ptr, int32_t *d_out_col_idx, int32_t *d_perm,
                      void *stream)
{
    if (n_rows < 0 || n_cols < 0 || nnz < 0 || !d_row_ptr || !d_out_row_ptr) return TCG_EINVAL;
    if (nnz > 0 && (!d_col_idx || !d_out_col_idx || !d_perm)) return TCG_EINVAL;
    if (nnz >= kIndexLimit || (int64_t)n_cols + 1 >= (int64_t)INT32_MAX) return TCG_ERANGE;
    TCG_TRY(refuse_capture(stream, "tcg_csr_transpose"));
    return csr_transpose_impl(n_rows, n_cols, nnz, d_row_ptr, d_col_idx, d_out_row_ptr, d_out_col_idx, d_perm,
                              static_cast<hipStream_t>(stream));
}

int tcg_reorder_rows(int32_t n, int64_t nnz, const int32_t *d_row_ptr, const int32_t *d_col_idx, uint64_t seed,
                     int32_t refine, int32_t *d_perm, void *stream)
{
    if (n < 0 || nnz < 0 || refine < 0 || !d_row_ptr) return TCG_EINVAL;
    if (n > 0 && !d_perm) return TCG_EINVAL;
    if (nnz > 0 && !d_col_idx) return TCG_EINVAL;
    if (nnz >= kIndexLimit || (int64_t)n + 1 >= (int64_t)INT32_MAX) return TCG_ERANGE;
    TCG_TRY(refuse_capture(stream, "tcg_reorder_rows"));
    return reorder_rows_impl(n, nnz, d_row_ptr, d_col_idx, seed, refine, d_perm, static_cast<hipStream_t>(stream));
}

int tcg_csr_permute(int32_t n, int64_t nnz, const int32_t *d_row_ptr, const int32_t *d_col_idx,
                    const int32_t *d_perm, int32_t *d_out_row_ptr, int32_t *d_out_col_idx, int32_t *d_edge_perm,
                    void *stream)
{
    if (n < 0 || nnz < 0 || !d_row_ptr || !d_out_row_ptr) return TCG_EINVAL;
    if (n > 0 && !d_perm) return TCG_EINVAL;
    if (nnz > 0 && (!d_col_idx || !d_out_col_idx)) return TCG_EINVAL;
    if (nnz >= kIndexLimit || (int64_t)n + 1 >= (int64_t)INT32_MAX) return TCG_ERANGE;
    TCG_TRY(refuse_capture(stream, "tcg_csr_permute"));
    return csr_permute_impl(n, nnz, d_row_ptr, d_col_idx, d_perm, d_out_row_ptr, d_out_col_idx, d_edge_perm,
                            static_cast<hipStream_t>(stream));
}

int tcg_edge_gather(int64_t n, const int32_t *d_perm, const float *d_in, float *d_out, void *stream)
{
    if (n < 0) return TCG_EINVAL;
    if (n > 0 && (!d_perm || !d_in || !d_out)) return TCG_EINVAL;
    return edge_gather_impl(n, d_perm, d_in, d_out, static_cast<hipStream_t>(stream));
}

int tcg_row_softmax(const tcg_meta *meta, const float *d_in, float *d_out, void *stream)
{
    if (!meta) return TCG_EINVAL;
    if (meta->nnz > 0 && (!d_in || !d_out)) return TCG_EINVAL;
    return row_softmax_impl(meta, d_in, d_out, static_cast<hipStream_t>(stream));
}

void tcg_sgt_free(tcg_meta *meta) { free_meta(meta); }

void tcg_release_cached_memory(void) { pool_release_all(); }

const char *tcg_strerror(int status)
{
    switch (status) {
    case TCG_OK: return "success";
    case TCG_EINVAL: return "invalid argument (null pointer, non-positive size, unsupported dtype, ld < D or misaligned pointer)";
    case TCG_ECSR: return "malformed CSR (row_ptr not monotone from 0 to nnz, or a column index out of range)";
    case TCG_ERANGE: return "size exceeds the int32 index space";
    case TCG_ENOMEM: return "out of memory";
    case TCG_ESCRATCH:
        snprintf(g_msg, sizeof(g_msg), "scratch buffer too small: %s", g_detail[0] ? g_detail : "(no detail recorded)");
        return g_msg;
    case TCG_EHIP:
        snprintf(g_msg, sizeof(g_msg), "HIP error: %s", g_hip_msg[0] ? g_hip_msg : "(no detail recorded)");
        return g_msg;
    case TCG_ECAPTURE:
        snprintf(g_msg, sizeof(g_msg), "not possible under stream capture: %s", g_detail[0] ? g_detail : "(no detail recorded)");
        return g_msg;
    default: return "unknown status";
    }
}

}  // extern "C"
