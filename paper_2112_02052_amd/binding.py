"""Thin ctypes binding of libtcgnn.so (include/tcgnn.h).  Argument marshalling only: every
step of the path runs in the library's HIP kernels.  torch supplies device memory and the
current stream; nothing here computes, and there is no CPU fallback -- if the library is
missing or a call fails, an exception is raised."""
import ctypes
import os

import torch

from .build import LIB_PATH

TCG_F32, TCG_BF16, TCG_F16 = 0, 1, 2
POLICY_AUTO, POLICY_GATHER, POLICY_TILE = 0, 1, 2

EXPORTED = ["tcg_sgt_build", "tcg_sgt_sizes", "tcg_sgt_export", "tcg_sgt_set_policy",
            "tcg_sgt_plan_stats", "tcg_spmm", "tcg_sddmm", "tcg_row_softmax", "tcg_sgt_free",
            "tcg_strerror", "tcg_release_cached_memory", "tcg_sddmm_pq", "tcg_row_softmax_backward",
            "tcg_csr_transpose", "tcg_edge_gather", "tcg_attention", "tcg_reorder_rows", "tcg_csr_permute",
            "tcg_sgt_reserve", "tcg_spmm_noalloc", "tcg_sgt_tile_stats", "tcg_attention_cos", "tcg_row_rnorm",
            "tcg_sgt_build_clustered", "tcg_row_unit_grad"]

_DTYPES = {torch.float32: TCG_F32, torch.bfloat16: TCG_BF16, torch.float16: TCG_F16}

_vp = ctypes.c_void_p
_i64p = ctypes.POINTER(ctypes.c_int64)
_lib = None


class TcgError(RuntimeError):
    def __init__(self, status, text):
        super().__init__("tcgnn status %d: %s" % (status, text))
        self.status = status


def load_library():
    """Loads libtcgnn.so; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libtcgnn.so is not built: run `python -m paper_2112_02052_amd.build` "
                           "(or __graft_entry__.build()) first")
    lib = ctypes.CDLL(LIB_PATH)
    lib.tcg_sgt_build.restype = ctypes.c_int
    lib.tcg_sgt_build.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, _vp, _vp, ctypes.c_int32,
                                  ctypes.c_int32, ctypes.c_int, _vp, ctypes.POINTER(_vp)]
    lib.tcg_sgt_sizes.restype = ctypes.c_int
    lib.tcg_sgt_sizes.argtypes = [_vp, _i64p, _i64p, _i64p, _i64p]
    lib.tcg_sgt_export.restype = ctypes.c_int
    lib.tcg_sgt_export.argtypes = [_vp, _vp, _vp, _vp, _vp, ctypes.c_int, _vp]
    lib.tcg_sgt_set_policy.restype = ctypes.c_int
    lib.tcg_sgt_set_policy.argtypes = [_vp, ctypes.c_int, ctypes.c_float, _vp]
    lib.tcg_sgt_plan_stats.restype = ctypes.c_int
    lib.tcg_sgt_plan_stats.argtypes = [_vp, _i64p, _i64p, _i64p, _i64p]
    lib.tcg_spmm.restype = ctypes.c_int
    lib.tcg_spmm.argtypes = [_vp, _vp, ctypes.c_int, ctypes.c_int32, ctypes.c_int64, _vp, _vp, ctypes.c_int,
                             ctypes.c_int64, _vp]
    lib.tcg_sgt_tile_stats.restype = ctypes.c_int
    lib.tcg_sgt_tile_stats.argtypes = [_vp, ctypes.c_int32, _i64p, _i64p, _vp]
    lib.tcg_sgt_reserve.restype = ctypes.c_int
    lib.tcg_sgt_reserve.argtypes = [_vp, ctypes.c_int32, _vp]
    lib.tcg_spmm_noalloc.restype = ctypes.c_int
    lib.tcg_spmm_noalloc.argtypes = lib.tcg_spmm.argtypes
    lib.tcg_sddmm.restype = ctypes.c_int
    lib.tcg_sddmm.argtypes = [_vp, _vp, ctypes.c_int, ctypes.c_int32, ctypes.c_int64, _vp, _vp]
    lib.tcg_row_softmax.restype = ctypes.c_int
    lib.tcg_row_softmax.argtypes = [_vp, _vp, _vp, _vp]
    lib.tcg_sgt_free.restype = None
    lib.tcg_sgt_free.argtypes = [_vp]
    lib.tcg_sddmm_pq.restype = ctypes.c_int
    lib.tcg_sddmm_pq.argtypes = [_vp, _vp, ctypes.c_int64, _vp, ctypes.c_int64, ctypes.c_int, ctypes.c_int32, _vp, _vp]
    lib.tcg_row_softmax_backward.restype = ctypes.c_int
    lib.tcg_row_softmax_backward.argtypes = [_vp, _vp, _vp, _vp, _vp]
    lib.tcg_csr_transpose.restype = ctypes.c_int
    lib.tcg_csr_transpose.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, _vp, _vp, _vp, _vp, _vp, _vp]
    lib.tcg_reorder_rows.restype = ctypes.c_int
    lib.tcg_reorder_rows.argtypes = [ctypes.c_int32, ctypes.c_int64, _vp, _vp, ctypes.c_uint64, ctypes.c_int32, _vp, _vp]
    lib.tcg_csr_permute.restype = ctypes.c_int
    lib.tcg_csr_permute.argtypes = [ctypes.c_int32, ctypes.c_int64, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
    lib.tcg_edge_gather.restype = ctypes.c_int
    lib.tcg_edge_gather.argtypes = [ctypes.c_int64, _vp, _vp, _vp, _vp]
    lib.tcg_attention.restype = ctypes.c_int
    lib.tcg_attention.argtypes = [_vp, _vp, ctypes.c_int, ctypes.c_int32, ctypes.c_int64, _vp, _vp, ctypes.c_int,
                                  ctypes.c_int64, _vp]
    lib.tcg_attention_cos.restype = ctypes.c_int
    lib.tcg_attention_cos.argtypes = [_vp, _vp, ctypes.c_int, ctypes.c_int32, ctypes.c_int64, _vp, ctypes.c_float, _vp, _vp,
                                      ctypes.c_int, ctypes.c_int64, _vp]
    lib.tcg_row_unit_grad.restype = ctypes.c_int
    lib.tcg_row_unit_grad.argtypes = [ctypes.c_int64, _vp, ctypes.c_int, ctypes.c_int32, ctypes.c_int64, _vp, ctypes.c_float,
                                      _vp, ctypes.c_int64, _vp, ctypes.c_int64, _vp]
    lib.tcg_row_rnorm.restype = ctypes.c_int
    lib.tcg_row_rnorm.argtypes = [ctypes.c_int64, _vp, ctypes.c_int, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, _vp, _vp]
    lib.tcg_sgt_build_clustered.restype = ctypes.c_int
    lib.tcg_sgt_build_clustered.argtypes = [ctypes.c_int32, ctypes.c_int64, _vp, _vp, ctypes.c_int32, ctypes.c_int32,
                                            ctypes.c_uint64, ctypes.c_int32, _vp, _vp, _vp, _vp, _vp, ctypes.POINTER(_vp)]
    lib.tcg_release_cached_memory.restype = None
    lib.tcg_release_cached_memory.argtypes = []
    lib.tcg_strerror.restype = ctypes.c_char_p
    lib.tcg_strerror.argtypes = [ctypes.c_int]
    _lib = lib
    return lib


def _check(status):
    if status != 0:
        raise TcgError(status, load_library().tcg_strerror(status).decode())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def _need_cuda(*tensors):
    for t in tensors:
        if t is not None and not t.is_cuda:
            raise ValueError("tensors must live on the GPU")


class Meta:
    """Owner of a tcg_meta handle.  Keeps the CSR tensors alive (the library borrows them)."""

    def __init__(self, handle, row_ptr, col_idx, n_rows, n_cols, window_h, tile_w):
        self._h = handle
        self.row_ptr, self.col_idx = row_ptr, col_idx
        self.n_rows, self.n_cols, self.window_h, self.tile_w = n_rows, n_cols, window_h, tile_w
        nw, u, t, nnz = (ctypes.c_int64() for _ in range(4))
        _check(load_library().tcg_sgt_sizes(self._h, nw, u, t, nnz))
        self.n_windows, self.total_unique, self.total_tiles, self.nnz = nw.value, u.value, t.value, nnz.value

    def free(self):
        if self._h is not None:
            torch.cuda.synchronize()
            load_library().tcg_sgt_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def sgt_build(row_ptr, col_idx, window_h=16, tile_w=8, n_cols=None, validate=True):
    """tcg_sgt_build: row_ptr int32[n_rows+1], col_idx int32[nnz] CUDA tensors."""
    _need_cuda(row_ptr, col_idx)
    if row_ptr.dtype != torch.int32 or col_idx.dtype != torch.int32:
        raise ValueError("CSR arrays must be int32")
    row_ptr, col_idx = row_ptr.contiguous(), col_idx.contiguous()
    n_rows = row_ptr.numel() - 1
    n_cols = n_rows if n_cols is None else int(n_cols)
    h = ctypes.c_void_p()
    _check(load_library().tcg_sgt_build(n_rows, n_cols, col_idx.numel(), _ptr(row_ptr), _ptr(col_idx),
                                        int(window_h), int(tile_w), int(bool(validate)), _stream(),
                                        ctypes.byref(h)))
    return Meta(h, row_ptr, col_idx, n_rows, n_cols, int(window_h), int(tile_w))


def sgt_export(meta):
    """tcg_sgt_export into fresh CUDA int32 tensors: dict of the four metadata arrays."""
    dev = meta.row_ptr.device
    out = dict(win_partition=torch.empty(meta.n_windows, dtype=torch.int32, device=dev),
               win_unique_ptr=torch.empty(meta.n_windows + 1, dtype=torch.int32, device=dev),
               edge_to_col=torch.empty(meta.nnz, dtype=torch.int32, device=dev),
               col_to_row=torch.empty(meta.total_unique, dtype=torch.int32, device=dev))
    _check(load_library().tcg_sgt_export(meta._h, _ptr(out["win_partition"]), _ptr(out["win_unique_ptr"]),
                                         _ptr(out["edge_to_col"]), _ptr(out["col_to_row"]), 1, _stream()))
    return out


def sgt_set_policy(meta, policy, min_reuse=0.0):
    _check(load_library().tcg_sgt_set_policy(meta._h, int(policy), float(min_reuse), _stream()))


def sgt_tile_stats(meta, tile_w):
    """tcg_sgt_tile_stats: (tiles with the translation, tiles without it) for tiles of tile_w columns."""
    t, u = ctypes.c_int64(), ctypes.c_int64()
    _check(load_library().tcg_sgt_tile_stats(meta._h, int(tile_w), t, u, _stream()))
    return t.value, u.value


def sgt_reserve(meta, max_D):
    """tcg_sgt_reserve: size the plan's scratch for feature widths up to max_D now (needed before capturing
    calls with D > 128 into a HIP graph)."""
    _check(load_library().tcg_sgt_reserve(meta._h, int(max_D), _stream()))


def sgt_plan_stats(meta):
    a, b, c, d = (ctypes.c_int64() for _ in range(4))
    _check(load_library().tcg_sgt_plan_stats(meta._h, a, b, c, d))
    return dict(n_tile_windows=a.value, nnz_tile=b.value, n_segments=c.value, n_long_rows=d.value)


def _features(meta, X, rows_needed):
    _need_cuda(X)
    if X.dim() != 2 or X.dtype not in _DTYPES or X.stride(1) != 1:
        raise ValueError("X must be a 2-D fp32/bf16/fp16 tensor with unit stride along features")
    if X.shape[0] < rows_needed:
        raise ValueError("X has %d rows, the graph needs %d" % (X.shape[0], rows_needed))
    return X


def spmm_noalloc(meta, X, w, Y):
    """tcg_spmm_noalloc: tcg_spmm with the split rows' partial sums in the library's static device array;
    the caller passes every buffer, the call allocates nothing."""
    return spmm(meta, X, w, Y, _entry="tcg_spmm_noalloc")


def spmm(meta, X, w=None, Y=None, y_dtype=torch.float32, _entry="tcg_spmm"):
    """tcg_spmm: Y = (w (.) A) X.  Returns Y (allocated here unless given)."""
    X = _features(meta, X, meta.n_cols)
    D = X.shape[1]
    if w is not None:
        _need_cuda(w)
        if w.dtype != torch.float32 or w.numel() != meta.nnz or not w.is_contiguous():
            raise ValueError("w must be a contiguous fp32 tensor with one value per stored entry")
    if Y is None:
        Y = torch.empty((meta.n_rows, D), dtype=y_dtype, device=X.device)
    _need_cuda(Y)
    if Y.dim() != 2 or Y.shape != (meta.n_rows, D) or Y.stride(1) != 1 or Y.dtype not in _DTYPES:
        raise ValueError("Y must be [n_rows, D] with unit stride along features")
    _check(getattr(load_library(), _entry)(meta._h, _ptr(X), _DTYPES[X.dtype], D, X.stride(0), _ptr(w), _ptr(Y),
                                           _DTYPES[Y.dtype], Y.stride(0) if meta.n_rows > 1 else max(D, Y.stride(0)),
                                           _stream()))
    return Y


def sddmm(meta, X, out=None):
    """tcg_sddmm: out[e] = <X[row(e)], X[col(e)]>, fp32 in CSR order."""
    X = _features(meta, X, max(meta.n_rows, meta.n_cols))
    if out is None:
        out = torch.empty(meta.nnz, dtype=torch.float32, device=X.device)
    _need_cuda(out)
    if out.dtype != torch.float32 or out.numel() != meta.nnz or not out.is_contiguous():
        raise ValueError("out must be a contiguous fp32 tensor with one value per stored entry")
    _check(load_library().tcg_sddmm(meta._h, _ptr(X), _DTYPES[X.dtype], X.shape[1], X.stride(0), _ptr(out),
                                    _stream()))
    return out


def release_cached_memory():
    """tcg_release_cached_memory: hand the library's cached device blocks back to the driver."""
    load_library().tcg_release_cached_memory()


def row_softmax(meta, v, out=None):
    """tcg_row_softmax over the stored entries of each row."""
    _need_cuda(v)
    if v.dtype != torch.float32 or v.numel() != meta.nnz or not v.is_contiguous():
        raise ValueError("v must be a contiguous fp32 tensor with one value per stored entry")
    if out is None:
        out = torch.empty_like(v)
    _check(load_library().tcg_row_softmax(meta._h, _ptr(v), _ptr(out), _stream()))
    return out


def sddmm_pq(meta, P, Q, out=None):
    """tcg_sddmm_pq: out[e] = <P[row(e)], Q[col(e)]>, fp32 in CSR order."""
    P = _features(meta, P, meta.n_rows)
    Q = _features(meta, Q, meta.n_cols)
    if P.dtype != Q.dtype or P.shape[1] != Q.shape[1]:
        raise ValueError("P and Q must have the same type and width")
    if out is None:
        out = torch.empty(meta.nnz, dtype=torch.float32, device=P.device)
    _need_cuda(out)
    if out.dtype != torch.float32 or out.numel() != meta.nnz or not out.is_contiguous():
        raise ValueError("out must be a contiguous fp32 tensor with one value per stored entry")
    _check(load_library().tcg_sddmm_pq(meta._h, _ptr(P), P.stride(0), _ptr(Q), Q.stride(0), _DTYPES[P.dtype],
                                       P.shape[1], _ptr(out), _stream()))
    return out


def row_softmax_backward(meta, p, dp, out=None):
    """tcg_row_softmax_backward: dv = p * (dp - rowsum(p * dp))."""
    _need_cuda(p, dp)
    for t in (p, dp):
        if t.dtype != torch.float32 or t.numel() != meta.nnz or not t.is_contiguous():
            raise ValueError("p and dp must be contiguous fp32 tensors with one value per stored entry")
    if out is None:
        out = torch.empty_like(dp)
    _check(load_library().tcg_row_softmax_backward(meta._h, _ptr(p), _ptr(dp), _ptr(out), _stream()))
    return out


def csr_transpose(row_ptr, col_idx, n_cols=None):
    """tcg_csr_transpose: (row_ptr_t, col_idx_t, perm) as CUDA int32 tensors."""
    _need_cuda(row_ptr, col_idx)
    if row_ptr.dtype != torch.int32 or col_idx.dtype != torch.int32:
        raise ValueError("CSR arrays must be int32")
    row_ptr, col_idx = row_ptr.contiguous(), col_idx.contiguous()
    n_rows = row_ptr.numel() - 1
    n_cols = n_rows if n_cols is None else int(n_cols)
    nnz = col_idx.numel()
    rpt = torch.empty(n_cols + 1, dtype=torch.int32, device=row_ptr.device)
    cit = torch.empty(nnz, dtype=torch.int32, device=row_ptr.device)
    perm = torch.empty(nnz, dtype=torch.int32, device=row_ptr.device)
    _check(load_library().tcg_csr_transpose(n_rows, n_cols, nnz, _ptr(row_ptr), _ptr(col_idx), _ptr(rpt), _ptr(cit),
                                            _ptr(perm), _stream()))
    return rpt, cit, perm


def edge_gather(perm, values, out=None):
    """tcg_edge_gather: out[k] = values[perm[k]]."""
    _need_cuda(perm, values)
    if perm.dtype != torch.int32 or values.dtype != torch.float32 or perm.numel() != values.numel():
        raise ValueError("perm must be int32 and values fp32, of equal length")
    perm, values = perm.contiguous(), values.contiguous()
    if out is None:
        out = torch.empty_like(values)
    _check(load_library().tcg_edge_gather(perm.numel(), _ptr(perm), _ptr(values), _ptr(out), _stream()))
    return out


def _square_csr(row_ptr, col_idx):
    _need_cuda(row_ptr, col_idx)
    if row_ptr.dtype != torch.int32 or col_idx.dtype != torch.int32:
        raise ValueError("CSR arrays must be int32")
    return row_ptr.contiguous(), col_idx.contiguous()


def reorder_rows(row_ptr, col_idx, seed=0, refine=2):
    """tcg_reorder_rows: perm (CUDA int32 [n], perm[new] = old) that puts rows with shared neighbours next
    to each other."""
    row_ptr, col_idx = _square_csr(row_ptr, col_idx)
    n = row_ptr.numel() - 1
    perm = torch.empty(n, dtype=torch.int32, device=row_ptr.device)
    _check(load_library().tcg_reorder_rows(n, col_idx.numel(), _ptr(row_ptr), _ptr(col_idx), int(seed) & (2 ** 64 - 1),
                                           int(refine), _ptr(perm), _stream()))
    return perm


def csr_permute(row_ptr, col_idx, perm, want_edge_perm=True):
    """tcg_csr_permute: (row_ptr', col_idx', edge_perm or None) of the symmetrically relabelled pattern."""
    row_ptr, col_idx = _square_csr(row_ptr, col_idx)
    _need_cuda(perm)
    n = row_ptr.numel() - 1
    nnz = col_idx.numel()
    if perm.dtype != torch.int32 or perm.numel() != n:
        raise ValueError("perm must be int32 with one entry per node")
    perm = perm.contiguous()
    rp2 = torch.empty(n + 1, dtype=torch.int32, device=row_ptr.device)
    ci2 = torch.empty(nnz, dtype=torch.int32, device=row_ptr.device)
    ep = torch.empty(nnz, dtype=torch.int32, device=row_ptr.device) if want_edge_perm else None
    _check(load_library().tcg_csr_permute(n, nnz, _ptr(row_ptr), _ptr(col_idx), _ptr(perm), _ptr(rp2), _ptr(ci2),
                                          _ptr(ep), _stream()))
    return rp2, ci2, ep


def attention(meta, X, Y=None, scores=None, y_dtype=torch.float32):
    """tcg_attention: Y[i] = sum_e softmax_i(<x_i, x_j>)_e x_j in one pass.  `scores` (optional fp32 [nnz])
    receives the raw scores."""
    X = _features(meta, X, max(meta.n_rows, meta.n_cols))
    D = X.shape[1]
    if Y is None:
        Y = torch.empty((meta.n_rows, D), dtype=y_dtype, device=X.device)
    _need_cuda(Y, scores)
    if Y.dim() != 2 or Y.shape != (meta.n_rows, D) or Y.stride(1) != 1 or Y.dtype not in _DTYPES:
        raise ValueError("Y must be [n_rows, D] with unit stride along features")
    if scores is not None and (scores.dtype != torch.float32 or scores.numel() != meta.nnz or not scores.is_contiguous()):
        raise ValueError("scores must be a contiguous fp32 tensor with one value per stored entry")
    _check(load_library().tcg_attention(meta._h, _ptr(X), _DTYPES[X.dtype], D, X.stride(0), _ptr(scores), _ptr(Y),
                                        _DTYPES[Y.dtype], Y.stride(0) if meta.n_rows > 1 else max(D, Y.stride(0)),
                                        _stream()))
    return Y


def row_rnorm(X, eps=1e-12, out=None):
    """tcg_row_rnorm: out[i] = 1 / max(|X[i]|, eps), fp32."""
    _need_cuda(X)
    if X.dim() != 2 or X.dtype not in _DTYPES or X.stride(1) != 1:
        raise ValueError("X must be a 2-D fp32/bf16/fp16 tensor with unit stride along features")
    if out is None:
        out = torch.empty(X.shape[0], dtype=torch.float32, device=X.device)
    _check(load_library().tcg_row_rnorm(X.shape[0], _ptr(X), _DTYPES[X.dtype], X.shape[1], X.stride(0), float(eps), _ptr(out),
                                        _stream()))
    return out


def row_unit_grad(X, rnorm, G, dX, scale=1.0):
    """tcg_row_unit_grad: dX[i] += scale * rnorm[i] * (G[i] - xn[i] <G[i], xn[i]>) with xn = rnorm * X; returns dX."""
    _need_cuda(X, rnorm, G, dX)
    if X.dim() != 2 or X.dtype not in _DTYPES or X.stride(1) != 1:
        raise ValueError("X must be a 2-D fp32/bf16/fp16 tensor with unit stride along features")
    n, D = X.shape
    for t in (G, dX):
        if t.dtype != torch.float32 or t.shape != X.shape or t.stride(1) != 1:
            raise ValueError("G and dX must be fp32 tensors of X's shape with unit stride along features")
    if rnorm.dtype != torch.float32 or rnorm.numel() != n or not rnorm.is_contiguous():
        raise ValueError("rnorm must be a contiguous fp32 tensor with one value per row")
    _check(load_library().tcg_row_unit_grad(n, _ptr(X), _DTYPES[X.dtype], D, X.stride(0) if n > 1 else max(D, X.stride(0)),
                                            _ptr(rnorm), float(scale), _ptr(G), G.stride(0) if n > 1 else max(D, G.stride(0)),
                                            _ptr(dX), dX.stride(0) if n > 1 else max(D, dX.stride(0)), _stream()))
    return dX


def attention_cos(meta, X, rnorm, beta, Y=None, scores=None, y_dtype=torch.float32):
    """tcg_attention_cos: Y[i] = sum_e softmax_i(beta * c)_e x_j with c_e = rnorm_i rnorm_j <x_i, x_j>; `scores`
    (optional fp32 [nnz]) receives c."""
    X = _features(meta, X, max(meta.n_rows, meta.n_cols))
    D = X.shape[1]
    _need_cuda(rnorm)
    if rnorm.dtype != torch.float32 or rnorm.numel() < max(meta.n_rows, meta.n_cols) or not rnorm.is_contiguous():
        raise ValueError("rnorm must be a contiguous fp32 tensor with one value per node")
    if Y is None:
        Y = torch.empty((meta.n_rows, D), dtype=y_dtype, device=X.device)
    _need_cuda(Y, scores)
    if Y.dim() != 2 or Y.shape != (meta.n_rows, D) or Y.stride(1) != 1 or Y.dtype not in _DTYPES:
        raise ValueError("Y must be [n_rows, D] with unit stride along features")
    if scores is not None and (scores.dtype != torch.float32 or scores.numel() != meta.nnz or not scores.is_contiguous()):
        raise ValueError("scores must be a contiguous fp32 tensor with one value per stored entry")
    _check(load_library().tcg_attention_cos(meta._h, _ptr(X), _DTYPES[X.dtype], D, X.stride(0), _ptr(rnorm), float(beta),
                                            _ptr(scores), _ptr(Y), _DTYPES[Y.dtype],
                                            Y.stride(0) if meta.n_rows > 1 else max(D, Y.stride(0)), _stream()))
    return Y


def sgt_build_clustered(row_ptr, col_idx, window_h=16, tile_w=8, seed=0, refine=2, want_edge_perm=True):
    """tcg_sgt_build_clustered: (meta of the relabelled graph, perm [new -> old], edge_perm or None).  The meta's
    row_ptr / col_idx are the relabelled pattern."""
    row_ptr, col_idx = _square_csr(row_ptr, col_idx)
    n, nnz = row_ptr.numel() - 1, col_idx.numel()
    dev = row_ptr.device
    perm = torch.empty(n, dtype=torch.int32, device=dev)
    rp2 = torch.empty(n + 1, dtype=torch.int32, device=dev)
    ci2 = torch.empty(nnz, dtype=torch.int32, device=dev)
    ep = torch.empty(nnz, dtype=torch.int32, device=dev) if want_edge_perm else None
    h = ctypes.c_void_p()
    _check(load_library().tcg_sgt_build_clustered(n, nnz, _ptr(row_ptr), _ptr(col_idx), int(window_h), int(tile_w),
                                                  int(seed) & (2 ** 64 - 1), int(refine), _stream(), _ptr(perm), _ptr(rp2),
                                                  _ptr(ci2), _ptr(ep), ctypes.byref(h)))
    return Meta(h, rp2, ci2, n, n, int(window_h), int(tile_w)), perm, ep
