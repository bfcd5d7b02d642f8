"""ctypes front end of the CPU oracle (oracle/oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the benchmark's
CPU-baseline leg.  The product package never imports this module, and this module never
imports the product package.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

_i32p = ctypes.POINTER(ctypes.c_int32)
_i64p = ctypes.POINTER(ctypes.c_int64)
_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)


def build(force=False):
    """Compile oracle.c with gcc into liboracle.so next to it."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
           _SRC, "-o", _LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_sgt.restype = ctypes.c_int64
        lib.oracle_sgt.argtypes = [ctypes.c_int32, _i32p, _i32p, ctypes.c_int32, ctypes.c_int32,
                                   _i32p, _i64p, _i32p, _i32p]
        lib.oracle_spmm.restype = None
        lib.oracle_spmm.argtypes = [ctypes.c_int32, _i32p, _i32p, _f32p, _f32p, ctypes.c_int32,
                                    ctypes.c_int64, _f64p, ctypes.c_int64]
        lib.oracle_sddmm.restype = None
        lib.oracle_sddmm.argtypes = [ctypes.c_int32, _i32p, _i32p, _f32p, ctypes.c_int32,
                                     ctypes.c_int64, _f64p]
        lib.oracle_row_softmax.restype = None
        lib.oracle_row_softmax.argtypes = [ctypes.c_int32, _i32p, _f64p, _f64p]
        lib.oracle_spmm_tiled.restype = ctypes.c_int
        lib.oracle_spmm_tiled.argtypes = [ctypes.c_int32, _i32p, _i32p, _i32p, _i32p,
                                          ctypes.c_int32, ctypes.c_int32, _f32p, _f32p,
                                          ctypes.c_int32, ctypes.c_int64, _f64p, ctypes.c_int64]
        lib.oracle_sddmm_tiled.restype = ctypes.c_int
        lib.oracle_sddmm_tiled.argtypes = [ctypes.c_int32, _i32p, _i32p, _i32p, ctypes.c_int32,
                                           ctypes.c_int32, _f32p, ctypes.c_int32, ctypes.c_int64,
                                           _f64p]
        lib.oracle_csr_transpose.restype = None
        lib.oracle_csr_transpose.argtypes = [ctypes.c_int32, ctypes.c_int32, _i32p, _i32p, _i32p, _i32p, _i32p]
        lib.oracle_sddmm_pq.restype = None
        lib.oracle_sddmm_pq.argtypes = [ctypes.c_int32, _i32p, _i32p, _f32p, ctypes.c_int64, _f32p,
                                        ctypes.c_int64, ctypes.c_int32, _f64p]
        lib.oracle_row_softmax_backward.restype = None
        lib.oracle_row_softmax_backward.argtypes = [ctypes.c_int32, _i32p, _f64p, _f64p, _f64p]
        lib.oracle_tile_counts.restype = ctypes.c_int
        lib.oracle_tile_counts.argtypes = [ctypes.c_int32, _i32p, _i32p, ctypes.c_int32, ctypes.c_int32, _i64p, _i64p]
        lib.oracle_sgt_parallel.restype = ctypes.c_int64
        lib.oracle_sgt_parallel.argtypes = lib.oracle_sgt.argtypes
        lib.oracle_spmm_f32acc.restype = None
        lib.oracle_spmm_f32acc.argtypes = [ctypes.c_int32, _i32p, _i32p, _f32p, _f32p, ctypes.c_int32,
                                           ctypes.c_int64, _f32p, ctypes.c_int64]
        lib.oracle_sddmm_f32acc.restype = None
        lib.oracle_sddmm_f32acc.argtypes = [ctypes.c_int32, _i32p, _i32p, _f32p, ctypes.c_int32,
                                            ctypes.c_int64, _f32p]
        _lib = lib
    return _lib


def _p(a, t):
    return a.ctypes.data_as(t)


def _csr(row_ptr, col_idx):
    rp = np.ascontiguousarray(row_ptr, dtype=np.int32)
    ci = np.ascontiguousarray(col_idx, dtype=np.int32)
    if rp.ndim != 1 or rp.size < 1 or rp[0] != 0 or rp[-1] != ci.size or np.any(np.diff(rp) < 0):
        raise ValueError("malformed CSR")
    return rp, ci


def num_threads():
    return int(_load().oracle_num_threads())


def sgt(row_ptr, col_idx, win_h, tile_w, parallel=False):
    """Sparse Graph Translation (Algorithm 1).  Returns a dict with
    win_partition [n_win] int32, win_unique_ptr [n_win+1] int64, edge_to_col [nnz] int32,
    col_to_row [U] int32.  parallel=True runs the windows on all host cores (the variant the
    benchmark times; same results)."""
    rp, ci = _csr(row_ptr, col_idx)
    n_rows = rp.size - 1
    if win_h < 1 or tile_w < 1:
        raise ValueError("win_h and tile_w must be positive")
    n_win = (n_rows + win_h - 1) // win_h
    win_partition = np.zeros(n_win, dtype=np.int32)
    win_unique_ptr = np.zeros(n_win + 1, dtype=np.int64)
    edge_to_col = np.zeros(ci.size, dtype=np.int32)
    col_to_row = np.zeros(max(ci.size, 1), dtype=np.int32)
    fn = _load().oracle_sgt_parallel if parallel else _load().oracle_sgt
    total = fn(n_rows, _p(rp, _i32p), _p(ci, _i32p), win_h, tile_w,
                               _p(win_partition, _i32p), _p(win_unique_ptr, _i64p),
                               _p(edge_to_col, _i32p), _p(col_to_row, _i32p))
    if total < 0:
        raise ValueError("oracle_sgt rejected its arguments")
    return dict(win_partition=win_partition, win_unique_ptr=win_unique_ptr,
                edge_to_col=edge_to_col, col_to_row=col_to_row[:total].copy())


def tile_counts(row_ptr, col_idx, win_h, tile_w):
    """(translated, untranslated) tile counts: sum over windows of ceil(U_w / tile_w), and of the number of
    aligned tile_w-wide column blocks of the original matrix that hold an entry of the window."""
    rp, ci = _csr(row_ptr, col_idx)
    t, u = ctypes.c_int64(), ctypes.c_int64()
    if _load().oracle_tile_counts(rp.size - 1, _p(rp, _i32p), _p(ci, _i32p), win_h, tile_w, ctypes.byref(t),
                                  ctypes.byref(u)) != 0:
        raise ValueError("oracle_tile_counts rejected its arguments")
    return t.value, u.value


def spmm_f32acc(row_ptr, col_idx, X, w=None):
    """Equation 1 with float accumulation (timed CPU baseline, not the parity oracle)."""
    rp, ci = _csr(row_ptr, col_idx)
    n_rows = rp.size - 1
    X = _features(X, int(ci.max()) + 1 if ci.size else 0)
    D = X.shape[1]
    wp = None
    if w is not None:
        w = np.ascontiguousarray(w, dtype=np.float32)
        wp = _p(w, _f32p)
    Y = np.zeros((n_rows, D), dtype=np.float32)
    _load().oracle_spmm_f32acc(n_rows, _p(rp, _i32p), _p(ci, _i32p), wp, _p(X, _f32p), D, D, _p(Y, _f32p), D)
    return Y


def sddmm_f32acc(row_ptr, col_idx, X):
    """Equation 2 with float accumulation (timed CPU baseline, not the parity oracle)."""
    rp, ci = _csr(row_ptr, col_idx)
    n_rows = rp.size - 1
    X = _features(X, max(n_rows, int(ci.max()) + 1 if ci.size else 0))
    out = np.zeros(ci.size, dtype=np.float32)
    _load().oracle_sddmm_f32acc(n_rows, _p(rp, _i32p), _p(ci, _i32p), _p(X, _f32p), X.shape[1], X.shape[1],
                                _p(out, _f32p))
    return out


def _features(X, n_need):
    X = np.ascontiguousarray(X, dtype=np.float32)
    if X.ndim != 2 or X.shape[0] < n_need:
        raise ValueError("X must be 2-D with a row for every referenced node")
    return X


def spmm(row_ptr, col_idx, X, w=None):
    """Y = (w (.) A) X in double (Equation 1); w None means unit edge values."""
    rp, ci = _csr(row_ptr, col_idx)
    n_rows = rp.size - 1
    X = _features(X, int(ci.max()) + 1 if ci.size else 0)
    D = X.shape[1]
    wp = None
    if w is not None:
        w = np.ascontiguousarray(w, dtype=np.float32)
        if w.shape != ci.shape:
            raise ValueError("w must have one value per stored entry")
        wp = _p(w, _f32p)
    Y = np.zeros((n_rows, D), dtype=np.float64)
    _load().oracle_spmm(n_rows, _p(rp, _i32p), _p(ci, _i32p), wp, _p(X, _f32p), D, D,
                        _p(Y, _f64p), D)
    return Y


def sddmm(row_ptr, col_idx, X):
    """out[e] = <X[row(e)], X[col(e)]> in double, CSR order (Equation 2)."""
    rp, ci = _csr(row_ptr, col_idx)
    n_rows = rp.size - 1
    X = _features(X, max(n_rows, int(ci.max()) + 1 if ci.size else 0))
    out = np.zeros(ci.size, dtype=np.float64)
    _load().oracle_sddmm(n_rows, _p(rp, _i32p), _p(ci, _i32p), _p(X, _f32p), X.shape[1],
                         X.shape[1], _p(out, _f64p))
    return out


def row_softmax(row_ptr, v):
    """Softmax over the stored entries of each row, in double."""
    rp = np.ascontiguousarray(row_ptr, dtype=np.int32)
    v = np.ascontiguousarray(v, dtype=np.float64)
    if rp[-1] != v.size:
        raise ValueError("v must have one value per stored entry")
    p = np.zeros_like(v)
    _load().oracle_row_softmax(rp.size - 1, _p(rp, _i32p), _p(v, _f64p), _p(p, _f64p))
    return p


def spmm_tiled(row_ptr, col_idx, edge_to_col, win_partition, win_h, tile_w, X, w=None):
    """Algorithm 2 executed from the translated graph; must equal spmm()."""
    rp, ci = _csr(row_ptr, col_idx)
    n_rows = rp.size - 1
    X = _features(X, int(ci.max()) + 1 if ci.size else 0)
    D = X.shape[1]
    e2c = np.ascontiguousarray(edge_to_col, dtype=np.int32)
    wpart = np.ascontiguousarray(win_partition, dtype=np.int32)
    wp = None
    if w is not None:
        w = np.ascontiguousarray(w, dtype=np.float32)
        wp = _p(w, _f32p)
    Y = np.zeros((n_rows, D), dtype=np.float64)
    rc = _load().oracle_spmm_tiled(n_rows, _p(rp, _i32p), _p(ci, _i32p), _p(e2c, _i32p),
                                   _p(wpart, _i32p), win_h, tile_w, wp, _p(X, _f32p), D, D,
                                   _p(Y, _f64p), D)
    if rc != 0:
        raise ValueError("translated graph is inconsistent: an edge lies outside its window's blocks")
    return Y


def sddmm_tiled(row_ptr, col_idx, edge_to_col, win_h, tile_w, X):
    """Algorithm 3 executed from the translated graph; must equal sddmm()."""
    rp, ci = _csr(row_ptr, col_idx)
    n_rows = rp.size - 1
    X = _features(X, max(n_rows, int(ci.max()) + 1 if ci.size else 0))
    e2c = np.ascontiguousarray(edge_to_col, dtype=np.int32)
    out = np.zeros(ci.size, dtype=np.float64)
    _load().oracle_sddmm_tiled(n_rows, _p(rp, _i32p), _p(ci, _i32p), _p(e2c, _i32p), win_h,
                               tile_w, _p(X, _f32p), X.shape[1], X.shape[1], _p(out, _f64p))
    return out


def csr_transpose(row_ptr, col_idx, n_cols):
    """CSR of the transpose: (row_ptr_t [n_cols+1], col_idx_t [nnz], perm [nnz]); entry k of the
    transpose is entry perm[k] of the input."""
    rp, ci = _csr(row_ptr, col_idx)
    if ci.size and int(ci.max()) >= n_cols:
        raise ValueError("column index out of range")
    rpt = np.zeros(n_cols + 1, dtype=np.int32)
    cit = np.zeros(ci.size, dtype=np.int32)
    perm = np.zeros(ci.size, dtype=np.int32)
    _load().oracle_csr_transpose(rp.size - 1, n_cols, _p(rp, _i32p), _p(ci, _i32p), _p(rpt, _i32p),
                                 _p(cit, _i32p), _p(perm, _i32p))
    return rpt, cit, perm


def sddmm_pq(row_ptr, col_idx, P, Q):
    """out[e] = <P[row(e)], Q[col(e)]> in double, CSR order."""
    rp, ci = _csr(row_ptr, col_idx)
    P = _features(P, rp.size - 1)
    Q = _features(Q, int(ci.max()) + 1 if ci.size else 0)
    if P.shape[1] != Q.shape[1]:
        raise ValueError("P and Q must have the same width")
    out = np.zeros(ci.size, dtype=np.float64)
    _load().oracle_sddmm_pq(rp.size - 1, _p(rp, _i32p), _p(ci, _i32p), _p(P, _f32p), P.shape[1],
                            _p(Q, _f32p), Q.shape[1], P.shape[1], _p(out, _f64p))
    return out


def row_softmax_backward(row_ptr, p, dp):
    """dv[e] = p[e] * (dp[e] - sum over the row of p * dp), in double."""
    rp = np.ascontiguousarray(row_ptr, dtype=np.int32)
    p = np.ascontiguousarray(p, dtype=np.float64)
    dp = np.ascontiguousarray(dp, dtype=np.float64)
    if rp[-1] != p.size or p.shape != dp.shape:
        raise ValueError("p and dp must have one value per stored entry")
    dv = np.zeros_like(p)
    _load().oracle_row_softmax_backward(rp.size - 1, _p(rp, _i32p), _p(p, _f64p), _p(dp, _f64p), _p(dv, _f64p))
    return dv
