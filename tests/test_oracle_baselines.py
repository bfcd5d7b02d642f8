"""Pins for the oracle functions added for measurement: the tile counts with and without the translation
(the quantity of the paper's SGT-effectiveness study, section 5.2) and the variants that the benchmark
times as CPU baselines (windows in parallel; float accumulation), which are never used for parity."""
import numpy as np
import pytest

import oracle
import workloads as W
from workloads.graphs import CSR


def dense_tile_counts(A, H, W_):
    """From the dense matrix: non-empty columns per window (translated: packed first, then cut into tiles)
    and non-empty aligned W-wide column blocks per window (untranslated)."""
    n, n_cols = A.shape
    t = u = 0
    for r0 in range(0, n, H):
        blk = A[r0:r0 + H]
        nonempty = blk.any(axis=0)
        t += -(-int(nonempty.sum()) // W_)
        pad = (-n_cols) % W_
        u += int(np.pad(nonempty, (0, pad)).reshape(-1, W_).any(axis=1).sum())
    return t, u


@pytest.mark.parametrize("seed", range(6))
def test_tile_counts_against_the_dense_matrix(seed):
    rng = np.random.default_rng(seed)
    n, n_cols = int(rng.integers(5, 60)), int(rng.integers(5, 70))
    A = rng.random((n, n_cols)) < rng.choice([0.05, 0.2, 0.6])
    rp = np.concatenate([[0], np.cumsum(A.sum(axis=1))]).astype(np.int32)
    ci = np.concatenate([np.flatnonzero(r)[::-1] for r in A] + [np.zeros(0, np.int64)]).astype(np.int32)  # unsorted rows
    for H, W_ in ((1, 1), (4, 3), (16, 8), (7, 16), (64, 4)):
        assert oracle.tile_counts(rp, ci, H, W_) == dense_tile_counts(A, H, W_)


def test_tile_counts_closed_forms():
    # Identity: a window of H rows holds H neighbouring columns: ceil(H / W) tiles either way when H is a
    # multiple of W and the window starts at a multiple of W.
    n = 64
    rp = np.arange(n + 1, dtype=np.int32)
    ci = np.arange(n, dtype=np.int32)
    assert oracle.tile_counts(rp, ci, 16, 8) == (4 * 2, 4 * 2)
    # One entry per row, 16 columns apart: 16 distinct columns per window pack into 2 tiles of 8, but sit in
    # 16 different column blocks of the original matrix -- the reduction the translation is for.
    ci = ((np.arange(n) % 16) * 16).astype(np.int32)
    assert oracle.tile_counts(rp, ci, 16, 8) == (4 * 2, 4 * 16)
    # the translated count equals the sum of win_partition
    c = W.make_config(3, n=3000, d=4)["csr"]
    m = oracle.sgt(c.row_ptr, c.col_idx, 16, 8)
    t, u = oracle.tile_counts(c.row_ptr, c.col_idx, 16, 8)
    assert t == int(m["win_partition"].sum()) and u >= t


@pytest.mark.parametrize("cfg,n,H,W_", [(1, 2048, 16, 8), (3, 6000, 16, 16), (4, 20000, 16, 8), (5, 64 * 50, 16, 8),
                                        (2, 1003, 12, 5), (4, 777, 1, 3), (3, 500, 500, 8)])
def test_parallel_translation_equals_the_sequential_one(cfg, n, H, W_):
    g = W.make_config(cfg, n=n, d=4)["csr"]
    a = oracle.sgt(g.row_ptr, g.col_idx, H, W_)
    b = oracle.sgt(g.row_ptr, g.col_idx, H, W_, parallel=True)
    for k in a:
        assert np.array_equal(a[k], b[k]), k


def test_parallel_translation_on_an_empty_graph():
    rp = np.zeros(9, dtype=np.int32)
    b = oracle.sgt(rp, np.zeros(0, np.int32), 4, 8, parallel=True)
    assert b["col_to_row"].size == 0 and np.array_equal(b["win_partition"], np.zeros(2, np.int32))


@pytest.mark.parametrize("cfg,n,D", [(1, 2048, 16), (2, 20000, 64), (3, 20000, 32), (4, 30000, 128)])
def test_float_accumulating_baselines_stay_within_the_fp32_tolerance(cfg, n, D):
    c = W.make_config(cfg, n=n, d=D)
    g, X, w = c["csr"], c["X"], c["w"]
    Y = oracle.spmm(g.row_ptr, g.col_idx, X, w)
    Yf = oracle.spmm_f32acc(g.row_ptr, g.col_idx, X, w)
    assert Yf.dtype == np.float32 and np.abs(Yf - Y).max() <= 1e-5 * np.abs(Y).max()
    e = oracle.sddmm(g.row_ptr, g.col_idx, X)
    ef = oracle.sddmm_f32acc(g.row_ptr, g.col_idx, X)
    assert ef.dtype == np.float32 and np.abs(ef - e).max() <= 1e-5 * np.abs(e).max()
