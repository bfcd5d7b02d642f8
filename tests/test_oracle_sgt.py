"""Pins for the oracle's Sparse Graph Translation (Algorithm 1 of the paper).

None of these re-implements the oracle's sort/unique/search: they check it against a dense
brute-force construction, invariants any correct translation satisfies, closed-form special
cases, and a hand-worked example.
"""
import json
import os

import numpy as np
import pytest

import oracle
import workloads as W


def dense_from_csr(rp, ci, n_cols):
    A = np.zeros((len(rp) - 1, n_cols), dtype=np.int64)
    for i in range(len(rp) - 1):
        for e in range(rp[i], rp[i + 1]):
            A[i, ci[e]] += 1
    return A


def brute_force_sgt(rp, ci, n_cols, H, W_):
    """Definition by picture: take the dense H x n_cols block of a window, list its non-empty
    columns left to right; that list is the condensed column order."""
    A = dense_from_csr(rp, ci, n_cols)
    n = A.shape[0]
    n_win = -(-n // H)
    part, uptr, c2r, e2c = [], [0], [], np.zeros(len(ci), dtype=np.int64)
    for w in range(n_win):
        blk = A[w * H:min(n, (w + 1) * H)]
        cols = [c for c in range(n_cols) if blk[:, c].any()]
        pos = {c: k for k, c in enumerate(cols)}
        part.append(-(-len(cols) // W_))
        uptr.append(uptr[-1] + len(cols))
        c2r += cols
        for e in range(rp[w * H], rp[min(n, (w + 1) * H)]):
            e2c[e] = pos[ci[e]]
    return np.array(part), np.array(uptr), np.array(c2r), e2c


def check_invariants(rp, ci, n_cols, H, W_, m):
    rp = np.asarray(rp, dtype=np.int64)
    n = len(rp) - 1
    n_win = -(-n // H)
    assert m["win_partition"].shape == (n_win,)
    assert m["win_unique_ptr"].shape == (n_win + 1,)
    assert m["edge_to_col"].shape == (len(ci),)          # same length as edgeList (section 4.1)
    uptr = m["win_unique_ptr"]
    assert uptr[0] == 0 and uptr[-1] == len(m["col_to_row"])
    covered = 0
    for w in range(n_win):
        lo, hi = rp[w * H], rp[min(n, (w + 1) * H)]
        covered += hi - lo
        U = uptr[w + 1] - uptr[w]
        assert U <= min(hi - lo, n_cols)
        assert m["win_partition"][w] == -(-U // W_)
        clean = m["col_to_row"][uptr[w]:uptr[w + 1]]
        assert np.all(np.diff(clean) > 0)                # ascending, each column once per window
        e2c = m["edge_to_col"][lo:hi]
        if hi > lo:
            assert e2c.min() >= 0 and e2c.max() < U
            assert np.array_equal(clean[e2c], ci[lo:hi])  # condensed id maps back to the neighbour
            assert len(np.unique(e2c)) == U              # every condensed column is used
    assert covered == len(ci)                            # tiles cover exactly nnz(A)


def test_hand_worked_example(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "four_node_example.json")))
    rp, ci = g["row_ptr"], g["col_idx"]
    for tw, exp in g["by_tile_w"].items():
        m = oracle.sgt(rp, ci, g["win_h"], int(tw))
        assert m["win_partition"].tolist() == exp["win_partition"]
        assert m["win_unique_ptr"].tolist() == g["win_unique_ptr"]
        assert m["col_to_row"].tolist() == g["col_to_row"]
        assert m["edge_to_col"].tolist() == g["edge_to_col"]
    m = oracle.sgt(rp, ci, 4, 2)
    assert m["col_to_row"].tolist() == g["one_window_h4"]["col_to_row"]
    assert m["edge_to_col"].tolist() == g["one_window_h4"]["edge_to_col"]
    assert m["win_partition"].tolist() == [2]


@pytest.mark.parametrize("n,H,W_,seed", [(5, 2, 2, 1), (17, 4, 3, 2), (40, 16, 8, 3), (64, 16, 16, 4),
                                         (33, 7, 1, 5), (48, 1, 8, 6), (50, 64, 8, 7)])
def test_brute_force_small(n, H, W_, seed):
    rng = np.random.default_rng(seed)
    A = rng.random((n, n + 3)) < 0.15                    # rectangular, asymmetric
    A[rng.integers(0, n)] = False                        # an empty row
    rp = np.concatenate([[0], np.cumsum(A.sum(1))]).astype(np.int32)
    ci = np.concatenate([np.nonzero(r)[0] for r in A]).astype(np.int32)
    m = oracle.sgt(rp, ci, H, W_)
    part, uptr, c2r, e2c = brute_force_sgt(rp, ci, n + 3, H, W_)
    assert np.array_equal(m["win_partition"], part)
    assert np.array_equal(m["win_unique_ptr"], uptr)
    assert np.array_equal(m["col_to_row"], c2r)
    assert np.array_equal(m["edge_to_col"], e2c)
    check_invariants(rp, ci, n + 3, H, W_, m)


def test_unsorted_rows_and_repeated_entries():
    # Columns inside a row in arbitrary order, one repeated (row, col) entry: the translation is
    # positional, so edge_to_col follows the given order and repeats share a condensed column.
    rp = np.array([0, 4, 6], dtype=np.int32)
    ci = np.array([9, 2, 9, 5, 5, 0], dtype=np.int32)
    m = oracle.sgt(rp, ci, 2, 2)
    assert m["col_to_row"].tolist() == [0, 2, 5, 9]
    assert m["edge_to_col"].tolist() == [3, 1, 3, 2, 2, 0]
    assert m["win_partition"].tolist() == [2]


def test_identity_closed_form():
    n, H = 100, 16
    rp = np.arange(n + 1, dtype=np.int32)
    ci = np.arange(n, dtype=np.int32)
    for W_ in (1, 4, 8, 16, 32):
        m = oracle.sgt(rp, ci, H, W_)
        Uw = np.diff(m["win_unique_ptr"])
        assert Uw.tolist() == [16] * 6 + [4]             # last window is ragged: 100 = 6*16 + 4
        assert np.array_equal(m["edge_to_col"], np.arange(n) % H)
        assert np.array_equal(m["col_to_row"], np.arange(n))
        assert np.array_equal(m["win_partition"], -(-Uw // W_))


def test_tile_width_one_and_single_window():
    c = W.make_config(1, n=256)
    g = c["csr"]
    m1 = oracle.sgt(g.row_ptr, g.col_idx, 16, 1)
    assert np.array_equal(m1["win_partition"], np.diff(m1["win_unique_ptr"]))   # W = 1: tiles = U_w
    mN = oracle.sgt(g.row_ptr, g.col_idx, g.n_rows, 8)                          # H = N: one window
    nonempty = np.unique(g.col_idx)
    assert np.array_equal(mN["col_to_row"], nonempty)
    assert np.array_equal(nonempty[mN["edge_to_col"]], g.col_idx)


def test_window_height_one_sorted_rows():
    c = W.make_config(2, n=500)
    g = c["csr"]
    m = oracle.sgt(g.row_ptr, g.col_idx, 1, 8)
    # H = 1 with sorted duplicate-free rows: nothing to share, edge k of a row is column k.
    assert np.array_equal(m["edge_to_col"], np.arange(g.nnz) - np.repeat(g.row_ptr[:-1], g.degrees()))
    assert np.array_equal(m["col_to_row"], g.col_idx)


def test_identical_rows_share_everything():
    k, H = 11, 16
    cols = np.sort(np.random.default_rng(0).choice(1000, k, replace=False)).astype(np.int32)
    rp = (np.arange(H + 1) * k).astype(np.int32)
    ci = np.tile(cols, H)
    m = oracle.sgt(rp, ci, H, 8)
    assert m["win_unique_ptr"].tolist() == [0, k]
    assert m["win_partition"].tolist() == [2]
    assert np.array_equal(m["edge_to_col"], np.tile(np.arange(k), H))


@pytest.mark.parametrize("k", [1, 2, 4, 8])
def test_dense_block_matrix_of_the_sparsity_sweep(k):
    # Table 6 of the paper: 4096 x 4096, k dense 16x16 blocks per 16-row window.  Sparsity column
    # of that table: 99.61, 99.22, 98.44, 96.88 percent for k = 1, 2, 4, 8.
    n = 4096 if k <= 2 else 1024
    g = W.dense_block_windows(n, k, seed=k)
    if n == 4096:
        printed = {1: 99.61, 2: 99.22}[k]
        assert abs(100.0 * (1 - g.nnz / n ** 2) - printed) < 0.005
    for W_ in (8, 16):
        m = oracle.sgt(g.row_ptr, g.col_idx, 16, W_)
        assert np.all(np.diff(m["win_unique_ptr"]) == 16 * k)
        assert np.all(m["win_partition"] == 16 * k // W_)
        # every condensed tile is full: density 1
        assert g.nnz == m["win_partition"].sum() * 16 * W_


@pytest.mark.parametrize("cfg,n,H,W_", [(1, 2048, 16, 8), (1, 2048, 16, 16), (2, 3000, 16, 8),
                                        (3, 2000, 16, 16), (4, 5000, 16, 32), (5, 1280, 16, 16),
                                        (4, 1003, 12, 5)])
def test_invariants_on_workload_graphs(cfg, n, H, W_):
    g = W.make_config(cfg, n=n, d=4)["csr"]
    m = oracle.sgt(g.row_ptr, g.col_idx, H, W_)
    check_invariants(g.row_ptr, g.col_idx, g.n_cols, H, W_, m)


def test_sddmm_block_count_recomputed_from_spmm_blocks():
    # Section 4.3: the same translated graph serves 16x8 operand tiles and 16x16 output tiles;
    # the 16-wide count follows from the 8-wide one.
    g = W.make_config(3, n=3000, d=4)["csr"]
    m8 = oracle.sgt(g.row_ptr, g.col_idx, 16, 8)
    m16 = oracle.sgt(g.row_ptr, g.col_idx, 16, 16)
    assert np.array_equal(m16["win_partition"], -(-m8["win_partition"] // 2))
    assert np.array_equal(m8["edge_to_col"], m16["edge_to_col"])


def test_empty_graph_and_empty_windows():
    m = oracle.sgt([0], [], 16, 8)
    assert m["win_partition"].size == 0 and m["col_to_row"].size == 0
    rp = np.zeros(40, dtype=np.int32)
    rp[20:] = 3                                             # only row 19 has entries
    m = oracle.sgt(rp, [5, 6, 7], 16, 2)
    assert m["win_partition"].tolist() == [0, 2, 0]
    assert m["win_unique_ptr"].tolist() == [0, 0, 3, 3]
