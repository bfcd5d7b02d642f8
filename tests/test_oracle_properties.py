"""Property tests of the oracles on random small inputs (hypothesis): the invariants that tie the
translated graph to the CSR it came from, the equality of the tiled and the plain forms, and the
invariants of the row clustering."""
import numpy as np
from hypothesis import given, settings, strategies as st

import oracle
import oracle.reorder as R


@st.composite
def csr_graphs(draw, square=False):
    n_rows = draw(st.integers(1, 40))
    n_cols = n_rows if square else draw(st.integers(1, 40))
    rows = [draw(st.lists(st.integers(0, n_cols - 1), max_size=12)) for _ in range(n_rows)]
    rp = np.concatenate([[0], np.cumsum([len(r) for r in rows])]).astype(np.int32)
    ci = np.array([c for r in rows for c in r], dtype=np.int32)
    return n_rows, n_cols, rp, ci


@settings(max_examples=60, deadline=None)
@given(csr_graphs(), st.integers(1, 20), st.integers(1, 9))
def test_sgt_invariants(graph, H, Wt):
    n_rows, n_cols, rp, ci = graph
    m = oracle.sgt(rp, ci, H, Wt)
    n_win = (n_rows + H - 1) // H
    up = m["win_unique_ptr"]
    assert len(m["win_partition"]) == n_win and up[0] == 0 and up[-1] == len(m["col_to_row"])
    for w in range(n_win):
        lo, hi = rp[w * H], rp[min((w + 1) * H, n_rows)]
        clean = m["col_to_row"][up[w]:up[w + 1]]
        assert np.all(np.diff(clean) > 0)                                     # every column once, ascending
        assert set(clean.tolist()) == set(ci[lo:hi].tolist())                 # exactly the window's columns
        assert m["win_partition"][w] == (len(clean) + Wt - 1) // Wt
        e2c = m["edge_to_col"][lo:hi]
        assert np.array_equal(clean[e2c], ci[lo:hi])                          # the map leads back to the column


@settings(max_examples=40, deadline=None)
@given(csr_graphs(), st.integers(1, 17), st.integers(1, 9), st.integers(0, 2 ** 31 - 1))
def test_tiled_forms_equal_plain_forms(graph, H, Wt, seed):
    n_rows, n_cols, rp, ci = graph
    rng = np.random.default_rng(seed)
    X = rng.integers(-4, 5, size=(max(n_rows, n_cols), 3)).astype(np.float32)      # integer values: exact sums
    w = rng.integers(-3, 4, size=len(ci)).astype(np.float32)
    m = oracle.sgt(rp, ci, H, Wt)
    Y = oracle.spmm(rp, ci, X, w)
    Yt = oracle.spmm_tiled(rp, ci, m["edge_to_col"], m["win_partition"], H, Wt, X, w)
    assert np.array_equal(Y, Yt)
    if n_rows == n_cols or n_cols <= n_rows:
        e = oracle.sddmm(rp, ci, X)
        et = oracle.sddmm_tiled(rp, ci, m["edge_to_col"], H, Wt, X)
        assert np.array_equal(e, et)


@settings(max_examples=40, deadline=None)
@given(csr_graphs(square=True), st.integers(0, 2 ** 40), st.integers(0, 3))
def test_row_clustering_invariants(graph, seed, refine):
    n, _, rp, ci = graph
    perm, label, parent = R.reorder_rows(rp, ci, seed=seed, refine=refine)
    perm2, label2, parent2 = R.reorder_rows_loops(rp, ci, seed=seed, refine=refine)
    assert np.array_equal(perm, perm2) and np.array_equal(label, label2) and np.array_equal(parent, parent2)
    assert sorted(perm.tolist()) == list(range(n))
    nrp, nci, ep = R.csr_permute(rp, ci, perm)
    assert sorted(ep.tolist()) == list(range(len(ci)))
    inv = np.empty(n, np.int64)
    inv[perm] = np.arange(n)
    assert np.array_equal(nci, inv[ci[ep]])
