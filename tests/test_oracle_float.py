"""Pins for the oracle's SpMM (Equation 1), SDDMM (Equation 2), row softmax and the
tile-form executions of Algorithms 2 and 3.  Checks are against dense matrix algebra done
by numpy on tiny graphs, closed forms and the hand-worked example -- never against a second
copy of the oracle's loops."""
import json
import os

import numpy as np
import pytest

import oracle
import workloads as W


def random_csr(n_rows, n_cols, p, seed, sort_rows=True):
    rng = np.random.default_rng(seed)
    A = rng.random((n_rows, n_cols)) < p
    rp = np.concatenate([[0], np.cumsum(A.sum(1))]).astype(np.int32)
    rows = []
    for r in A:
        c = np.nonzero(r)[0]
        if not sort_rows:
            c = rng.permutation(c)
        rows.append(c)
    ci = np.concatenate(rows).astype(np.int32) if rp[-1] else np.zeros(0, np.int32)
    return A, rp, ci


def dense_weighted(rp, ci, w, shape):
    M = np.zeros(shape, dtype=np.float64)
    for i in range(len(rp) - 1):
        for e in range(rp[i], rp[i + 1]):
            M[i, ci[e]] += 1.0 if w is None else float(w[e])
    return M


def test_hand_worked_example(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "four_node_example.json")))
    X = np.array(g["X"], dtype=np.float32)
    assert oracle.spmm(g["row_ptr"], g["col_idx"], X).tolist() == g["spmm_unit"]
    assert oracle.spmm(g["row_ptr"], g["col_idx"], X, g["w"]).tolist() == g["spmm_weighted"]
    assert oracle.sddmm(g["row_ptr"], g["col_idx"], X).tolist() == g["sddmm"]


@pytest.mark.parametrize("n,m,D,p,seed,weighted", [(7, 9, 3, 0.4, 0, False), (33, 20, 5, 0.2, 1, True),
                                                    (64, 64, 16, 0.1, 2, True), (20, 50, 1, 0.3, 3, False)])
def test_spmm_equals_dense_product(n, m, D, p, seed, weighted):
    _, rp, ci = random_csr(n, m, p, seed, sort_rows=False)
    rng = np.random.default_rng(seed + 100)
    X = rng.standard_normal((m, D)).astype(np.float32)
    w = rng.standard_normal(len(ci)).astype(np.float32) if weighted else None
    Y = oracle.spmm(rp, ci, X, w)
    ref = dense_weighted(rp, ci, w, (n, m)) @ X.astype(np.float64)     # asymmetric: a transposed
    np.testing.assert_allclose(Y, ref, rtol=1e-13, atol=1e-13)          # operand would fail here


@pytest.mark.parametrize("n,D,p,seed", [(6, 2, 0.5, 0), (40, 7, 0.2, 1), (64, 32, 0.1, 2)])
def test_sddmm_equals_sampled_gram_matrix(n, D, p, seed):
    A, rp, ci = random_csr(n, n, p, seed, sort_rows=False)
    X = np.random.default_rng(seed + 7).standard_normal((n, D)).astype(np.float32)
    out = oracle.sddmm(rp, ci, X)
    G = X.astype(np.float64) @ X.astype(np.float64).T
    rows = np.repeat(np.arange(n), np.diff(rp))
    np.testing.assert_allclose(out, G[rows, ci], rtol=1e-13, atol=1e-13)
    # scatter back: (X X^T) (.) A
    F = np.zeros((n, n))
    F[rows, ci] = out
    np.testing.assert_allclose(F, G * A, rtol=1e-13, atol=1e-13)


def test_spmm_identity_and_ones():
    n, D = 50, 6
    X = np.random.default_rng(0).standard_normal((n, D)).astype(np.float32)
    rp = np.arange(n + 1, dtype=np.int32)
    ci = np.arange(n, dtype=np.int32)
    assert np.array_equal(oracle.spmm(rp, ci, X), X.astype(np.float64))       # A = I
    c = W.make_config(2, n=700, d=3)
    g, w = c["csr"], c["w"]
    ones = np.ones((g.n_rows, 3), dtype=np.float32)
    Y = oracle.spmm(g.row_ptr, g.col_idx, ones)
    assert np.array_equal(Y[:, 0], g.degrees().astype(np.float64))            # X = 1: degree
    Yw = oracle.spmm(g.row_ptr, g.col_idx, ones, w)
    wsum = np.add.reduceat(w.astype(np.float64), g.row_ptr[:-1])              # all rows non-empty
    np.testing.assert_allclose(Yw[:, 2], wsum, rtol=1e-14)


@pytest.mark.parametrize("cfg,n", [(1, 2048), (2, 20000)])
def test_symmetric_normalisation_eigenvector(cfg, n):
    # With self-loops, w_ij = 1/sqrt(deg_i deg_j) and X[:, d] = sqrt(deg):
    # sum_j w_ij sqrt(deg_j) = deg_i / sqrt(deg_i) = sqrt(deg_i), so Y = X at full workload size.
    c = W.make_config(cfg, n=n, d=2)
    g = c["csr"]
    s = np.sqrt(g.degrees().astype(np.float64))
    X = np.stack([s, -2.0 * s], axis=1).astype(np.float32)
    Y = oracle.spmm(g.row_ptr, g.col_idx, X, c["w"])
    np.testing.assert_allclose(Y, X.astype(np.float64), rtol=2e-6)            # fp32 inputs


def test_sddmm_special_cases():
    g = W.make_config(1, n=512, d=4)["csr"]
    rows = g.row_of_edge()
    rng = np.random.default_rng(3)
    labels = rng.integers(0, 5, g.n_rows)
    onehot = np.eye(5, dtype=np.float32)[labels]
    out = oracle.sddmm(g.row_ptr, g.col_idx, onehot)
    assert np.array_equal(out, (labels[rows] == labels[g.col_idx]).astype(np.float64))
    X = rng.standard_normal((g.n_rows, 9)).astype(np.float32)
    out = oracle.sddmm(g.row_ptr, g.col_idx, X)
    loops = rows == g.col_idx
    np.testing.assert_allclose(out[loops], (X.astype(np.float64) ** 2).sum(1), rtol=1e-14)
    # symmetric structure: the value on (i, j) equals the value on (j, i)
    key = {(int(i), int(j)): v for i, j, v in zip(rows, g.col_idx, out)}
    assert all(key[(j, i)] == v for (i, j), v in key.items())


def test_linearity_on_integer_inputs():
    g = W.make_config(3, n=1500, d=4)["csr"]
    rng = np.random.default_rng(0)
    X1 = rng.integers(-8, 9, (g.n_rows, 8)).astype(np.float32)
    X2 = rng.integers(-8, 9, (g.n_rows, 8)).astype(np.float32)
    assert np.array_equal(oracle.spmm(g.row_ptr, g.col_idx, X1 + X2),
                          oracle.spmm(g.row_ptr, g.col_idx, X1) + oracle.spmm(g.row_ptr, g.col_idx, X2))


def test_row_softmax():
    g = W.make_config(3, n=1200, d=4)["csr"]
    v = np.random.default_rng(1).standard_normal(g.nnz) * 5
    p = oracle.row_softmax(g.row_ptr, v)
    deg = g.degrees()
    sums = np.zeros(g.n_rows)
    np.add.at(sums, g.row_of_edge(), p)
    np.testing.assert_allclose(sums[deg > 0], 1.0, rtol=1e-13)
    assert np.all(sums[deg == 0] == 0) and (deg == 0).any()
    assert np.all(p > 0)
    np.testing.assert_allclose(oracle.row_softmax(g.row_ptr, v + 3.25), p, rtol=1e-12)   # shift invariance
    # closed form for a row with two entries: logistic of the difference
    q = oracle.row_softmax([0, 2, 3], [0.3, -1.1, 42.0])
    np.testing.assert_allclose(q, [1 / (1 + np.exp(-1.4)), 1 / (1 + np.exp(1.4)), 1.0], rtol=1e-14)
    # huge values do not overflow thanks to the max subtraction
    q = oracle.row_softmax([0, 2], [1000.0, 1000.0])
    assert q.tolist() == [0.5, 0.5]
    # softmax weights then SpMM of ones: every non-empty row aggregates to exactly ~1
    Y = oracle.spmm(g.row_ptr, g.col_idx, np.ones((g.n_rows, 1), np.float32), p.astype(np.float32))
    np.testing.assert_allclose(Y[deg > 0, 0], 1.0, rtol=1e-6)


@pytest.mark.parametrize("cfg,n,H,W_,D", [(1, 300, 16, 8, 5), (3, 900, 16, 8, 4), (5, 640, 16, 16, 3),
                                          (2, 333, 7, 3, 2), (4, 1000, 16, 32, 2)])
def test_tile_form_reproduces_csr_form(cfg, n, H, W_, D):
    # The translation keeps the result exact (sections 1 and 4.1): Algorithms 2 and 3 run from the
    # translated graph give what Equations 1 and 2 give.
    c = W.make_config(cfg, n=n, d=D)
    g, X = c["csr"], c["X"]
    w = np.random.default_rng(0).standard_normal(g.nnz).astype(np.float32)
    m = oracle.sgt(g.row_ptr, g.col_idx, H, W_)
    Yt = oracle.spmm_tiled(g.row_ptr, g.col_idx, m["edge_to_col"], m["win_partition"], H, W_, X, w)
    np.testing.assert_allclose(Yt, oracle.spmm(g.row_ptr, g.col_idx, X, w), rtol=1e-12, atol=1e-12)
    Et = oracle.sddmm_tiled(g.row_ptr, g.col_idx, m["edge_to_col"], H, W_, X)
    np.testing.assert_allclose(Et, oracle.sddmm(g.row_ptr, g.col_idx, X), rtol=1e-13, atol=1e-13)


def test_tile_form_detects_bad_metadata():
    c = W.make_config(1, n=128, d=2)
    g = c["csr"]
    m = oracle.sgt(g.row_ptr, g.col_idx, 16, 8)
    short = m["win_partition"].copy()
    short[0] -= 1                                            # one block too few for window 0
    with pytest.raises(ValueError):
        oracle.spmm_tiled(g.row_ptr, g.col_idx, m["edge_to_col"], short, 16, 8, c["X"])


def test_repeated_entries_add_up():
    rp, ci = [0, 3], [1, 1, 0]
    X = np.array([[1.0], [10.0]], dtype=np.float32)
    assert oracle.spmm(rp, ci, X).tolist() == [[21.0]]
    assert oracle.sddmm([0, 3, 3], ci, X).tolist() == [10.0, 10.0, 1.0]
