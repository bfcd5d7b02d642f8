"""Pins for the oracle's backward-pass building blocks: CSR transpose, two-operand SDDMM, row-softmax
gradient, and the gradient formulas composed from them (the chain rule applied to Equations 1 and 2).
Gradients are checked against central finite differences of the forward oracles."""
import numpy as np
import pytest

import oracle
import workloads as W


def small_graph(n_rows, n_cols, p, seed, dup=False):
    rng = np.random.default_rng(seed)
    A = rng.random((n_rows, n_cols)) < p
    rows = [rng.permutation(np.nonzero(r)[0]) for r in A]      # unsorted columns inside a row
    if dup and len(rows[0]):
        rows[0] = np.concatenate([rows[0], rows[0][:1]])       # one repeated entry
    rp = np.concatenate([[0], np.cumsum([len(r) for r in rows])]).astype(np.int32)
    ci = np.concatenate(rows).astype(np.int32)
    return rp, ci


def dense_of(rp, ci, vals, shape):
    M = np.zeros(shape)
    for i in range(len(rp) - 1):
        for e in range(rp[i], rp[i + 1]):
            M[i, ci[e]] += vals[e]
    return M


@pytest.mark.parametrize("n_rows,n_cols,p,seed", [(5, 7, 0.5, 0), (30, 12, 0.3, 1), (12, 30, 0.2, 2), (40, 40, 0.1, 3)])
def test_transpose_against_dense(n_rows, n_cols, p, seed):
    rp, ci = small_graph(n_rows, n_cols, p, seed, dup=True)
    nnz = len(ci)
    vals = np.random.default_rng(seed).standard_normal(nnz)
    rpt, cit, perm = oracle.csr_transpose(rp, ci, n_cols)
    assert rpt.shape == (n_cols + 1,) and rpt[0] == 0 and rpt[-1] == nnz
    assert sorted(perm.tolist()) == list(range(nnz))                      # a permutation of the entries
    rows_of = np.repeat(np.arange(n_rows), np.diff(rp))
    assert np.array_equal(cit, rows_of[perm])                             # entry k is entry perm[k] of the input
    assert np.array_equal(np.repeat(np.arange(n_cols), np.diff(rpt)), ci[perm])
    np.testing.assert_array_equal(dense_of(rpt, cit, vals[perm], (n_cols, n_rows)),
                                  dense_of(rp, ci, vals, (n_rows, n_cols)).T)
    # inside a transposed row: ascending input row, input order among equals (the unique stable result)
    for c in range(n_cols):
        seg = perm[rpt[c]:rpt[c + 1]]
        assert np.all(np.diff(seg) > 0)
    # transposing twice gives the row-major order with sorted positions back
    rptt, citt, perm2 = oracle.csr_transpose(rpt, cit, n_rows)
    assert np.array_equal(rptt, rp)
    np.testing.assert_array_equal(dense_of(rptt, citt, vals[perm][perm2], (n_rows, n_cols)),
                                  dense_of(rp, ci, vals, (n_rows, n_cols)))


def test_transpose_of_symmetric_workload_is_itself():
    g = W.make_config(1, n=300, d=2)["csr"]
    rpt, cit, perm = oracle.csr_transpose(g.row_ptr, g.col_idx, g.n_cols)
    assert np.array_equal(rpt, g.row_ptr) and np.array_equal(cit, g.col_idx)
    assert not np.array_equal(perm, np.arange(g.nnz))


def test_sddmm_pq_against_dense_and_special_cases():
    rp, ci = small_graph(9, 14, 0.4, 5)
    rng = np.random.default_rng(0)
    P = rng.standard_normal((9, 6)).astype(np.float32)
    Q = rng.standard_normal((14, 6)).astype(np.float32)
    out = oracle.sddmm_pq(rp, ci, P, Q)
    G = P.astype(np.float64) @ Q.astype(np.float64).T
    rows = np.repeat(np.arange(9), np.diff(rp))
    np.testing.assert_allclose(out, G[rows, ci], rtol=1e-13, atol=1e-13)    # P Q^T sampled; swapping P and Q fails
    g = W.make_config(3, n=400, d=5)
    X = g["X"]
    assert np.array_equal(oracle.sddmm_pq(g["csr"].row_ptr, g["csr"].col_idx, X, X),
                          oracle.sddmm(g["csr"].row_ptr, g["csr"].col_idx, X))


def num_grad(f, x, eps=1e-3):
    """Central differences of a scalar function of a float32 array (perturbed in float32)."""
    g = np.zeros(x.shape, dtype=np.float64)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        idx = it.multi_index
        old = x[idx]
        x[idx] = old + eps
        hi = f(x)
        up = float(x[idx])
        x[idx] = old - eps
        lo = f(x)
        dn = float(x[idx])
        x[idx] = old
        g[idx] = (hi - lo) / (up - dn)
    return g


def test_spmm_gradients_by_finite_differences():
    rp, ci = small_graph(7, 9, 0.4, 11, dup=True)
    rng = np.random.default_rng(1)
    X = rng.standard_normal((9, 3)).astype(np.float32)
    w = rng.standard_normal(len(ci)).astype(np.float32)
    G = rng.standard_normal((7, 3)).astype(np.float32)              # dL/dY for L = sum(Y * G)
    loss = lambda X_, w_: float((oracle.spmm(rp, ci, X_, w_) * G).sum())
    rpt, cit, perm = oracle.csr_transpose(rp, ci, 9)
    dX = oracle.spmm(rpt, cit, G, w[perm])                          # (w (.) A)^T G
    dw = oracle.sddmm_pq(rp, ci, G, X)                              # <G_i, X_j> per entry
    np.testing.assert_allclose(dX, num_grad(lambda X_: loss(X_, w), X.copy()), rtol=2e-3, atol=2e-3)
    np.testing.assert_allclose(dw, num_grad(lambda w_: loss(X, w_), w.copy()), rtol=2e-3, atol=2e-3)


def test_sddmm_gradient_by_finite_differences():
    rp, ci = small_graph(8, 8, 0.4, 12)
    rng = np.random.default_rng(2)
    X = rng.standard_normal((8, 4)).astype(np.float32)
    gout = rng.standard_normal(len(ci)).astype(np.float32)          # dL/dout for L = sum(out * gout)
    loss = lambda X_: float((oracle.sddmm(rp, ci, X_) * gout).sum())
    rpt, cit, perm = oracle.csr_transpose(rp, ci, 8)
    dX = oracle.spmm(rp, ci, X, gout) + oracle.spmm(rpt, cit, X, gout[perm])
    np.testing.assert_allclose(dX, num_grad(loss, X.copy()), rtol=2e-3, atol=2e-3)


def test_row_softmax_gradient_by_finite_differences():
    rp = np.array([0, 3, 3, 7, 8], dtype=np.int32)
    rng = np.random.default_rng(3)
    v = rng.standard_normal(8)
    dp = rng.standard_normal(8)
    p = oracle.row_softmax(rp, v)
    dv = oracle.row_softmax_backward(rp, p, dp)
    num = np.zeros(8)
    for k in range(8):
        e = np.zeros(8)
        e[k] = 1e-6
        num[k] = ((oracle.row_softmax(rp, v + e) - oracle.row_softmax(rp, v - e)) * dp).sum() / 2e-6
    np.testing.assert_allclose(dv, num, rtol=1e-6, atol=1e-8)
    assert abs(dv[:3].sum()) < 1e-12 and abs(dv[3:7].sum()) < 1e-12   # softmax gradients sum to zero per row
    assert dv[7] == 0.0                                               # a one-entry row is constant
