"""Pins for the layer oracle (oracle/layers.py: dense fp64 definitions differentiated by PyTorch) against
things it does not share code with: the CSR oracle in C (itself pinned elsewhere), closed forms, a
hand-worked two-node case and central finite differences."""
import numpy as np
import pytest

import oracle
import oracle.layers as L
import workloads as W


def graph(n, p, seed, self_loops=True):
    rng = np.random.default_rng(seed)
    A = rng.random((n, n)) < p
    if self_loops:
        A |= np.eye(n, dtype=bool)
    rows = [rng.permutation(np.nonzero(r)[0]) for r in A]
    rp = np.concatenate([[0], np.cumsum([len(r) for r in rows])]).astype(np.int32)
    ci = np.concatenate(rows).astype(np.int32) if rp[-1] else np.zeros(0, np.int32)
    return rp, ci


def f32(a):
    return np.asarray(a, dtype=np.float32)


def test_two_node_attention_by_hand():
    # rows: 0 -> {0, 1}, 1 -> {1};  X = I.  Scores of row 0 are (1, 0), so P = (e, 1) / (e + 1) and
    # H_0 = (e, 1) / (e + 1); row 1 has a single entry, P = 1 and H_1 = x_1.
    rp = np.array([0, 2, 3], np.int32)
    ci = np.array([0, 1, 1], np.int32)
    X = np.eye(2)
    H, P, dX = L.self_attention(rp, ci, X, np.zeros((2, 2)))
    e = np.e
    np.testing.assert_allclose(P, [e / (e + 1), 1 / (e + 1), 1.0], rtol=1e-14)
    np.testing.assert_allclose(H, [[e / (e + 1), 1 / (e + 1)], [0.0, 1.0]], rtol=1e-14)
    assert np.all(dX == 0)
    # AGNN with beta = 0 ignores the features: uniform attention over each row's entries
    H, P, dX, dbeta = L.agnn_conv(rp, ci, np.array([[3.0, 1.0], [-2.0, 5.0]]), 0.0, np.ones((2, 2)))
    np.testing.assert_allclose(P, [0.5, 0.5, 1.0], rtol=1e-14)
    np.testing.assert_allclose(H, [[0.5, 3.0], [-2.0, 5.0]], rtol=1e-14)


def test_rejects_repeated_entries():
    with pytest.raises(ValueError):
        L.dense_pattern(np.array([0, 2], np.int32), np.array([0, 0], np.int32), 1)


@pytest.mark.parametrize("n,p,seed", [(17, 0.3, 0), (60, 0.1, 1)])
def test_spmm_and_sddmm_gradients_against_the_csr_oracle(n, p, seed):
    rp, ci = graph(n, p, seed, self_loops=False)
    rng = np.random.default_rng(seed)
    X = f32(rng.standard_normal((n, 5)))
    w = f32(rng.standard_normal(len(ci)))
    dY = f32(rng.standard_normal((n, 5)))
    Y, dX, dw = L.spmm_grads(rp, ci, n, w, X, dY)
    np.testing.assert_allclose(Y, oracle.spmm(rp, ci, X, w), rtol=1e-12, atol=1e-12)
    rpt, cit, perm = oracle.csr_transpose(rp, ci, n)
    np.testing.assert_allclose(dX, oracle.spmm(rpt, cit, dY, w[perm]), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dw, oracle.sddmm_pq(rp, ci, dY, X), rtol=1e-12, atol=1e-12)
    ds = rng.standard_normal(len(ci))
    s, dXs = L.sddmm_grads(rp, ci, X, ds)
    np.testing.assert_allclose(s, oracle.sddmm(rp, ci, X), rtol=1e-12, atol=1e-12)
    ref = oracle.spmm(rp, ci, X, f32(ds)) + oracle.spmm(rpt, cit, X, f32(ds)[perm])
    np.testing.assert_allclose(dXs, ref, rtol=1e-5, atol=1e-5)        # ds was rounded to fp32 for the C oracle


def test_attention_layers_against_the_csr_oracle_chain():
    n = 40
    rp, ci = graph(n, 0.15, 3)
    rng = np.random.default_rng(3)
    X = f32(rng.standard_normal((n, 6)))
    H, P, _ = L.self_attention(rp, ci, X, np.zeros((n, 6)))
    p_ref = oracle.row_softmax(rp, oracle.sddmm(rp, ci, X))
    np.testing.assert_allclose(P, p_ref, rtol=1e-12)
    np.testing.assert_allclose(H, oracle.spmm(rp, ci, X, f32(p_ref)), rtol=1e-6, atol=1e-6)
    beta = 1.7
    Xn = f32(X / np.linalg.norm(X.astype(np.float64), axis=1, keepdims=True))
    H, P, _, _ = L.agnn_conv(rp, ci, X, beta, np.zeros((n, 6)))
    p_ref = oracle.row_softmax(rp, beta * oracle.sddmm(rp, ci, Xn))
    np.testing.assert_allclose(P, p_ref, rtol=1e-5)                   # Xn was rounded to fp32 for the C oracle
    np.testing.assert_allclose(H, oracle.spmm(rp, ci, X, f32(p_ref)), rtol=1e-5, atol=1e-5)


def central(f, x, h=1e-5):
    g = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        k = it.multi_index
        xp, xm = x.copy(), x.copy()
        xp[k] += h
        xm[k] -= h
        g[k] = (f(xp) - f(xm)) / (2 * h)
    return g


def test_attention_gradients_by_finite_differences():
    n, d = 9, 3
    rp, ci = graph(n, 0.3, 5)
    rng = np.random.default_rng(5)
    X = rng.standard_normal((n, d))
    dH = rng.standard_normal((n, d))
    zeros = np.zeros((n, d))
    _, _, dX = L.self_attention(rp, ci, X, dH)
    num = central(lambda x: float((L.self_attention(rp, ci, x, zeros)[0] * dH).sum()), X)
    np.testing.assert_allclose(dX, num, rtol=1e-6, atol=1e-8)
    beta = 0.8
    _, _, dX, dbeta = L.agnn_conv(rp, ci, X, beta, dH)
    num = central(lambda x: float((L.agnn_conv(rp, ci, x, beta, zeros)[0] * dH).sum()), X)
    np.testing.assert_allclose(dX, num, rtol=1e-6, atol=1e-8)
    numb = central(lambda b: float((L.agnn_conv(rp, ci, X, float(b[0]), zeros)[0] * dH).sum()), np.array([beta]))
    np.testing.assert_allclose(dbeta, numb[0], rtol=1e-6)


def test_gcn_layer_closed_form_and_gradients():
    # With 1/sqrt(deg_i deg_j) edge values, X[:, d] = sqrt(deg) is a fixed point of the aggregation:
    # identity weights give H = X + b.
    c = W.make_config(1, n=200, d=4)
    g, w = c["csr"], c["w"]
    s = np.sqrt(g.degrees().astype(np.float64))
    X = np.repeat(s[:, None], 4, axis=1)
    b = np.array([0.5, -1.0, 2.0, 0.0])
    rng = np.random.default_rng(0)
    dH = rng.standard_normal((200, 4))
    H, dX, dW, db, dw = L.gcn_conv(g.row_ptr, g.col_idx, g.n_cols, w, X, np.eye(4), b, dH)
    np.testing.assert_allclose(H, X + b, rtol=1e-6)                   # the edge values are fp32
    np.testing.assert_allclose(db, dH.sum(axis=0), rtol=1e-12)
    # dW = (A dH)^T X for symmetric A;  dX = A^T dH W;  dw_e = <dH_i, (X W^T)_j>
    AdH = oracle.spmm(g.row_ptr, g.col_idx, f32(dH), w)
    np.testing.assert_allclose(dW, AdH.T @ X, rtol=1e-5, atol=1e-5)
    np.testing.assert_allclose(dX, AdH, rtol=1e-5, atol=1e-5)
    np.testing.assert_allclose(dw, oracle.sddmm_pq(g.row_ptr, g.col_idx, f32(dH), f32(X)), rtol=1e-5, atol=1e-5)


def test_model_gradients_by_finite_differences():
    n = 12
    rp, ci = graph(n, 0.25, 7)
    rng = np.random.default_rng(7)
    w = rng.random(len(ci)) + 0.1
    X = rng.standard_normal((n, 5))
    dOut = rng.standard_normal((n, 3))
    params = [rng.standard_normal((4, 5)) * 0.5, rng.standard_normal(4) * 0.1,
              rng.standard_normal((3, 4)) * 0.5, rng.standard_normal(3) * 0.1]
    out, grads = L.gcn_model(rp, ci, w, X, params, dOut)
    np.testing.assert_allclose(np.exp(out).sum(axis=1), 1.0, rtol=1e-12)   # log-softmax rows
    for k in (0, 3):
        def f(v, k=k):
            q = list(params)
            q[k] = v
            return float((L.gcn_model(rp, ci, w, X, q, dOut)[0] * dOut).sum())
        np.testing.assert_allclose(grads[k], central(f, params[k]), rtol=1e-5, atol=1e-7)
    betas = [1.0, 0.5]
    out, grads = L.agnn_model(rp, ci, X, params, betas, dOut)
    assert len(grads) == 6
    for k in (0, 2):
        def f(v, k=k):
            q = list(params)
            q[k] = v
            return float((L.agnn_model(rp, ci, X, q, betas, dOut)[0] * dOut).sum())
        np.testing.assert_allclose(grads[k], central(f, params[k]), rtol=1e-5, atol=1e-7)

    def fb(v):
        return float((L.agnn_model(rp, ci, X, params, [float(v[0]), betas[1]], dOut)[0] * dOut).sum())
    np.testing.assert_allclose(grads[4], central(fb, np.array([betas[0]]))[0], rtol=1e-5)


def test_row_unit_grad_against_reverse_mode_and_closed_forms():
    """Pins of oracle.layers.row_unit_grad: the vector-Jacobian product of torch's own row normalisation, its
    orthogonality to the row (the derivative of a unit vector has no component along it), zero for a gradient
    along the row, plain scaling for a gradient across it, and central finite differences of x -> x / |x|."""
    import torch
    rng = np.random.default_rng(0)
    X = rng.standard_normal((7, 5))
    G = rng.standard_normal((7, 5))
    got = L.row_unit_grad(X, G, scale=1.7)
    Xt = torch.tensor(X, requires_grad=True)
    torch.nn.functional.normalize(Xt, p=2.0, dim=1).backward(torch.tensor(G))
    assert np.allclose(got, 1.7 * Xt.grad.numpy(), rtol=1e-12, atol=1e-14)
    assert np.abs((got * X).sum(axis=1)).max() < 1e-12
    assert np.abs(L.row_unit_grad(X, 3.0 * X)).max() < 1e-12
    x = np.array([[3.0, 4.0, 0.0]])
    assert np.allclose(L.row_unit_grad(x, np.array([[0.0, 0.0, 2.0]])), [[0.0, 0.0, 0.4]])        # across: G / |x|
    h = 1e-6
    fd = np.zeros((1, 3))
    g = np.array([[0.3, -1.1, 0.7]])
    for d in range(3):
        e = np.zeros((1, 3))
        e[0, d] = h
        up, dn = (x + e) / np.linalg.norm(x + e), (x - e) / np.linalg.norm(x - e)
        fd[0, d] = ((up - dn) / (2 * h) * g).sum()
    assert np.allclose(L.row_unit_grad(x, g), fd, atol=1e-8)


def test_isolated_nodes_and_zero_rows():
    # node 2 has no entries: its output row is zero, and in a second propagation its zero feature row
    # must neither produce NaN nor receive a gradient through the normalisation.
    rp = np.array([0, 2, 3, 3], np.int32)
    ci = np.array([0, 2, 1], np.int32)
    X = np.array([[1.0, 2.0], [0.5, -1.0], [0.0, 0.0]])
    dH = np.ones((3, 2))
    H, P, dX, dbeta = L.agnn_conv(rp, ci, X, 1.0, dH)
    assert np.all(H[2] == 0) and np.isfinite(dX).all() and np.isfinite(dbeta)
    # row 0 attends to itself (cos = 1) and to the zero row (cos = 0): P = (e, 1) / (e + 1)
    np.testing.assert_allclose(P, [np.e / (np.e + 1), 1 / (np.e + 1), 1.0], rtol=1e-14)
    np.testing.assert_allclose(H[0], np.e / (np.e + 1) * X[0], rtol=1e-14)
