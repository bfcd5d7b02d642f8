"""GPU parity of the backward-pass building blocks against the oracle: CSR transpose (bit-exact),
two-operand SDDMM, row-softmax gradient, and the composed gradients of SpMM and SDDMM."""
import numpy as np
import pytest
import torch

import oracle
import paper_2112_02052_amd as tcg
import workloads as W

from gpu_util import TOL_F32, TOL_MFMA, dev, norm_err, upload_csr, upload_x
from test_gpu_parity import csr_from_rows, hub_graph

pytestmark = pytest.mark.gpu


def hub_and_gaps_graph():
    """A row of 10,000 entries (several whole entry tiles of the transpose's row search lie inside it), a run of
    6,000 rows without entries, and short rows around them."""
    rng = np.random.default_rng(11)
    n_cols = 20000
    rows = [rng.choice(n_cols, size=int(rng.integers(0, 4)), replace=False) for _ in range(300)]
    rows.append(rng.choice(n_cols, size=10000, replace=False))
    rows += [np.zeros(0, dtype=np.int64)] * 6000
    rows += [rng.choice(n_cols, size=int(rng.integers(1, 12)), replace=False) for _ in range(900)]
    return csr_from_rows(rows, n_cols)


def asymmetric_graph(n_rows, n_cols, seed, max_deg=40):
    rng = np.random.default_rng(seed)
    rows = [rng.choice(n_cols, size=int(rng.integers(0, max_deg)), replace=False) for _ in range(n_rows)]
    rows[1] = rng.choice(n_cols, size=min(n_cols, 700), replace=False)       # one long row
    return csr_from_rows(rows, n_cols)


@pytest.mark.parametrize("make", [lambda: asymmetric_graph(300, 5000, 1), lambda: asymmetric_graph(5000, 300, 2),
                                  lambda: hub_graph(3000), lambda: W.make_config(4, n=40000, d=2)["csr"],
                                  lambda: W.make_config(3, n=17, d=2)["csr"],
                                  lambda: asymmetric_graph(8193, 700, 3, max_deg=6),
                                  lambda: W.make_config(3, d=2)["csr"], hub_and_gaps_graph,
                                  lambda: csr_from_rows([[], [], []], 5), lambda: csr_from_rows([[2, 2, 0]], 3)])
def test_csr_transpose_bit_exact(make):
    g = make()
    rp, ci = upload_csr(g)
    rpt, cit, perm = tcg.csr_transpose(rp, ci, g.n_cols)
    torch.cuda.synchronize()
    ref = oracle.csr_transpose(g.row_ptr, g.col_idx, g.n_cols)
    assert np.array_equal(rpt.cpu().numpy(), ref[0])
    assert np.array_equal(cit.cpu().numpy(), ref[1])
    assert np.array_equal(perm.cpu().numpy(), ref[2])


def test_edge_gather_and_softmax_backward():
    g = hub_graph(2500)
    rp, ci = upload_csr(g)
    meta = tcg.sgt_build(rp, ci, 16, 8)
    rng = np.random.default_rng(0)
    v = rng.standard_normal(g.nnz).astype(np.float32) * 3
    dp = rng.standard_normal(g.nnz).astype(np.float32)
    p = tcg.row_softmax(meta, torch.from_numpy(v).to(dev()))
    dv = tcg.row_softmax_backward(meta, p, torch.from_numpy(dp).to(dev()))
    torch.cuda.synchronize()
    ref = oracle.row_softmax_backward(g.row_ptr, p.cpu().numpy().astype(np.float64), dp.astype(np.float64))
    assert norm_err(dv.cpu().numpy(), ref) <= TOL_F32
    perm = torch.from_numpy(rng.permutation(g.nnz).astype(np.int32)).to(dev())
    out = tcg.edge_gather(perm, p)
    torch.cuda.synchronize()
    assert torch.equal(out, p[perm.long()])
    meta.free()


@pytest.mark.parametrize("x_dtype,policy,tol", [("f32", tcg.POLICY_AUTO, TOL_F32), ("bf16", tcg.POLICY_GATHER, TOL_F32),
                                                ("bf16", tcg.POLICY_TILE, TOL_F32), ("f16", tcg.POLICY_TILE, TOL_F32),
                                                ("f32", tcg.POLICY_TILE, TOL_F32)])
def test_sddmm_pq(x_dtype, policy, tol):
    rnd = {"f32": lambda a: a, "bf16": W.round_to_bf16, "f16": lambda a: a.astype(np.float16).astype(np.float32)}[x_dtype]
    for g, D in ((asymmetric_graph(900, 2000, 3), 64), (asymmetric_graph(2000, 900, 4), 40),
                 (W.make_config(5, n=64 * 20, d=2, permute=False)["csr"], 256)):
        P = rnd(W.features_normal(g.n_rows, D, 1))
        Q = rnd(W.features_normal(g.n_cols, D, 2, stream=7))
        rp, ci = upload_csr(g)
        meta = tcg.sgt_build(rp, ci, 16, 16, n_cols=g.n_cols)
        tcg.sgt_set_policy(meta, policy)
        out = tcg.sddmm_pq(meta, upload_x(P, x_dtype), upload_x(Q, x_dtype))
        torch.cuda.synchronize()
        assert norm_err(out.cpu().numpy(), oracle.sddmm_pq(g.row_ptr, g.col_idx, P, Q)) <= tol
        meta.free()


def test_spmm_backward_composition():
    # Y = (w (.) A) X on an asymmetric rectangular A: dX through the transposed structure, dw by SDDMM.
    g = asymmetric_graph(1500, 2600, 5)
    D = 64
    X = W.features_normal(g.n_cols, D, 3)
    w = np.random.default_rng(1).standard_normal(g.nnz).astype(np.float32)
    G = W.features_normal(g.n_rows, D, 4, stream=9)                     # dL/dY
    rp, ci = upload_csr(g)
    meta = tcg.sgt_build(rp, ci, 16, 8, n_cols=g.n_cols)
    rpt, cit, perm = tcg.csr_transpose(rp, ci, g.n_cols)
    meta_t = tcg.sgt_build(rpt, cit, 16, 8, n_cols=g.n_rows)
    wd, Gd, Xd = torch.from_numpy(w).to(dev()), upload_x(G, "f32"), upload_x(X, "f32")
    dX = tcg.spmm(meta_t, Gd, tcg.edge_gather(perm, wd))
    dw = tcg.sddmm_pq(meta, Gd, Xd)
    torch.cuda.synchronize()
    rpt_o, cit_o, perm_o = oracle.csr_transpose(g.row_ptr, g.col_idx, g.n_cols)
    assert norm_err(dX.cpu().numpy(), oracle.spmm(rpt_o, cit_o, G, w[perm_o])) <= TOL_F32
    assert norm_err(dw.cpu().numpy(), oracle.sddmm_pq(g.row_ptr, g.col_idx, G, X)) <= TOL_F32
    meta.free()
    meta_t.free()


def test_attention_layer_backward_composition():
    # Y = (softmax(SDDMM(X)) (.) A) X, loss = sum(Y * G): every gradient step through the library,
    # compared with the same chain evaluated by the oracle.
    c = W.make_config(3, n=6000)
    g, X = c["csr"], c["X"]
    G = W.features_normal(g.n_rows, X.shape[1], 5, stream=11)
    rp, ci = upload_csr(g)
    meta = tcg.sgt_build(rp, ci, 16, 8)
    rpt, cit, perm = tcg.csr_transpose(rp, ci, g.n_cols)
    meta_t = tcg.sgt_build(rpt, cit, 16, 8)
    Xd, Gd = upload_x(X, "f32"), upload_x(G, "f32")
    e = tcg.sddmm(meta, Xd)
    p = tcg.row_softmax(meta, e)
    dp = tcg.sddmm_pq(meta, Gd, Xd)                                     # dL/dp
    de = tcg.row_softmax_backward(meta, p, dp)                          # dL/de
    dX = (tcg.spmm(meta_t, Gd, tcg.edge_gather(perm, p))                # through the aggregation
          + tcg.spmm(meta, Xd, de) + tcg.spmm(meta_t, Xd, tcg.edge_gather(perm, de)))   # through the scores
    torch.cuda.synchronize()
    e_o = oracle.sddmm(g.row_ptr, g.col_idx, X)
    p_o = oracle.row_softmax(g.row_ptr, e_o)
    dp_o = oracle.sddmm_pq(g.row_ptr, g.col_idx, G, X)
    de_o = oracle.row_softmax_backward(g.row_ptr, p_o, dp_o)
    rpt_o, cit_o, perm_o = oracle.csr_transpose(g.row_ptr, g.col_idx, g.n_cols)
    f32 = lambda a: a.astype(np.float32)
    dX_o = (oracle.spmm(rpt_o, cit_o, G, f32(p_o[perm_o])) + oracle.spmm(g.row_ptr, g.col_idx, X, f32(de_o))
            + oracle.spmm(rpt_o, cit_o, X, f32(de_o[perm_o])))
    assert norm_err(de.cpu().numpy(), de_o) <= 1e-4       # the softmax amplifies the fp32 rounding of the scores
    assert norm_err(dX.cpu().numpy(), dX_o) <= 1e-4
    meta.free()
    meta_t.free()


@pytest.mark.parametrize("x_dtype", ["f32", "bf16", "f16"])
def test_fused_attention_matches_the_three_call_chain(x_dtype):
    rnd = {"f32": lambda a: a, "bf16": W.round_to_bf16, "f16": lambda a: a.astype(np.float16).astype(np.float32)}[x_dtype]
    cases = [(W.make_config(3, n=20000), None), (W.make_config(4, n=6000, d=128), None),
             (W.make_config(5, n=64 * 30, d=256, permute=False), None), (W.make_config(1, n=700, d=16), None)]
    g_hub = hub_graph(2500)
    cases.append((dict(csr=g_hub, X=W.features_normal(g_hub.n_cols, 64, 8)), None))
    for c, _ in cases:
        g = c["csr"]
        X = rnd(c["X"] * (0.3 if x_dtype != "f32" else 1.0))         # keep 16-bit scores in a sane range
        X = rnd(X)
        rp, ci = upload_csr(g)
        meta = tcg.sgt_build(rp, ci, 16, 8)
        Xd = upload_x(X, x_dtype)
        scores = torch.full((g.nnz,), float("nan"), device=dev())
        Y = torch.full((g.n_rows, X.shape[1]), float("nan"), device=dev())
        tcg.attention(meta, Xd, Y=Y, scores=scores)
        torch.cuda.synchronize()
        e_o = oracle.sddmm(g.row_ptr, g.col_idx, X)
        p_o = oracle.row_softmax(g.row_ptr, e_o)
        Y_o = oracle.spmm(g.row_ptr, g.col_idx, X, p_o.astype(np.float32))
        assert norm_err(scores.cpu().numpy(), e_o) <= TOL_F32
        assert norm_err(Y.cpu().numpy(), Y_o) <= 1e-4
        deg = g.degrees()
        assert np.all(Y.cpu().numpy()[deg == 0] == 0)
        # the library's own three-call chain agrees (its SpMM may take the MFMA path for 16-bit features,
        # which rounds the attention weights to the feature type)
        Y3 = tcg.spmm(meta, Xd, tcg.row_softmax(meta, tcg.sddmm(meta, Xd)))
        torch.cuda.synchronize()
        assert norm_err(Y.cpu().numpy(), Y3.cpu().numpy().astype(np.float64)) <= (1e-4 if x_dtype == "f32" else TOL_MFMA)
        meta.free()


@pytest.mark.parametrize("x_dtype", ["f32", "bf16"])
def test_cosine_attention_matches_the_chain_on_normalised_rows(x_dtype):
    # tcg_row_rnorm + tcg_attention_cos against the oracle's chain: c_e = <x_i, x_j> / (|x_i| |x_j|) (the oracle's
    # SDDMM scaled in double), row softmax of beta * c, aggregation of the unnormalised rows.  Hub rows (split
    # segments merged under the online softmax), empty rows and one all-zero feature row included.
    c = W.make_config(3, n=20000, d=32)
    g = c["csr"]
    X = W.round_to_bf16(c["X"]) if x_dtype == "bf16" else c["X"].copy()
    X[17, :] = 0.0
    beta = 1.7
    rp, ci = upload_csr(g)
    Xd = upload_x(X, x_dtype)
    meta = tcg.sgt_build(rp, ci, 16, 8)
    r = tcg.row_rnorm(Xd)
    nrm = np.sqrt((X.astype(np.float64) ** 2).sum(axis=1))
    r_ref = 1.0 / np.maximum(nrm, 1e-12)
    assert norm_err(r.cpu().numpy()[nrm > 0], r_ref[nrm > 0]) <= TOL_F32
    cs = torch.empty(g.nnz, device=dev())
    Y = tcg.attention_cos(meta, Xd, r, beta, scores=cs)
    torch.cuda.synchronize()
    rows = np.repeat(np.arange(g.n_rows), np.diff(g.row_ptr))
    c_ref = oracle.sddmm(g.row_ptr, g.col_idx, X) * r_ref[rows] * r_ref[g.col_idx]
    p_ref = oracle.row_softmax(g.row_ptr, beta * c_ref)
    Y_ref = oracle.spmm(g.row_ptr, g.col_idx, X, p_ref.astype(np.float32))
    assert norm_err(cs.cpu().numpy(), c_ref) <= TOL_F32
    assert norm_err(Y.cpu().numpy(), Y_ref) <= 1e-4            # the chain's end-to-end bound (exp of an fp32 score)
    meta.free()


@pytest.mark.parametrize("x_dtype,D", [("f32", 32), ("f32", 50), ("bf16", 64), ("f32", 3)])
def test_row_unit_grad(x_dtype, D):
    """tcg_row_unit_grad against the oracle, accumulated into a non-zero dX, with a zero row (clamped norm)."""
    import oracle.layers as L
    rng = np.random.default_rng(5)
    n = 1000
    X = rng.standard_normal((n, D)).astype(np.float32)
    X[17] = 0.0
    if x_dtype == "bf16":
        X = W.round_to_bf16(X)
    G = rng.standard_normal((n, D)).astype(np.float32)
    base = rng.standard_normal((n, D)).astype(np.float32)
    Xd = upload_x(X, x_dtype)
    r = tcg.row_rnorm(Xd)
    dX = torch.from_numpy(base.copy()).to(dev())
    tcg.row_unit_grad(Xd, r, torch.from_numpy(G).to(dev()), dX, scale=0.7)
    torch.cuda.synchronize()
    ref = base.astype(np.float64) + L.row_unit_grad(X, G, scale=0.7)
    got = dX.cpu().numpy()
    keep = np.arange(n) != 17
    assert norm_err(got[keep], ref[keep]) <= TOL_F32
    assert np.allclose(got[17], ref[17], rtol=1e-5)          # the clamped row: G / eps, far above the others

