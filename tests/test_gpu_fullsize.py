"""GPU parity at the full sizes of the benchmark workloads, in the launch configuration bench.py
times (window 16 x 8, default policy).  The oracle is fast enough to check every output element."""
import numpy as np
import pytest
import torch

import oracle
import paper_2112_02052_amd as tcg
import workloads as W

from gpu_util import TOL_F32, TOL_MFMA, check_sgt, dev, norm_err, upload_csr, upload_x

pytestmark = pytest.mark.gpu


def test_config4_full_size_sgt_spmm_sddmm():
    c = W.make_config(4)
    g, X = c["csr"], c["X"]
    assert (g.n_rows, g.nnz) == (1000000, 19070000)
    rp, ci = upload_csr(g)
    meta = tcg.sgt_build(rp, ci, 16, 8, validate=False)
    check_sgt(meta, g, 16, 8)
    ref = oracle.spmm(g.row_ptr, g.col_idx, X)
    Y = tcg.spmm(meta, upload_x(X, "f32"))
    torch.cuda.synchronize()
    assert norm_err(Y.cpu().numpy(), ref) <= TOL_F32
    del Y
    Xb = W.round_to_bf16(X)
    refb = oracle.spmm(g.row_ptr, g.col_idx, Xb)
    Yb = tcg.spmm(meta, upload_x(Xb, "bf16"))
    torch.cuda.synchronize()
    assert norm_err(Yb.cpu().numpy(), refb) <= TOL_F32      # gather path: exact products, fp32 sums
    del Yb, refb, ref
    e = tcg.sddmm(meta, upload_x(X, "f32"))
    torch.cuda.synchronize()
    assert norm_err(e.cpu().numpy(), oracle.sddmm(g.row_ptr, g.col_idx, X)) <= TOL_F32
    meta.free()


def test_config3_full_size_attention_layer():
    c = W.make_config(3)
    g, X = c["csr"], c["X"]
    rp, ci = upload_csr(g)
    meta = tcg.sgt_build(rp, ci, 16, 16)
    check_sgt(meta, g, 16, 16)
    Xd = upload_x(X, "f32")
    e = tcg.sddmm(meta, Xd)
    p = tcg.row_softmax(meta, e)
    Y = tcg.spmm(meta, Xd, p)
    torch.cuda.synchronize()
    e_ref = oracle.sddmm(g.row_ptr, g.col_idx, X)
    assert norm_err(e.cpu().numpy(), e_ref) <= TOL_F32
    assert norm_err(p.cpu().numpy(), oracle.row_softmax(g.row_ptr, e.cpu().numpy().astype(np.float64))) <= TOL_F32
    p_ref = oracle.row_softmax(g.row_ptr, e_ref)
    Y_ref = oracle.spmm(g.row_ptr, g.col_idx, X, p_ref.astype(np.float32))
    assert norm_err(Y.cpu().numpy(), Y_ref) <= 1e-4
    # rows of the softmax sum to one, so aggregating ones gives ones on non-empty rows
    ones = torch.ones((g.n_rows, 4), device=dev())
    S = tcg.spmm(meta, ones, p).cpu().numpy()
    deg = g.degrees()
    np.testing.assert_allclose(S[deg > 0], 1.0, rtol=1e-5)
    assert np.all(S[deg == 0] == 0)
    meta.free()


@pytest.mark.parametrize("permute", [True, False])
def test_config5_full_size_bf16(permute):
    c = W.make_config(5, permute=permute)
    g, X = c["csr"], c["X"]
    assert g.n_rows == 200000 and X.shape[1] == 256 and c["x_dtype"] == "bf16"
    rp, ci = upload_csr(g)
    meta = tcg.sgt_build(rp, ci, 16, 16)
    check_sgt(meta, g, 16, 16)
    st = tcg.sgt_plan_stats(meta)
    if permute:
        assert st["n_tile_windows"] < 0.01 * meta.n_windows     # no sharing left: gather path
    else:
        assert st["n_tile_windows"] > 0.95 * meta.n_windows     # clustered windows: MFMA path
    Xd = upload_x(X, "bf16")
    e = tcg.sddmm(meta, Xd)
    Y = tcg.spmm(meta, Xd)
    torch.cuda.synchronize()
    assert norm_err(e.cpu().numpy(), oracle.sddmm(g.row_ptr, g.col_idx, X)) <= TOL_F32
    assert norm_err(Y.cpu().numpy(), oracle.spmm(g.row_ptr, g.col_idx, X)) <= TOL_F32   # unit weights are exact in bf16
    w = np.random.default_rng(0).uniform(0.5, 1.5, g.nnz).astype(np.float32)
    Yw = tcg.spmm(meta, Xd, torch.from_numpy(w).to(dev()))
    torch.cuda.synchronize()
    assert norm_err(Yw.cpu().numpy(), oracle.spmm(g.row_ptr, g.col_idx, X, w)) <= (TOL_F32 if permute else TOL_MFMA)
    meta.free()


def test_config5_full_size_fp32_features_on_the_tile_path():
    # The clustered graph in its original order with fp32 features: the default policy sends the windows to the
    # tile kernels, which split fp32 operands into bf16 triples -- fp32 tolerance at full size, with edge values.
    c = W.make_config(5, permute=False)
    g = c["csr"]
    X = W.features_normal(g.n_cols, 256, 9)                      # full fp32 mantissas (the workload's X is bf16-exact)
    rp, ci = upload_csr(g)
    meta = tcg.sgt_build(rp, ci, 16, 8)
    assert tcg.sgt_plan_stats(meta)["n_tile_windows"] > 0.95 * meta.n_windows
    Xd = upload_x(X, "f32")
    w = np.random.default_rng(0).standard_normal(g.nnz).astype(np.float32)
    e = tcg.sddmm(meta, Xd)
    Y = tcg.spmm(meta, Xd, torch.from_numpy(w).to(dev()))
    torch.cuda.synchronize()
    assert norm_err(e.cpu().numpy(), oracle.sddmm(g.row_ptr, g.col_idx, X)) <= TOL_F32
    assert norm_err(Y.cpu().numpy(), oracle.spmm(g.row_ptr, g.col_idx, X, w)) <= TOL_F32
    meta.free()


def test_config5_full_size_with_row_clustering():
    # Workload 5 as given (communities hidden by the random relabelling), clustered and relabelled on the
    # GPU as `bench.py --workload 5 --reorder 2` does: the permutation is bit-exact against the oracle at
    # full size, most windows move to the MFMA tile path, and aggregation / edge scores on the relabelled
    # graph equal the oracle's on the original graph, rows and edges carried through the relabelling.
    import oracle.reorder as R
    c = W.make_config(5)
    g, X = c["csr"], c["X"]
    rp, ci = upload_csr(g)
    perm = tcg.reorder_rows(rp, ci, seed=0, refine=2)
    perm_ref, _, _ = R.reorder_rows(g.row_ptr, g.col_idx, seed=0, refine=2)
    assert np.array_equal(perm.cpu().numpy(), perm_ref)
    rp2, ci2, ep = tcg.csr_permute(rp, ci, perm)
    ref_csr = R.csr_permute(g.row_ptr, g.col_idx, perm_ref)
    assert np.array_equal(rp2.cpu().numpy(), ref_csr[0]) and np.array_equal(ci2.cpu().numpy(), ref_csr[1])
    assert np.array_equal(ep.cpu().numpy(), ref_csr[2])
    meta = tcg.sgt_build(rp2, ci2, 16, 8)
    assert meta.total_unique < 1.1e6                              # 3.8 M before, 0.83 M in the original order
    assert tcg.sgt_plan_stats(meta)["n_tile_windows"] > 0.95 * meta.n_windows
    Xd = upload_x(X, "bf16")[perm.long()].contiguous()
    Y = tcg.spmm(meta, Xd)
    e = tcg.sddmm(meta, Xd)
    torch.cuda.synchronize()
    Y_ref = oracle.spmm(g.row_ptr, g.col_idx, X)
    e_ref = oracle.sddmm(g.row_ptr, g.col_idx, X)
    assert norm_err(Y.cpu().numpy(), Y_ref[perm_ref]) <= TOL_F32          # unit weights are exact in bf16
    assert norm_err(e.cpu().numpy(), e_ref[ref_csr[2]]) <= TOL_F32
    meta.free()
