"""GPU parity of the row-clustering pass and the symmetric CSR permutation against the oracle: the
permutation and the relabelled pattern are integer results and must match bit for bit; aggregation on
the relabelled graph must commute with the relabelling."""
import numpy as np
import pytest
import torch

import oracle
import oracle.reorder as R
import paper_2112_02052_amd as tcg
import workloads as W

from gpu_util import TOL_F32, TOL_MFMA, check_sgt, dev, norm_err, upload_csr, upload_x
from workloads.graphs import CSR
from test_gpu_parity import csr_from_rows, hub_graph

pytestmark = pytest.mark.gpu


def square_random(n, max_deg, seed, dup=True):
    rng = np.random.default_rng(seed)
    rows = [rng.integers(0, n, size=int(rng.integers(0, max_deg))) if dup
            else rng.choice(n, size=int(rng.integers(0, min(max_deg, n))), replace=False) for _ in range(n)]
    return csr_from_rows(rows, n)


CASES = [
    lambda: W.make_config(5, n=64 * 120, d=2)["csr"],            # planted communities, relabelled
    lambda: W.make_config(5, n=64 * 40, d=2, permute=False)["csr"],
    lambda: W.make_config(4, n=60000, d=2)["csr"],               # R-MAT: hub rows above 4096 entries, empty rows
    lambda: W.make_config(2, n=5000, d=2)["csr"],
    lambda: hub_graph(6000),
    lambda: square_random(700, 300, 3),                          # repeated entries, rows above 128 entries
    lambda: square_random(17, 5, 4),
    lambda: csr_from_rows([[]], 1),
    lambda: csr_from_rows([[], [], []], 3),
]


@pytest.mark.parametrize("case", range(len(CASES)))
@pytest.mark.parametrize("refine", [0, 2])
def test_reorder_rows_bit_exact(case, refine):
    g = CASES[case]()
    rp, ci = upload_csr(g)
    seed = 1234 + case
    perm = tcg.reorder_rows(rp, ci, seed=seed, refine=refine)
    torch.cuda.synchronize()
    ref, _, _ = R.reorder_rows(g.row_ptr, g.col_idx, seed=seed, refine=refine)
    assert np.array_equal(perm.cpu().numpy(), ref)


def test_reorder_is_deterministic_and_seeded():
    g = W.make_config(5, n=64 * 60, d=2)["csr"]
    rp, ci = upload_csr(g)
    a = tcg.reorder_rows(rp, ci, seed=7)
    b = tcg.reorder_rows(rp, ci, seed=7)
    c = tcg.reorder_rows(rp, ci, seed=8)
    assert torch.equal(a, b) and not torch.equal(a, c)


@pytest.mark.parametrize("case", [0, 2, 4, 5, 7, 8])
def test_csr_permute_bit_exact(case):
    g = CASES[case]()
    rp, ci = upload_csr(g)
    perm_np = np.random.default_rng(case).permutation(g.n_rows).astype(np.int32)
    perm = torch.from_numpy(perm_np).to(dev())
    rp2, ci2, ep = tcg.csr_permute(rp, ci, perm)
    torch.cuda.synchronize()
    ref = R.csr_permute(g.row_ptr, g.col_idx, perm_np)
    assert np.array_equal(rp2.cpu().numpy(), ref[0])
    assert np.array_equal(ci2.cpu().numpy(), ref[1])
    assert np.array_equal(ep.cpu().numpy(), ref[2])
    rp3, ci3, none = tcg.csr_permute(rp, ci, perm, want_edge_perm=False)
    assert none is None and torch.equal(ci3, ci2) and torch.equal(rp3, rp2)


def test_errors():
    g = W.make_config(1, n=300, d=2)["csr"]
    rp, ci = upload_csr(g)
    bad = torch.zeros(g.n_rows, dtype=torch.int32, device=dev())            # not a permutation
    with pytest.raises(tcg.TcgError):
        tcg.csr_permute(rp, ci, bad)
    out_of_range = torch.arange(g.n_rows, dtype=torch.int32, device=dev())
    out_of_range[5] = g.n_rows + 3
    with pytest.raises(tcg.TcgError):
        tcg.csr_permute(rp, ci, out_of_range)
    wide = csr_from_rows([[0, 5], [1]], 6)                                  # columns beyond the row count
    rpw, ciw = upload_csr(wide)
    with pytest.raises(tcg.TcgError):
        tcg.reorder_rows(rpw, ciw)
    with pytest.raises(tcg.TcgError):
        tcg.csr_permute(rpw, ciw, torch.arange(2, dtype=torch.int32, device=dev()))


def test_aggregation_commutes_with_the_relabelling_and_windows_condense():
    # Workload 5 (communities hidden by a random relabelling): cluster, relabel, translate; the
    # relabelled graph gives the same aggregation (rows in the new order), with far fewer distinct
    # columns per window, and the default policy now picks the MFMA tile path.
    c = W.make_config(5, n=64 * 300)
    g, X = c["csr"], c["X"]
    rp, ci = upload_csr(g)
    perm = tcg.reorder_rows(rp, ci, seed=0, refine=2)
    rp2, ci2, ep = tcg.csr_permute(rp, ci, perm)
    meta0 = tcg.sgt_build(rp, ci, 16, 8)
    meta1 = tcg.sgt_build(rp2, ci2, 16, 8)
    assert meta1.total_unique < 0.4 * meta0.total_unique
    assert tcg.sgt_plan_stats(meta1)["n_tile_windows"] > 0.5 * meta1.n_windows
    ref = oracle.spmm(g.row_ptr, g.col_idx, X, None)
    Xd = upload_x(X, "bf16")
    Xp = Xd[perm.long()].contiguous()
    for policy, tol in ((tcg.POLICY_GATHER, TOL_F32), (tcg.POLICY_AUTO, TOL_F32)):   # unit edge values: exact in bf16
        tcg.sgt_set_policy(meta1, policy)
        Y1 = tcg.spmm(meta1, Xp)
        torch.cuda.synchronize()
        assert norm_err(Y1.cpu().numpy(), ref[perm.cpu().numpy()]) <= tol
    # edge values follow through edge_perm
    w = np.random.default_rng(0).standard_normal(g.nnz).astype(np.float32)
    wd = torch.from_numpy(w).to(dev())
    tcg.sgt_set_policy(meta1, tcg.POLICY_GATHER)
    Yw = tcg.spmm(meta1, Xp, tcg.edge_gather(ep, wd))
    torch.cuda.synchronize()
    assert norm_err(Yw.cpu().numpy(), oracle.spmm(g.row_ptr, g.col_idx, X, w)[perm.cpu().numpy()]) <= TOL_F32
    meta0.free()
    meta1.free()


def test_clustered_build_gives_the_oracle_results_on_the_original_labelling():
    # tcg_sgt_build_clustered = reorder + permute + translate.  Its permutation and relabelled pattern are the
    # oracle's bit for bit; SpMM / SDDMM run on the relabelled graph and, taken back to the original labelling,
    # equal the oracle's results on the original graph; and the windows condense (the point of the exercise).
    c = W.make_config(5, n=64 * 150, d=64)
    g = c["csr"]
    X = W.round_to_bf16(c["X"])
    rp, ci = upload_csr(g)
    meta, perm, ep = tcg.sgt_build_clustered(rp, ci, 16, 8, seed=0, refine=2)
    perm_ref = R.reorder_rows(g.row_ptr, g.col_idx, seed=0, refine=2)[0]
    assert np.array_equal(perm.cpu().numpy(), perm_ref)
    rp2_ref, ci2_ref, ep_ref = R.csr_permute(g.row_ptr, g.col_idx, perm_ref)
    assert np.array_equal(meta.row_ptr.cpu().numpy(), rp2_ref) and np.array_equal(meta.col_idx.cpu().numpy(), ci2_ref)
    assert np.array_equal(ep.cpu().numpy(), ep_ref)
    check_sgt(meta, CSR(g.n_rows, g.n_cols, rp2_ref, ci2_ref), 16, 8)
    plain = tcg.sgt_build(rp, ci, 16, 8)
    assert meta.total_unique < 0.5 * plain.total_unique
    assert tcg.sgt_plan_stats(meta)["n_tile_windows"] > 0.9 * meta.n_windows
    plain.free()
    pl = perm.long()
    Xd = upload_x(X, "bf16")
    Yp = tcg.spmm(meta, Xd[pl].contiguous())
    Ep = tcg.sddmm(meta, Xd[pl].contiguous())
    torch.cuda.synchronize()
    Y = torch.empty_like(Yp)
    Y[pl] = Yp
    E = torch.empty_like(Ep)
    E[ep.long()] = Ep
    assert norm_err(Y.cpu().numpy(), oracle.spmm(g.row_ptr, g.col_idx, X, None)) <= TOL_MFMA
    assert norm_err(E.cpu().numpy(), oracle.sddmm(g.row_ptr, g.col_idx, X)) <= TOL_MFMA
    meta.free()
