"""Seeded random sweep over shapes, window sizes, feature widths, types and policies: every drawn case
is checked against the oracle (SGT bit-exact, SpMM / SDDMM within tolerance).  Catches corner cases the
hand-picked parity cases miss (tiny graphs, widths of one 16-byte chunk, ragged last windows, ...)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2112_02052_amd as tcg
import workloads as W

from gpu_util import TOL_F32, TOL_MFMA, check_sgt, dev, norm_err, upload_csr, upload_x
from test_gpu_parity import csr_from_rows

pytestmark = pytest.mark.gpu


def random_case(rng):
    n_rows = int(rng.choice([1, 2, 15, 16, 17, 31, 100, 257, 1000, 3000]))
    n_cols = int(rng.choice([1, 3, 16, 50, 300, 2000, 5000]))
    kind = rng.integers(0, 3)
    rows = []
    for i in range(n_rows):
        if kind == 0:
            k = int(rng.integers(0, min(n_cols, 12) + 1))
        elif kind == 1:
            k = int(min(n_cols, rng.pareto(1.2) * 3))
        else:
            k = int(rng.integers(0, 3)) if rng.random() < 0.8 else int(min(n_cols, rng.integers(100, 900)))
        k = min(k, n_cols)
        cols = rng.choice(n_cols, size=k, replace=False)
        if kind == 2 and k:                                    # windows that share neighbours
            base = (i // 16) * 7 % n_cols
            cols = (base + np.arange(min(k, n_cols))) % n_cols
        rows.append(np.unique(cols) if rng.random() < 0.5 else rng.permutation(np.unique(cols)))
    H = int(rng.choice([16, 16, 16, 1, 5, 32]))
    Wt = int(rng.choice([8, 16, 4, 32]))
    D = int(rng.choice([1, 4, 8, 16, 24, 32, 64, 100, 128, 256, 520]))
    x_dtype = str(rng.choice(["f32", "bf16", "f16"]))
    policy = int(rng.choice([tcg.POLICY_AUTO, tcg.POLICY_GATHER, tcg.POLICY_TILE]))
    if policy == tcg.POLICY_TILE and H not in (16, 32):
        policy = tcg.POLICY_AUTO
    weighted = bool(rng.random() < 0.5)
    return csr_from_rows(rows, n_cols), H, Wt, D, x_dtype, policy, weighted


@pytest.mark.parametrize("seed", range(40))
def test_random_case(seed):
    rng = np.random.default_rng(1000 + seed)
    g, H, Wt, D, x_dtype, policy, weighted = random_case(rng)
    rnd = {"f32": lambda a: a, "bf16": W.round_to_bf16, "f16": lambda a: a.astype(np.float16).astype(np.float32)}[x_dtype]
    n_feat = max(g.n_rows, g.n_cols)
    X = rnd(W.features_normal(n_feat, D, seed))
    w = rng.uniform(0.5, 1.5, g.nnz).astype(np.float32) if weighted else None
    rp, ci = upload_csr(g)
    meta = tcg.sgt_build(rp, ci, H, Wt, n_cols=g.n_cols)
    check_sgt(meta, g, H, Wt)
    tcg.sgt_set_policy(meta, policy)
    Xd = upload_x(X, x_dtype)
    wd = torch.from_numpy(w).to(dev()) if weighted else None
    Y = tcg.spmm(meta, Xd, wd)
    e = tcg.sddmm(meta, Xd)
    torch.cuda.synchronize()
    mfma = x_dtype != "f32" and policy != tcg.POLICY_GATHER and weighted
    assert norm_err(Y.cpu().numpy(), oracle.spmm(g.row_ptr, g.col_idx, X, w)) <= (TOL_MFMA if mfma else TOL_F32)
    assert norm_err(e.cpu().numpy(), oracle.sddmm(g.row_ptr, g.col_idx, X)) <= TOL_F32
    rpt, cit, perm = tcg.csr_transpose(rp, ci, g.n_cols)
    torch.cuda.synchronize()
    ref = oracle.csr_transpose(g.row_ptr, g.col_idx, g.n_cols)
    assert np.array_equal(rpt.cpu().numpy(), ref[0]) and np.array_equal(cit.cpu().numpy(), ref[1])
    assert np.array_equal(perm.cpu().numpy(), ref[2])
    meta.free()
