"""Seeded random differential test: many small cases with random graph structure (mixtures of short rows, shared
neighbourhoods, dense windows, hubs, empty rows), feature width, type, padding, edge values, window height and
policy, each compared with the oracle.  Complements the targeted cases in test_gpu_parity.py: the kernels choose
among a dozen code paths from exactly these parameters."""
import numpy as np
import pytest
import torch

import oracle
import paper_2112_02052_amd as tcg
import workloads as W
from gpu_util import TOL_F32, TOL_MFMA, dev, norm_err, upload_csr, upload_x
from workloads.graphs import CSR

pytestmark = pytest.mark.gpu


def random_graph(rng):
    n_rows = int(rng.integers(1, 700))
    n_cols = int(rng.integers(1, 900))
    kind = rng.integers(0, 4)
    rows = []
    shared = np.sort(rng.choice(n_cols, size=min(n_cols, int(rng.integers(1, 80))), replace=False))
    for i in range(n_rows):
        r = rng.random()
        if r < 0.15:
            k = 0
        elif r < 0.9:
            k = int(rng.integers(1, 40))
        elif r < 0.98:
            k = int(rng.integers(100, 400))
        else:
            k = int(rng.integers(400, 3000))
        k = min(k, n_cols)
        if kind == 1 or (kind == 2 and (i // 16) % 2 == 0):          # rows of a window draw from a shared set
            cols = rng.choice(shared, size=min(k, len(shared)), replace=False)
        elif kind == 3 and (i // 16) % 3 == 0:                        # dense window
            cols = shared
        else:
            cols = rng.choice(n_cols, size=k, replace=False)
        cols = np.asarray(cols, dtype=np.int32)
        if rng.random() < 0.5:
            cols = np.sort(cols)
        rows.append(cols)
    rp = np.zeros(n_rows + 1, dtype=np.int32)
    rp[1:] = np.cumsum([len(r) for r in rows])
    ci = np.concatenate(rows) if rp[-1] else np.zeros(0, np.int32)
    return CSR(n_rows, n_cols, rp, ci.astype(np.int32))


@pytest.mark.parametrize("seed", range(24))
def test_random_shapes_against_the_oracle(seed):
    rng = np.random.default_rng(1000 + seed)
    for case in range(10):
        g = random_graph(rng)
        D = int(rng.choice([1, 2, 4, 8, 12, 16, 20, 32, 40, 64, 68, 72, 96, 128, 136, 200, 256, 264, 300]))
        x_dtype = str(rng.choice(["f32", "bf16", "f16"]))
        H = int(rng.choice([16, 16, 16, 32, 8]))
        policy = [tcg.POLICY_AUTO, tcg.POLICY_GATHER, tcg.POLICY_TILE][int(rng.integers(0, 3))]
        if policy == tcg.POLICY_TILE and H == 8:
            policy = tcg.POLICY_AUTO
        weighted = rng.random() < 0.5
        pad = int(rng.choice([0, 0, 4, 8, 3]))
        X = W.features_normal(max(g.n_rows, g.n_cols), D, seed * 100 + case)
        X = W.round_to_bf16(X) if x_dtype == "bf16" else (X.astype(np.float16).astype(np.float32) if x_dtype == "f16" else X)
        w = rng.standard_normal(g.nnz).astype(np.float32) if weighted else None
        tag = dict(seed=seed, case=case, n_rows=g.n_rows, n_cols=g.n_cols, nnz=g.nnz, D=D, x=x_dtype, H=H, policy=int(policy),
                   weighted=weighted, pad=pad)
        print(tag, flush=True)
        rp, ci = upload_csr(g)
        meta = tcg.sgt_build(rp, ci, H, 8, n_cols=g.n_cols)
        tcg.sgt_set_policy(meta, policy)
        Xd = upload_x(X, x_dtype)
        if pad:
            big = torch.zeros((Xd.shape[0], D + pad), dtype=Xd.dtype, device=dev())
            big[:, :D] = Xd
            Xd = big[:, :D]
        tile_possible = policy != tcg.POLICY_GATHER and x_dtype != "f32"
        tol_w = TOL_MFMA if (weighted and tile_possible) else TOL_F32   # rounded edge values only on the 16-bit MFMA path
        Y = torch.full((g.n_rows, D), float("nan"), device=dev())
        tcg.spmm(meta, Xd, None if w is None else torch.from_numpy(w).to(dev()), Y=Y)
        torch.cuda.synchronize()
        assert norm_err(Y.cpu().numpy(), oracle.spmm(g.row_ptr, g.col_idx, X[:g.n_cols], w)) <= tol_w, tag
        e = torch.full((g.nnz,), float("nan"), device=dev())
        tcg.sddmm(meta, Xd, out=e)
        torch.cuda.synchronize()
        assert norm_err(e.cpu().numpy(), oracle.sddmm(g.row_ptr, g.col_idx, X)) <= TOL_F32, tag
        meta.free()
