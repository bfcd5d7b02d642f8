"""Helpers shared by the GPU parity tests: upload inputs, run the library through its binding,
compare with the oracle.  Nothing here computes a reference value by itself."""
import numpy as np
import torch

import oracle
import paper_2112_02052_amd as tcg

TORCH_DT = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}
# Tolerances, normalised by the largest magnitude of the oracle's result:
#   fp32 path (fp32 features, or bf16/f16 features on the gather path: exact products, fp32 sums) 1e-5
#   bf16 / f16 MFMA path (edge values rounded to the feature type)                               1e-2
TOL_F32 = 1e-5
TOL_MFMA = 1e-2


def dev():
    return torch.device("cuda:0")


def upload_csr(g):
    return torch.from_numpy(g.row_ptr).to(dev()), torch.from_numpy(g.col_idx).to(dev())


def upload_x(X, x_dtype):
    """X: float32 numpy holding values exactly representable in x_dtype."""
    t = torch.from_numpy(np.ascontiguousarray(X)).to(dev()).to(TORCH_DT[x_dtype])
    assert torch.equal(t.to(torch.float32).cpu(), torch.from_numpy(np.ascontiguousarray(X)))
    return t


def norm_err(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    assert got.shape == ref.shape
    scale = np.abs(ref).max() if ref.size else 1.0
    if ref.size == 0:
        return 0.0
    return float(np.abs(got - ref).max() / max(scale, 1e-300))


def check_sgt(meta, g, H, W_):
    ref = oracle.sgt(g.row_ptr, g.col_idx, H, W_)
    got = {k: v.cpu().numpy() for k, v in tcg.sgt_export(meta).items()}
    assert meta.total_unique == ref["col_to_row"].size
    assert meta.total_tiles == int(ref["win_partition"].astype(np.int64).sum())
    assert meta.n_windows == ref["win_partition"].size
    assert np.array_equal(got["win_partition"], ref["win_partition"])
    assert np.array_equal(got["win_unique_ptr"].astype(np.int64), ref["win_unique_ptr"])
    assert np.array_equal(got["col_to_row"], ref["col_to_row"])
    assert np.array_equal(got["edge_to_col"], ref["edge_to_col"])
    return ref
