"""tcg_spmm_noalloc (the entry point for callers that cannot allocate device memory) against tcg_spmm:
same kernels, the split rows' partial sums in the library's static device array instead of the plan's
buffer.  Two calls in a row share that array, the second on a smaller input; results must be bit-identical
to tcg_spmm's (which the parity tests hold to the oracle) and are checked against the oracle as well."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2112_02052_amd as tcg
import workloads as W

from gpu_util import TOL_F32, dev, norm_err, upload_csr, upload_x

pytestmark = pytest.mark.gpu


def test_spmm_noalloc_matches_spmm_on_two_calls_in_a_row():
    # R-MAT graphs have hub rows, i.e. split rows whose partial sums go through the scratch.
    cases = [(4, 60000, 128, "f32", True), (4, 9000, 64, "bf16", False)]     # the second one is smaller
    prepared = []
    for cfg, n, D, x_dtype, weighted in cases:
        c = W.make_config(cfg, n=n, d=D)
        g = c["csr"]
        X = W.round_to_bf16(c["X"]) if x_dtype == "bf16" else c["X"]
        w = (W.features_uniform(g.nnz, 1, 9)[:, 0].copy() if weighted else None)
        rp, ci = upload_csr(g)
        meta = tcg.sgt_build(rp, ci, 16, 8)
        assert tcg.sgt_plan_stats(meta)["n_long_rows"] > 0
        Xd = upload_x(X, x_dtype)
        wd = torch.from_numpy(w).to(dev()) if weighted else None
        Y_ref = tcg.spmm(meta, Xd, wd)
        Y = torch.full((g.n_rows, D), float("nan"), device=dev())
        prepared.append((g, X, w, meta, Xd, wd, Y_ref, Y))
    torch.cuda.synchronize()
    for g, X, w, meta, Xd, wd, Y_ref, Y in prepared:                         # back to back, nothing in between
        tcg.spmm_noalloc(meta, Xd, wd, Y)
    torch.cuda.synchronize()
    for g, X, w, meta, Xd, wd, Y_ref, Y in prepared:
        assert torch.equal(Y, Y_ref)
        assert norm_err(Y.cpu().numpy(), oracle.spmm(g.row_ptr, g.col_idx, X, w)) <= TOL_F32
        meta.free()


def test_spmm_noalloc_rejects_a_plan_beyond_the_static_buffer():
    # 64 MiB / 4 bytes / D = 4096 leaves room for 4096 split-row segments; this graph has more.
    c = W.make_config(4, n=200000, d=4)
    g = c["csr"]
    rp, ci = upload_csr(g)
    meta = tcg.sgt_build(rp, ci, 16, 8)
    D = 4096
    X = torch.zeros((g.n_cols, D), device=dev())
    Y = torch.full((g.n_rows, D), 7.0, device=dev())
    lib = tcg.load_library()
    st = lib.tcg_spmm_noalloc(meta._h, ctypes.c_void_p(X.data_ptr()), 0, D, D, None, ctypes.c_void_p(Y.data_ptr()),
                              0, D, None)
    torch.cuda.synchronize()
    assert st == -6 and b"static buffer" in lib.tcg_strerror(st)
    assert bool((Y == 7.0).all())                                            # nothing was written
    with pytest.raises(tcg.TcgError):
        tcg.spmm_noalloc(meta, X, None, Y)
    meta.free()
