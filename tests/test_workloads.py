"""The seeded input generators: structure, sizes and determinism."""
import numpy as np
import pytest
import torch

import workloads as W
from workloads import rng as wrng


def check_csr(g, symmetric=True):
    rp = g.row_ptr.astype(np.int64)
    assert g.row_ptr.dtype == np.int32 and g.col_idx.dtype == np.int32
    assert rp[0] == 0 and rp[-1] == g.nnz and np.all(np.diff(rp) >= 0)
    assert g.col_idx.min() >= 0 and g.col_idx.max() < g.n_cols
    rows = g.row_of_edge().astype(np.int64)
    key = rows * g.n_cols + g.col_idx
    assert np.all(np.diff(key) > 0)                      # ascending unique columns per row
    if symmetric:
        assert np.array_equal(np.sort(g.col_idx.astype(np.int64) * g.n_cols + rows), key)


def test_splitmix_known_answer_and_counter_property():
    # First output of the published splitmix64 generator started from state 0.
    with np.errstate(over="ignore"):
        assert int(wrng._mix(np.uint64(0x9E3779B97F4A7C15))) == 0xE220A8397B1DCDAF
    a = W.splitmix64(3, 5, 0, 1000)
    b = np.concatenate([W.splitmix64(3, 5, 0, 123), W.splitmix64(3, 5, 123, 877)])
    assert np.array_equal(a, b)                          # value k depends only on k
    assert not np.array_equal(a, W.splitmix64(4, 5, 0, 1000))
    assert not np.array_equal(a, W.splitmix64(3, 6, 0, 1000))
    u = W.uniform01(0, 1, 0, 200000)
    assert 0 <= u.min() and u.max() < 1 and abs(u.mean() - 0.5) < 5e-3
    z = W.normal01(0, 2, 0, 200000)
    assert abs(z.mean()) < 1e-2 and abs(z.std() - 1) < 1e-2


def test_config1_exact_sizes():
    c = W.make_config(1)
    g = c["csr"]
    assert (g.n_rows, g.nnz) == (2048, 2 * 4096 + 2048)
    assert c["X"].shape == (2048, 16) and c["X"].dtype == np.float32
    assert np.abs(c["X"]).max() <= 1
    check_csr(g)
    assert np.all(g.col_idx[g.row_ptr[:-1]] <= np.arange(2048))   # self-loop present => first col <= i
    deg = g.degrees()
    rows = g.row_of_edge()
    np.testing.assert_allclose(c["w"], 1 / np.sqrt(deg[rows] * deg[g.col_idx]), rtol=1e-6)
    c2 = W.make_config(1)
    assert np.array_equal(c2["csr"].col_idx, g.col_idx) and np.array_equal(c2["X"], c["X"])


def test_config2_power_law():
    g = W.make_config(2, d=2)["csr"]
    check_csr(g)
    deg = g.degrees()
    assert g.n_rows == 20000 and deg.min() >= 1 and 300 < deg.max() <= 520
    assert 4.0 < deg.mean() < 7.0


@pytest.mark.parametrize("cfg,n", [(3, 4000), (4, 6000)])
def test_rmat_small(cfg, n):
    c = W.make_config(cfg, n=n, d=2)
    g = c["csr"]
    check_csr(g)
    assert not np.any(g.row_of_edge() == g.col_idx)     # self pairs dropped
    deg = g.degrees()
    assert deg.max() > 20 * max(1.0, deg.mean()) / 4    # skewed
    assert (deg == 0).any()


def test_config5_clusters():
    g = W.make_config(5, n=64 * 50, d=2, permute=False)["csr"]
    check_csr(g)
    rows = g.row_of_edge()
    intra = (rows // 64) == (g.col_idx // 64)
    assert 0.98 < intra.mean() < 0.995                  # about 1 % of the pairs join communities
    assert abs(intra.sum() / (50 * 64 * 63) - 0.3) < 0.02
    gp = W.make_config(5, n=64 * 50, d=2, permute=True)["csr"]
    check_csr(gp)
    assert gp.nnz == g.nnz
    rows = gp.row_of_edge()
    assert ((rows // 64) == (gp.col_idx // 64)).mean() < 0.1


def test_bf16_rounding_matches_torch():
    x = W.features_normal(1000, 8, 0)
    x[0, :4] = [1.00390625, 1.01171875, -1.00390625, 3.0e-39]   # ties (to even) and a denormal
    r = W.round_to_bf16(x)
    t = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(r, t)
    bits = W.bf16_bits(x)
    assert np.array_equal(bits.view(np.int16), torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy())
    c = W.make_config(5, n=640)
    assert c["x_dtype"] == "bf16" and np.array_equal(W.round_to_bf16(c["X"]), c["X"])


def test_window_fill_controls_the_sharing():
    g = W.window_fill(2048, 48, 0.5, seed=3)
    assert g.n_rows == 2048 and g.col_idx.max() < 2048
    for w in (0, 17, 127):
        cols = np.unique(g.col_idx[g.row_ptr[16 * w]:g.row_ptr[16 * w + 16]])
        assert cols.size <= 48
    reuse = g.nnz / sum(np.unique(g.col_idx[g.row_ptr[16 * w]:g.row_ptr[16 * w + 16]]).size for w in range(128))
    assert 7.0 < reuse < 9.0                                    # about 16 * fill entries per distinct column
    g2 = W.window_fill(2048, 48, 0.5, seed=3)
    assert np.array_equal(g.col_idx, g2.col_idx)
