"""Pins for the row-clustering oracle (oracle/reorder.py): the hash against the published splitmix64
sequence, the vectorised form against explicit loops, the invariants each step must satisfy, the
symmetric CSR permutation against dense algebra, and the effect the pass exists for (fewer distinct
columns per window on a graph with planted communities)."""
from collections import Counter

import numpy as np
import pytest

import oracle
import oracle.reorder as R
import workloads as W


def random_square(n, p, seed, dup=False, long_row=False):
    rng = np.random.default_rng(seed)
    A = rng.random((n, n)) < p
    rows = [rng.permutation(np.nonzero(r)[0]) for r in A]
    if dup and len(rows[0]):
        rows[0] = np.concatenate([rows[0], rows[0][:2]])
    if long_row:
        rows[n // 2] = rng.integers(0, n, size=300)              # more than 128 entries, with repeats
    rp = np.concatenate([[0], np.cumsum([len(r) for r in rows])]).astype(np.int32)
    ci = (np.concatenate(rows) if rp[-1] else np.zeros(0)).astype(np.int32)
    return rp, ci


def test_hash_is_splitmix64():
    # First outputs of splitmix64 from state 0 (the reference implementation's well-known sequence):
    # the state advances by the golden-ratio increment, so node id k with seed 0 is output k.
    got = R.node_hash(0, np.arange(3))
    assert [int(x) for x in got] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    assert int(R.node_hash(5, np.array([0]))[0]) != int(got[0])


@pytest.mark.parametrize("n,p,seed,refine", [(1, 0.0, 0, 0), (7, 0.4, 1, 0), (40, 0.1, 2, 1), (90, 0.05, 3, 2),
                                             (160, 0.02, 4, 3), (64, 0.3, 5, 2)])
def test_vectorised_form_equals_loops(n, p, seed, refine):
    rp, ci = random_square(n, p, seed, dup=True, long_row=n >= 90)
    a = R.reorder_rows(rp, ci, seed=seed, refine=refine)
    b = R.reorder_rows_loops(rp, ci, seed=seed, refine=refine)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


def test_step_invariants():
    rp, ci = random_square(200, 0.03, 7)
    seed = 11
    perm, label, parent = R.reorder_rows(rp, ci, seed=seed, refine=0)
    n = 200
    h = [int(x) for x in R.node_hash(seed, np.arange(n))]
    for v in range(n):
        nb = set(ci[rp[v]:rp[v + 1]].tolist()) | {v}
        assert parent[v] in nb
        assert (h[parent[v]], parent[v]) == min((h[u], u) for u in nb)
        assert parent[label[v]] == label[v]                       # a root is its own parent
    # following parents from v ends in label[v]
    for v in range(n):
        p = v
        while parent[p] != p:
            assert h[parent[p]] < h[p]
            p = parent[p]
        assert p == label[v]
    assert sorted(perm.tolist()) == list(range(n))
    keys = [(label[v], parent[v], v) for v in perm]
    assert keys == sorted(keys)
    # one refinement round: majority label of the neighbours, ties to the smallest id
    _, label1, _ = R.reorder_rows(rp, ci, seed=seed, refine=1)
    for v in range(n):
        cnt = Counter(label[ci[rp[v]:rp[v + 1]]].tolist())
        if cnt:
            top = max(cnt.values())
            assert label1[v] == min(k for k, c in cnt.items() if c == top)
        else:
            assert label1[v] == label[v]


def test_isolated_nodes_and_empty_graph():
    rp = np.zeros(6, np.int32)
    ci = np.zeros(0, np.int32)
    perm, label, parent = R.reorder_rows(rp, ci, seed=3, refine=2)
    assert np.array_equal(parent, np.arange(5)) and np.array_equal(label, np.arange(5))
    assert np.array_equal(perm, np.arange(5))
    with pytest.raises(ValueError):
        R.reorder_rows(np.array([0, 1], np.int32), np.array([4], np.int32))


def test_csr_permute_against_dense():
    n = 30
    rp, ci = random_square(n, 0.2, 9)
    rng = np.random.default_rng(9)
    vals = rng.standard_normal(len(ci))
    perm = rng.permutation(n).astype(np.int32)
    A = np.zeros((n, n))
    rows = np.repeat(np.arange(n), np.diff(rp))
    A[rows, ci] = vals
    nrp, nci, eperm = R.csr_permute(rp, ci, perm)
    B = np.zeros((n, n))
    B[np.repeat(np.arange(n), np.diff(nrp)), nci] = vals[eperm]
    np.testing.assert_array_equal(B, A[np.ix_(perm, perm)])
    # entries keep their order inside a row
    for i in range(n):
        assert np.array_equal(eperm[nrp[i]:nrp[i + 1]], np.arange(rp[perm[i]], rp[perm[i] + 1]))
    # aggregation commutes with the relabelling: Y'[i] = Y[perm[i]] when X' = X[perm]
    X = rng.standard_normal((n, 3)).astype(np.float32)
    w = vals.astype(np.float32)
    Y = oracle.spmm(rp, ci, X, w)
    Yp = oracle.spmm(nrp, nci, X[perm], w[eperm])
    np.testing.assert_allclose(Yp, Y[perm], rtol=1e-12, atol=1e-12)
    with pytest.raises(ValueError):
        R.csr_permute(rp, ci, np.zeros(n, np.int32))


def test_recovers_planted_communities():
    # 64-node communities hidden by a random relabelling (workload 5): after the pass the windows see
    # far fewer distinct columns, and refinement rounds improve on the plain trees.
    c = W.make_config(5, n=64 * 150, d=2)
    g = c["csr"]
    u_before = oracle.sgt(g.row_ptr, g.col_idx, 16, 8)["col_to_row"].size
    u_after = []
    for refine in (0, 2):
        perm, _, _ = R.reorder_rows(g.row_ptr, g.col_idx, seed=0, refine=refine)
        nrp, nci, _ = R.csr_permute(g.row_ptr, g.col_idx, perm)
        u_after.append(oracle.sgt(nrp, nci, 16, 8)["col_to_row"].size)
    assert u_after[0] < 0.4 * u_before
    assert u_after[1] < 0.9 * u_after[0]
