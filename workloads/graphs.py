"""Seeded synthetic graph generators.  Every generator returns a CSR structure with int32
row pointers / column indices and ascending, duplicate-free columns inside each row.

The shapes follow the paper's evaluation graphs (Table 4 of the paper: small citation-like
graphs, power-law graphs, batched dense-cluster graphs, large irregular graphs) without
reproducing any dataset: all structure is drawn from the counter-based generator in
`workloads.rng`.
"""
from dataclasses import dataclass

import numpy as np

from .rng import splitmix64, uniform01


@dataclass
class CSR:
    n_rows: int
    n_cols: int
    row_ptr: np.ndarray  # int32 [n_rows + 1]
    col_idx: np.ndarray  # int32 [nnz]

    @property
    def nnz(self):
        return int(self.col_idx.shape[0])

    def degrees(self):
        return np.diff(self.row_ptr.astype(np.int64))

    def row_of_edge(self):
        """int32 [nnz]: the row each stored entry belongs to."""
        return np.repeat(np.arange(self.n_rows, dtype=np.int32), self.degrees())


def _csr_from_keys(keys, n_rows, n_cols):
    """keys = row * n_cols + col (int64, any order, may repeat) -> CSR (sorted, unique)."""
    keys = np.unique(keys)
    if keys.size >= 2**31:
        raise ValueError("nnz does not fit int32")
    rows = keys // n_cols
    cols = (keys - rows * n_cols).astype(np.int32)
    counts = np.bincount(rows, minlength=n_rows)
    row_ptr = np.zeros(n_rows + 1, dtype=np.int64)
    np.cumsum(counts, out=row_ptr[1:])
    return CSR(n_rows, n_cols, row_ptr.astype(np.int32), cols)


def csr_from_directed_pairs(src, dst, n, self_loops=False):
    src = np.asarray(src, dtype=np.int64)
    dst = np.asarray(dst, dtype=np.int64)
    keys = src * n + dst
    if self_loops:
        d = np.arange(n, dtype=np.int64)
        keys = np.concatenate([keys, d * n + d])
    return _csr_from_keys(keys, n, n)


def csr_from_undirected_pairs(u, v, n, self_loops=False):
    """Symmetrise: both (u,v) and (v,u) are stored; duplicates collapse."""
    u = np.asarray(u, dtype=np.int64)
    v = np.asarray(v, dtype=np.int64)
    return csr_from_directed_pairs(np.concatenate([u, v]), np.concatenate([v, u]), n, self_loops)


def _first_distinct_pairs(u, v, n, want):
    """Drop u==v, canonicalise (min,max), keep first occurrences in draw order, take `want`."""
    keep = u != v
    u, v = u[keep], v[keep]
    lo = np.minimum(u, v).astype(np.int64)
    hi = np.maximum(u, v).astype(np.int64)
    key = lo * n + hi
    _, first = np.unique(key, return_index=True)
    first.sort()
    first = first[:want]
    return lo[first], hi[first]


def erdos_renyi_gnm(n, m, seed, self_loops=True):
    """G(n, m): exactly m distinct undirected pairs (i != j), uniform; symmetrised."""
    got_u = np.zeros(0, dtype=np.int64)
    got_v = np.zeros(0, dtype=np.int64)
    start = 0
    while True:
        cnt = 2 * m + 64
        r = splitmix64(seed, 11, start, 2 * cnt)
        start += 2 * cnt
        u = np.concatenate([got_u, (r[0::2] % np.uint64(n)).astype(np.int64)])
        v = np.concatenate([got_v, (r[1::2] % np.uint64(n)).astype(np.int64)])
        got_u, got_v = _first_distinct_pairs(u, v, n, m)
        if got_u.size == m:
            break
    return csr_from_undirected_pairs(got_u, got_v, n, self_loops)


def chung_lu_powerlaw(n, seed, exponent=2.1, mean_degree=5.0, max_degree=500.0, self_loops=True):
    """Chung-Lu style graph: expected degree of node i proportional to (i+1)^(-1/(exponent-1)),
    scaled to `mean_degree` and capped at `max_degree`; n*mean_degree/2 endpoint pairs are
    drawn with probability proportional to the expected degrees; self pairs and repeats dropped."""
    alpha = 1.0 / (exponent - 1.0)
    theta = (np.arange(n, dtype=np.float64) + 1.0) ** (-alpha)
    for _ in range(32):
        theta *= mean_degree * n / theta.sum()
        np.minimum(theta, max_degree, out=theta)
    cdf = np.cumsum(theta)
    cdf /= cdf[-1]
    m = int(round(n * mean_degree / 2.0))
    r = uniform01(seed, 21, 0, 2 * m)
    u = np.minimum(np.searchsorted(cdf, r[0::2], side="right"), n - 1)
    v = np.minimum(np.searchsorted(cdf, r[1::2], side="right"), n - 1)
    keep = u != v
    return csr_from_undirected_pairs(u[keep], v[keep], n, self_loops)


def rmat(n, scale, n_samples, seed, a=0.57, b=0.19, c=0.19, d=0.05, self_loops=False,
         batch=1 << 21):
    """R-MAT (Chakrabarti, Zhan, Faloutsos 2004) on a 2^scale grid, no noise.  Candidate pairs
    with an id >= n are rejected and the next candidates take their place, until `n_samples`
    pairs are accepted.  Self pairs are then dropped, the rest deduplicated and symmetrised."""
    assert n <= (1 << scale)
    assert abs(a + b + c + d - 1.0) < 1e-12
    src_parts, dst_parts = [], []
    accepted = 0
    cand = 0
    while accepted < n_samples:
        r = uniform01(seed, 31, cand * scale, batch * scale).reshape(batch, scale)
        cand += batch
        row_bit = r >= (a + b)                       # quadrants c, d -> lower half
        col_bit = ((r >= a) & (r < a + b)) | (r >= a + b + c)   # quadrants b, d -> right half
        weights = (np.int64(1) << np.arange(scale - 1, -1, -1, dtype=np.int64))
        src = row_bit.astype(np.int64) @ weights
        dst = col_bit.astype(np.int64) @ weights
        ok = (src < n) & (dst < n)
        src, dst = src[ok], dst[ok]
        take = min(src.size, n_samples - accepted)
        src_parts.append(src[:take])
        dst_parts.append(dst[:take])
        accepted += take
    src = np.concatenate(src_parts)
    dst = np.concatenate(dst_parts)
    keep = src != dst
    return csr_from_undirected_pairs(src[keep], dst[keep], n, self_loops)


def clustered_communities(n_comm, comm_size, p_intra, inter_frac, seed, permute=True,
                          self_loops=False):
    """`n_comm` communities of `comm_size` nodes; each intra-community pair kept with
    probability `p_intra`; plus round(inter_frac * #intra pairs) uniform pairs joining different
    communities.  With `permute`, node labels are shuffled by a seeded uniform permutation
    (applied to rows and columns alike)."""
    n = n_comm * comm_size
    ia, ib = np.triu_indices(comm_size, k=1)
    per = ia.size
    u_parts, v_parts = [], []
    chunk = max(1, (1 << 22) // per)
    for c0 in range(0, n_comm, chunk):
        c1 = min(n_comm, c0 + chunk)
        r = uniform01(seed, 41, c0 * per, (c1 - c0) * per).reshape(c1 - c0, per)
        cc, pp = np.nonzero(r < p_intra)
        base = (cc.astype(np.int64) + c0) * comm_size
        u_parts.append(base + ia[pp])
        v_parts.append(base + ib[pp])
    u = np.concatenate(u_parts)
    v = np.concatenate(v_parts)
    n_inter = int(round(inter_frac * u.size))
    iu = np.zeros(0, dtype=np.int64)
    iv = np.zeros(0, dtype=np.int64)
    start = 0
    while iu.size < n_inter:
        cnt = 2 * (n_inter - iu.size) + 64
        r = splitmix64(seed, 42, start, 2 * cnt)
        start += 2 * cnt
        x = (r[0::2] % np.uint64(n)).astype(np.int64)
        y = (r[1::2] % np.uint64(n)).astype(np.int64)
        ok = (x // comm_size) != (y // comm_size)
        iu = np.concatenate([iu, x[ok]])[:n_inter]
        iv = np.concatenate([iv, y[ok]])[:n_inter]
    u = np.concatenate([u, iu])
    v = np.concatenate([v, iv])
    if permute:
        keys = splitmix64(seed, 43, 0, n)
        perm = np.argsort(keys, kind="stable").astype(np.int64)
        u, v = perm[u], perm[v]
    return csr_from_undirected_pairs(u, v, n, self_loops)


def dense_block_windows(n, blocks_per_window, seed, block=16):
    """The paper's sparsity-sweep matrix (Table 6 and the text under it): an n x n adjacency
    in which every `block`-row window holds `blocks_per_window` fully dense block x block
    tiles at distinct, randomly chosen block columns."""
    assert n % block == 0
    nb = n // block
    assert blocks_per_window <= nb
    src_parts, dst_parts = [], []
    rr, cc = np.meshgrid(np.arange(block), np.arange(block), indexing="ij")
    for w in range(nb):
        keys = splitmix64(seed, 51, w * nb, nb)
        cols = np.argsort(keys, kind="stable")[:blocks_per_window]
        for bc in cols:
            src_parts.append((w * block + rr).ravel())
            dst_parts.append((int(bc) * block + cc).ravel())
    return csr_from_directed_pairs(np.concatenate(src_parts), np.concatenate(dst_parts), n)


def window_fill(n, unique_per_window, fill, seed, block=16):
    """Windows with a chosen amount of neighbour sharing: every `block`-row window draws
    `unique_per_window` distinct columns and every (row, column) pair of that window x column set is
    stored with probability `fill`, so a window's entries per distinct column -- the reuse that decides
    between the gather and the tile path -- is about block * fill."""
    assert n % block == 0 and unique_per_window <= n
    nb = n // block
    src_parts, dst_parts = [], []
    for w in range(nb):
        draws = (splitmix64(seed, 61, w * 4 * unique_per_window, 4 * unique_per_window) % np.uint64(n)).astype(np.int64)
        _, first = np.unique(draws, return_index=True)
        cols = draws[np.sort(first)][:unique_per_window]           # distinct, in drawing order
        assert cols.size == unique_per_window, "column space too small for this many distinct columns"
        r = uniform01(seed, 62, w * block * unique_per_window, block * unique_per_window)
        rr, cc = np.nonzero(r.reshape(block, unique_per_window) < fill)
        src_parts.append(w * block + rr)
        dst_parts.append(cols[cc])
    return csr_from_directed_pairs(np.concatenate(src_parts), np.concatenate(dst_parts), n)


def sym_norm_weights(csr):
    """Edge weights 1/sqrt(deg_i * deg_j) in CSR order (float32), deg = stored row length.
    Needs a square structure whose every referenced column has a non-empty row."""
    deg = csr.degrees().astype(np.float64)
    rows = csr.row_of_edge()
    w = 1.0 / np.sqrt(deg[rows] * deg[csr.col_idx])
    return w.astype(np.float32)
