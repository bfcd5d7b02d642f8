"""CPU oracle of the row-clustering pass that can run before SGT (the paper calls row reordering
"orthogonal and complementary" to SGT in its related-work section and gives no algorithm; this is the
library's own cheap heuristic, so the oracle states its steps and the GPU path must reproduce the
permutation bit for bit).

TEST INFRASTRUCTURE ONLY, like the rest of this package.  Plain numpy, vectorised so that the
full-size workloads finish in seconds; `reorder_rows_loops` is the same thing in explicit Python
loops for small cases and serves as a cross-check of the vectorised form.

The heuristic (square n x n pattern, nodes = rows = columns):
  1. hash(v) = splitmix64 of (seed, v); nodes are compared by (hash, id).
  2. parent(v) = the smallest node of {v} + N(v)          (N(v) = stored columns of row v)
  3. root(v)   = the fixed point of v -> parent(v)          (hashes fall along the chain, so it ends)
  4. label = root; then `refine` synchronous rounds of
        label'(v) = the most frequent label among the first min(deg, 128) stored neighbours of v
                    (repeated entries count; ties go to the smallest label id; empty rows keep theirs)
  5. perm = the nodes sorted by (label, parent, id); perm[new] = old.
Nodes that share neighbours tend to share the smallest neighbour, so they end up in the same tree and
next to each other: the 16-row windows built afterwards see fewer distinct columns.
"""
import numpy as np

REFINE_MAX_NEIGHBOURS = 128

_M64 = (1 << 64) - 1


def node_hash(seed, ids):
    """splitmix64 output function applied to seed + (id + 1) * golden ratio increment; uint64."""
    with np.errstate(over="ignore"):
        z = np.uint64(seed & _M64) + (np.asarray(ids, dtype=np.uint64) + np.uint64(1)) * np.uint64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return z ^ (z >> np.uint64(31))


def _check_square(row_ptr, col_idx):
    n = len(row_ptr) - 1
    if len(col_idx) and (col_idx.min() < 0 or col_idx.max() >= n):
        raise ValueError("row clustering needs a square pattern (columns are node ids)")
    return n


def parents(row_ptr, col_idx, seed):
    n = _check_square(row_ptr, col_idx)
    h = node_hash(seed, np.arange(n))
    rows = np.repeat(np.arange(n, dtype=np.int64), np.diff(row_ptr))
    cand_row = np.concatenate([rows, np.arange(n, dtype=np.int64)])          # every node is its own candidate
    cand_col = np.concatenate([np.asarray(col_idx, dtype=np.int64), np.arange(n, dtype=np.int64)])
    order = np.lexsort((cand_col, h[cand_col], cand_row))                    # by row, then (hash, id)
    first = np.ones(len(order), dtype=bool)
    first[1:] = cand_row[order][1:] != cand_row[order][:-1]
    return cand_col[order][first].astype(np.int32)                           # one winner per row, rows ascending


def roots(parent):
    root = parent.copy()
    while True:
        nxt = root[root]
        if np.array_equal(nxt, root):
            return root
        root = nxt


def refine_once(row_ptr, col_idx, label):
    n = len(row_ptr) - 1
    deg = np.minimum(np.diff(row_ptr), REFINE_MAX_NEIGHBOURS)
    rows = np.repeat(np.arange(n, dtype=np.int64), deg)
    start = np.repeat(np.asarray(row_ptr[:-1], dtype=np.int64), deg)
    within = np.arange(len(rows), dtype=np.int64) - np.repeat(np.cumsum(deg) - deg, deg)
    nb_label = label[col_idx[start + within]].astype(np.int64)
    order = np.lexsort((nb_label, rows))
    r, l = rows[order], nb_label[order]
    run_start = np.ones(len(r), dtype=bool)
    run_start[1:] = (r[1:] != r[:-1]) | (l[1:] != l[:-1])
    idx = np.nonzero(run_start)[0]
    count = np.diff(np.append(idx, len(r)))
    rr, ll = r[idx], l[idx]
    best = np.lexsort((ll, -count, rr))                                      # per row: most frequent, then smallest label
    pick = np.ones(len(best), dtype=bool)
    pick[1:] = rr[best][1:] != rr[best][:-1]
    out = label.copy()
    out[rr[best][pick]] = ll[best][pick].astype(label.dtype)
    return out


def reorder_rows(row_ptr, col_idx, seed=0, refine=0):
    """Returns (perm, label, parent): perm[new] = old, int32."""
    row_ptr = np.asarray(row_ptr)
    col_idx = np.asarray(col_idx)
    n = _check_square(row_ptr, col_idx)
    parent = parents(row_ptr, col_idx, seed)
    label = roots(parent)
    for _ in range(refine):
        label = refine_once(row_ptr, col_idx, label)
    perm = np.lexsort((np.arange(n), parent, label)).astype(np.int32)
    return perm, label, parent


def reorder_rows_loops(row_ptr, col_idx, seed=0, refine=0):
    """The same steps in explicit loops (small inputs only)."""
    n = _check_square(np.asarray(row_ptr), np.asarray(col_idx))
    h = [int(x) for x in node_hash(seed, np.arange(n))]
    parent = []
    for v in range(n):
        best = v
        for e in range(row_ptr[v], row_ptr[v + 1]):
            u = int(col_idx[e])
            if (h[u], u) < (h[best], best):
                best = u
        parent.append(best)
    label = []
    for v in range(n):
        p = v
        while parent[p] != p:
            p = parent[p]
        label.append(p)
    for _ in range(refine):
        new = list(label)
        for v in range(n):
            counts = {}
            for e in range(row_ptr[v], min(row_ptr[v + 1], row_ptr[v] + REFINE_MAX_NEIGHBOURS)):
                lb = label[int(col_idx[e])]
                counts[lb] = counts.get(lb, 0) + 1
            if counts:
                top = max(counts.values())
                new[v] = min(lb for lb, c in counts.items() if c == top)
        label = new
    perm = sorted(range(n), key=lambda v: (label[v], parent[v], v))
    return np.array(perm, np.int32), np.array(label, np.int32), np.array(parent, np.int32)


def csr_permute(row_ptr, col_idx, perm):
    """Symmetric permutation of a square CSR pattern: new row i is old row perm[i], and every column id c
    becomes the new position of node c.  Entries keep their order inside a row.  Returns
    (row_ptr', col_idx', edge_perm) with entry k of the result being entry edge_perm[k] of the input."""
    row_ptr = np.asarray(row_ptr)
    col_idx = np.asarray(col_idx)
    perm = np.asarray(perm, dtype=np.int64)
    n = len(row_ptr) - 1
    if sorted(perm.tolist()) != list(range(n)):
        raise ValueError("perm is not a permutation of the nodes")
    inv = np.empty(n, dtype=np.int64)
    inv[perm] = np.arange(n)
    deg = np.diff(row_ptr)[perm]
    new_ptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int32)
    start = np.repeat(np.asarray(row_ptr[:-1], dtype=np.int64)[perm], deg)
    within = np.arange(int(new_ptr[-1]), dtype=np.int64) - np.repeat(new_ptr[:-1].astype(np.int64), deg)
    edge_perm = (start + within).astype(np.int32)
    new_col = inv[col_idx[edge_perm]].astype(np.int32)
    return new_ptr, new_col, edge_perm
