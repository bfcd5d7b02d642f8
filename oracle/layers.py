"""CPU oracle of the GNN layers (GCN and AGNN layers of the paper's evaluation section, and the
self-attention aggregation SDDMM -> row softmax -> SpMM), values and gradients.

TEST INFRASTRUCTURE ONLY, like the rest of this package.

Every layer is written out by its definition on the DENSE n x n adjacency in fp64 with plain PyTorch
CPU operations; gradients come from PyTorch's reverse-mode differentiation of those dense formulas.
Nothing here knows about CSR kernels, windows or tiles.  The patterns must not contain repeated
(i, j) entries (a dense mask cannot represent them).

    GCN layer        H = A_w (X W^T) + b          A_w[i, j] = edge value of (i, j), 0 elsewhere
    AGNN layer       P = softmax over the stored entries of each row of beta * cos(x_i, x_j);  H = P X
    self-attention   P = softmax over the stored entries of each row of <x_i, x_j>;            H = P X
"""
import numpy as np
import torch


def _rows_of_edges(row_ptr):
    return np.repeat(np.arange(len(row_ptr) - 1), np.diff(row_ptr))


def dense_pattern(row_ptr, col_idx, n_cols, values=None):
    """(mask, A): boolean n_rows x n_cols pattern and the fp64 matrix of edge values (ones if None)."""
    n_rows = len(row_ptr) - 1
    rows = _rows_of_edges(row_ptr)
    mask = np.zeros((n_rows, n_cols), dtype=bool)
    mask[rows, col_idx] = True
    if int(mask.sum()) != len(col_idx):
        raise ValueError("the layer oracle needs a pattern without repeated entries")
    A = np.zeros((n_rows, n_cols), dtype=np.float64)
    A[rows, col_idx] = 1.0 if values is None else np.asarray(values, dtype=np.float64)
    return mask, A


def _t(a, grad=False):
    return torch.tensor(np.asarray(a, dtype=np.float64), dtype=torch.float64, requires_grad=grad)


def _masked_row_softmax(S, mask):
    """Softmax over the True entries of each row; rows without entries give zeros."""
    neg = torch.full_like(S, -float("inf"))
    Sm = torch.where(mask, S, neg)
    m = Sm.max(dim=1, keepdim=True).values
    m = torch.where(torch.isfinite(m), m, torch.zeros_like(m))
    E = torch.where(mask, torch.exp(Sm - m), torch.zeros_like(S))
    den = E.sum(dim=1, keepdim=True)
    return E / torch.where(den > 0, den, torch.ones_like(den))


def _unit_rows(H):
    """Rows scaled to unit Euclidean length; an all-zero row stays zero and passes no gradient (the
    derivative of the square root is never taken at zero)."""
    sq = (H * H).sum(dim=1, keepdim=True)
    pos = sq > 0
    nrm = torch.where(pos, torch.sqrt(torch.where(pos, sq, torch.ones_like(sq))), torch.zeros_like(sq))
    return H / nrm.clamp_min(1e-12)


def _run(fn, inputs, upstream):
    """Evaluates fn on fp64 leaf tensors; returns (value, [gradients of <value, upstream>])."""
    leaves = [_t(a, grad=True) for a in inputs]
    out = fn(*leaves)
    grads = torch.autograd.grad((out * _t(upstream)).sum(), leaves, allow_unused=True)
    return out.detach().numpy(), [None if g is None else g.numpy() for g in grads]


def gcn_conv(row_ptr, col_idx, n_cols, edge_values, X, W, b, dH):
    """GCN layer H = A_w (X W^T) + b.  Returns H and (dX, dW, db, d edge_values in CSR order) for the
    upstream gradient dH."""
    _, A = dense_pattern(row_ptr, col_idx, n_cols, edge_values)
    rows = _rows_of_edges(row_ptr)

    def f(A_, X_, W_, b_):
        return A_ @ (X_ @ W_.T) + b_

    H, (dA, dX, dW, db) = _run(f, [A, X, W, b], dH)
    return H, dX, dW, db, dA[rows, col_idx]


def agnn_conv(row_ptr, col_idx, X, beta, dH):
    """AGNN propagation H = P X, P = row softmax of beta * cos(x_i, x_j) on the pattern.
    Returns H, the attention P in CSR order, dX and dbeta."""
    n = len(row_ptr) - 1
    mask_np, _ = dense_pattern(row_ptr, col_idx, n)
    mask = torch.tensor(mask_np)
    rows = _rows_of_edges(row_ptr)
    keep = {}

    def f(X_, beta_):
        Xn = _unit_rows(X_)
        P = _masked_row_softmax(beta_ * (Xn @ Xn.T), mask)
        keep["P"] = P.detach().numpy()
        return P @ X_

    H, (dX, dbeta) = _run(f, [X, np.float64(beta)], dH)
    return H, keep["P"][rows, col_idx], dX, float(dbeta)


def self_attention(row_ptr, col_idx, X, dH):
    """H = P X with P = row softmax of <x_i, x_j> on the pattern.  Returns H, P in CSR order, dX."""
    n = len(row_ptr) - 1
    mask_np, _ = dense_pattern(row_ptr, col_idx, n)
    mask = torch.tensor(mask_np)
    rows = _rows_of_edges(row_ptr)
    keep = {}

    def f(X_):
        P = _masked_row_softmax(X_ @ X_.T, mask)
        keep["P"] = P.detach().numpy()
        return P @ X_

    H, (dX,) = _run(f, [X], dH)
    return H, keep["P"][rows, col_idx], dX


def spmm_grads(row_ptr, col_idx, n_cols, edge_values, X, dY):
    """Y = A_w X: returns Y, dX = A_w^T dY and dw_e = <dY_i, X_j> in CSR order."""
    _, A = dense_pattern(row_ptr, col_idx, n_cols, edge_values)
    rows = _rows_of_edges(row_ptr)
    Y, (dA, dX) = _run(lambda A_, X_: A_ @ X_, [A, X], dY)
    return Y, dX, dA[rows, col_idx]


def sddmm_grads(row_ptr, col_idx, X, ds):
    """s_e = <x_i, x_j>: returns s in CSR order and dX for the upstream gradient ds (CSR order)."""
    n = len(row_ptr) - 1
    rows = _rows_of_edges(row_ptr)
    G = np.zeros((n, n), dtype=np.float64)
    G[rows, col_idx] = np.asarray(ds, dtype=np.float64)
    S, (dX,) = _run(lambda X_: X_ @ X_.T, [X], G)
    return S[rows, col_idx], dX


def row_unit_grad(X, G, scale=1.0, eps=1e-12):
    """The way back through the row normalisation xn_i = x_i / max(|x_i|, eps): for the gradient G with respect
    to xn, returns scale * r_i (G_i - xn_i <G_i, xn_i>) with r_i = 1 / max(|x_i|, eps), row by row in fp64 --
    the derivative of x / |x| applied to G_i wherever |x_i| >= eps."""
    X = np.asarray(X, dtype=np.float64)
    G = np.asarray(G, dtype=np.float64)
    out = np.zeros_like(X)
    for i in range(X.shape[0]):
        r = 1.0 / max(float(np.sqrt(np.dot(X[i], X[i]))), eps)
        xn = r * X[i]
        out[i] = scale * r * (G[i] - xn * np.dot(G[i], xn))
    return out


def gcn_model(row_ptr, col_idx, edge_values, X, params, dOut):
    """Two-layer GCN of the paper's evaluation: log_softmax(A_w relu(A_w X W1^T + b1) W2^T + b2).
    params = (W1, b1, W2, b2); returns the output and the parameter gradients for upstream dOut."""
    n = len(row_ptr) - 1
    _, A = dense_pattern(row_ptr, col_idx, n, edge_values)
    At, Xt = _t(A), _t(X)

    def f(W1, b1, W2, b2):
        H = torch.relu(At @ (Xt @ W1.T) + b1)
        return torch.log_softmax(At @ (H @ W2.T) + b2, dim=1)

    return _run(f, list(params), dOut)


def agnn_model(row_ptr, col_idx, X, params, betas, dOut):
    """AGNN of the paper's evaluation: linear embedding + relu, len(betas) attention propagations, linear
    read-out, log_softmax.  params = (We, be, Wr, br); returns the output and gradients of params + betas."""
    n = len(row_ptr) - 1
    mask = torch.tensor(dense_pattern(row_ptr, col_idx, n)[0])
    Xt = _t(X)
    n_layers = len(betas)

    def f(We, be, Wr, br, *bs):
        H = torch.relu(Xt @ We.T + be)
        for k in range(n_layers):
            Hn = _unit_rows(H)
            H = _masked_row_softmax(bs[k] * (Hn @ Hn.T), mask) @ H
        return torch.log_softmax(H @ Wr.T + br, dim=1)

    return _run(f, list(params) + [np.float64(b) for b in betas], dOut)
