"""GNN layers on top of the library's graph kernels (the user surface of the paper's section 4 listing:
pre-built GCN / AGNN layers plus differentiable low-level spmm / sddmm).

Everything that touches the graph -- aggregation, edge scores, row softmax and all of their gradients --
runs in libtcgnn.so; PyTorch supplies the dense update phase (a linear layer, i.e. a ROCm BLAS GEMM, which
the paper leaves to the vendor library as well), the element-wise glue and the autograd tape.

Gradients (A is the n_rows x n_cols pattern, e an edge (i, j), w its value):
    Y = (w . A) X         dX = (w . A)^T dY                      dw_e = <dY_i, X_j>
    s_e = <X_i, X_j>      dX = (ds . A) X + (ds . A)^T X
    p = row_softmax(s)    ds_e = p_e (dp_e - sum_{e' in row} p_e' dp_e')
The transposed products use a second SGT plan built on the transposed pattern; the permutation that the
transposition returns carries edge values from one edge order to the other.  When the pattern is symmetric
(every undirected graph) the transposed pattern is the pattern itself: no second plan is built, and the two
products of a score gradient, (ds . A) X + (ds . A)^T X, become one with the edge values ds_ij + ds_ji.
"""
import torch

from . import binding as _b


class TiledGraph:
    """A CSR pattern on the GPU with its SGT plan, and -- built on first use -- the plan of the transposed
    pattern that the backward pass needs.  Stands where the paper's listing has `tiledGraph`."""

    def __init__(self, row_ptr, col_idx, n_cols=None, window_h=16, tile_w=8, validate=True):
        self.row_ptr = row_ptr.contiguous()
        self.col_idx = col_idx.contiguous()
        self.window_h, self.tile_w = window_h, tile_w
        self.meta = _b.sgt_build(self.row_ptr, self.col_idx, window_h, tile_w, n_cols=n_cols, validate=validate)
        self.n_rows, self.n_cols, self.nnz = self.meta.n_rows, self.meta.n_cols, self.meta.nnz
        self._t = None
        self.symmetric = False          # known once transposed() has run

    def transposed(self):
        """(plan of A^T, perm) with edge k of A^T being edge perm[k] of A.  For a symmetric pattern the plan is
        the graph's own (self.symmetric is set) and perm pairs every edge with its reverse."""
        if self._t is None:
            rpt, cit, perm = _b.csr_transpose(self.row_ptr, self.col_idx, n_cols=self.n_cols)
            self.symmetric = bool(self.n_rows == self.n_cols and torch.equal(rpt, self.row_ptr)
                                  and torch.equal(cit, self.col_idx))
            if self.symmetric:
                meta_t = self.meta
            else:
                meta_t = _b.sgt_build(rpt, cit, self.window_h, self.tile_w, n_cols=self.n_rows, validate=False)
            self._t = (meta_t, perm)
        return self._t

    def both_sides(self, X, g):
        """(g . A) X + (g . A)^T X for edge values g: the gradient of a score s_e = <X_i, X_j> with respect to X."""
        meta_t, perm = self.transposed()
        g_t = _b.edge_gather(perm, g)
        if self.symmetric:
            return _b.spmm(self.meta, X, g_t.add_(g))
        out = _b.spmm(self.meta, X, g)
        out += _b.spmm(meta_t, X, g_t)
        return out

    def set_policy(self, policy, min_reuse=0.0):
        _b.sgt_set_policy(self.meta, policy, min_reuse)
        if self._t is not None and self._t[0] is not self.meta:
            _b.sgt_set_policy(self._t[0], policy, min_reuse)

    def free(self):
        if self._t is not None:
            if self._t[0] is not self.meta:
                self._t[0].free()
            self._t = None
        self.meta.free()


def _f32c(t):
    return t.contiguous() if t.dtype == torch.float32 else t.to(torch.float32).contiguous()


class _SpMM(torch.autograd.Function):
    @staticmethod
    def forward(ctx, graph, X, w):
        ctx.graph = graph
        ctx.save_for_backward(X, w)
        return _b.spmm(graph.meta, X.contiguous(), None if w is None else _f32c(w))

    @staticmethod
    def backward(ctx, dY):
        graph = ctx.graph
        X, w = ctx.saved_tensors
        dX = dw = None
        dY = dY.contiguous()
        if ctx.needs_input_grad[1]:
            meta_t, perm = graph.transposed()
            w_t = None if w is None else _b.edge_gather(perm, _f32c(w))
            dX = _b.spmm(meta_t, dY.to(X.dtype), w_t).to(X.dtype)
        if w is not None and ctx.needs_input_grad[2]:
            dw = _b.sddmm_pq(graph.meta, dY.to(X.dtype), X.contiguous()).to(w.dtype)
        return None, dX, dw


class _SDDMM(torch.autograd.Function):
    @staticmethod
    def forward(ctx, graph, X):
        ctx.graph = graph
        ctx.save_for_backward(X)
        return _b.sddmm(graph.meta, X.contiguous())

    @staticmethod
    def backward(ctx, ds):
        graph = ctx.graph
        (X,) = ctx.saved_tensors
        dX = graph.both_sides(X.contiguous(), _f32c(ds))
        return None, dX.to(X.dtype)


class _RowSoftmax(torch.autograd.Function):
    @staticmethod
    def forward(ctx, graph, s):
        p = _b.row_softmax(graph.meta, _f32c(s))
        ctx.graph = graph
        ctx.save_for_backward(p)
        return p

    @staticmethod
    def backward(ctx, dp):
        (p,) = ctx.saved_tensors
        return None, _b.row_softmax_backward(ctx.graph.meta, p, _f32c(dp))


class _SelfAttention(torch.autograd.Function):
    """Y_i = sum_e softmax_i(<X_i, X_j>)_e X_j through the fused forward kernel."""

    @staticmethod
    def forward(ctx, graph, X):
        Xc = X.contiguous()
        s = torch.empty(graph.nnz, dtype=torch.float32, device=X.device)
        Y = _b.attention(graph.meta, Xc, scores=s)
        ctx.graph = graph
        ctx.save_for_backward(Xc, s)
        return Y

    @staticmethod
    def backward(ctx, dY):
        graph = ctx.graph
        Xc, s = ctx.saved_tensors
        meta_t, perm = graph.transposed()
        dY = dY.contiguous().to(Xc.dtype)
        p = _b.row_softmax(graph.meta, s)
        dp = _b.sddmm_pq(graph.meta, dY, Xc)
        ds = _b.row_softmax_backward(graph.meta, p, dp)
        dX = _b.spmm(meta_t, dY, _b.edge_gather(perm, p))          # through the aggregated values
        dX += graph.both_sides(Xc, ds)                             # through both sides of the scores
        return None, dX.to(Xc.dtype)


class _CosAttention(torch.autograd.Function):
    """Y_i = sum_e softmax_i(beta cos(x_i, x_j))_e x_j -- the AGNN propagation -- through the fused kernel
    forward (inverse row norms from one small kernel, X gathered once per edge) and the library's building
    blocks backward.  With r = 1 / max(|x|, eps), xn = r x, c_e = <xn_i, xn_j>, p = row softmax of beta c:
        dp = sddmm_pq(dY, X),  ds = row_softmax_backward(p, dp),  dbeta = sum_e ds_e c_e,
        dXn = (ds . A) Xn + (ds . A)^T Xn,   dX = (p . A)^T dY + beta r (dXn - xn <dXn, xn>)
    (dc = beta ds, and everything after it is linear in dc, so beta joins r in the last step; for a row shorter than
    eps the projection term vanishes with xn, as in the clamped normalisation)."""

    EPS = 1e-12

    @staticmethod
    def forward(ctx, graph, X, beta):
        Xc = _f32c(X) if X.dtype == torch.float32 else X.contiguous()
        r = _b.row_rnorm(Xc, _CosAttention.EPS)
        c = torch.empty(graph.nnz, dtype=torch.float32, device=X.device)
        ctx.beta_value = float(beta)          # read once: the kernels take it as a plain number
        Y = _b.attention_cos(graph.meta, Xc, r, ctx.beta_value, scores=c)
        ctx.graph = graph
        ctx.save_for_backward(Xc, r, c, beta)
        return Y

    @staticmethod
    def backward(ctx, dY):
        graph = ctx.graph
        Xc, r, c, beta = ctx.saved_tensors
        meta_t, perm = graph.transposed()
        dY = dY.contiguous().to(Xc.dtype)
        p = _b.row_softmax(graph.meta, c * beta)
        dp = _b.sddmm_pq(graph.meta, dY, Xc)
        ds = _b.row_softmax_backward(graph.meta, p, dp)
        dbeta = torch.dot(ds, c) if ctx.needs_input_grad[2] else None
        dX = None
        if ctx.needs_input_grad[1]:
            Xn = (Xc.to(torch.float32) * r[:, None]).to(Xc.dtype)
            dXn = graph.both_sides(Xn, ds)
            dX = _b.spmm(meta_t, dY, _b.edge_gather(perm, p))
            _b.row_unit_grad(Xc, r, dXn, dX, scale=ctx.beta_value)     # dX += beta r (dXn - xn <dXn, xn>)
            dX = dX.to(Xc.dtype)
        return None, dX, dbeta


def _tall_tn(A, B, chunk=4096):
    """A^T B for tall A [N, p] and B [N, q]: the reduction over the N nodes is cut into chunks that run as
    one batched GEMM and are then added, which gives the BLAS library parallel work when p and q are
    small (a plain GEMM call reduces over all N inside a handful of workgroups)."""
    N = A.shape[0]
    S = N // chunk
    if S < 2:
        return A.t() @ B
    head = S * chunk
    A, B = A.contiguous(), B.contiguous()
    out = torch.bmm(A[:head].view(S, chunk, -1).transpose(1, 2), B[:head].view(S, chunk, -1)).sum(dim=0)
    if head < N:
        out += A[head:].t() @ B[head:]
    return out


class _NodeLinear(torch.autograd.Function):
    """Z = X W^T with one row of X per node (the update phase); only the weight gradient differs from
    torch's own linear: it uses the chunked reduction above."""

    @staticmethod
    def forward(ctx, X, W):
        ctx.save_for_backward(X, W)
        return X @ W.t()

    @staticmethod
    def backward(ctx, dZ):
        X, W = ctx.saved_tensors
        dX = dZ @ W if ctx.needs_input_grad[0] else None
        dW = _tall_tn(dZ, X) if ctx.needs_input_grad[1] else None
        return dX, dW


class NodeLinear(torch.nn.Module):
    """Linear update of node features, Z = X W^T (+ b), initialised like torch.nn.Linear."""

    def __init__(self, in_features, out_features, bias=True):
        super().__init__()
        ref = torch.nn.Linear(in_features, out_features, bias=bias)
        self.in_features, self.out_features = in_features, out_features
        self.weight = torch.nn.Parameter(ref.weight.detach().clone())
        self.bias = torch.nn.Parameter(ref.bias.detach().clone()) if bias else None

    def forward(self, X):
        Z = _NodeLinear.apply(X, self.weight)
        return Z if self.bias is None else Z + self.bias


def spmm(graph, X, w=None):
    """Differentiable Y = (w . A) X (Eq. 1); w = None means unit edge values."""
    return _SpMM.apply(graph, X, w)


def sddmm(graph, X):
    """Differentiable s_e = <X_i, X_j> over the edges (Eq. 2), fp32 in CSR order."""
    return _SDDMM.apply(graph, X)


def row_softmax(graph, s):
    """Differentiable softmax over the stored entries of each row."""
    return _RowSoftmax.apply(graph, s)


def self_attention(graph, X):
    """Differentiable fused SDDMM -> row softmax -> SpMM with X as query, key and value."""
    return _SelfAttention.apply(graph, X)


def _fused_attention_ok(X):
    """The fused attention kernels read rows in 16-byte pieces of at most 2 KB."""
    row_bytes = X.shape[1] * X.element_size()
    return row_bytes % 16 == 0 and row_bytes <= 2048 and (X.stride(0) * X.element_size()) % 16 == 0


def cos_attention(graph, X, beta):
    """Differentiable Y_i = sum_e softmax_i(beta cos(x_i, x_j))_e x_j (fused forward); beta: 0-d tensor."""
    return _CosAttention.apply(graph, X, beta)


class GCNConv(torch.nn.Module):
    """Graph convolution: neighbour aggregation with fixed edge values (the symmetric normalisation
    1/sqrt(deg_i deg_j) in the GCN model) and a linear update.  The update is applied on whichever side
    of the aggregation handles the narrower features, which changes rounding only."""

    def __init__(self, in_dim, out_dim, bias=True):
        super().__init__()
        self.linear = NodeLinear(in_dim, out_dim, bias=False)
        self.bias = torch.nn.Parameter(torch.zeros(out_dim)) if bias else None

    def forward(self, X, graph, edge_values=None):
        if self.linear.in_features > self.linear.out_features:
            out = self.linear.out_features
            pad = (-out) % 4
            if pad and graph.nnz >= (1 << 20):
                # A handful of classes on a large graph: aggregate rows padded with zero columns to whole
                # 16-byte pieces (the vector kernels; 10 fp32 columns would go piece by piece) and drop the
                # padding afterwards.  On small graphs the extra launches cost more than they save.
                W = torch.nn.functional.pad(self.linear.weight, (0, 0, 0, pad))
                H = spmm(graph, _NodeLinear.apply(X, W), edge_values)[:, :out]
            else:
                H = spmm(graph, self.linear(X), edge_values)
        else:
            H = self.linear(spmm(graph, X, edge_values))
        return H if self.bias is None else H + self.bias


class AGNNConv(torch.nn.Module):
    """Attention-based propagation: edge scores beta * cos(x_i, x_j) by SDDMM on the normalised rows,
    softmax over each row's edges, aggregation of the unnormalised rows with those weights."""

    def __init__(self, init_beta=1.0, learn_beta=True):
        super().__init__()
        beta = torch.tensor(float(init_beta))
        if learn_beta:
            self.beta = torch.nn.Parameter(beta)
        else:
            self.register_buffer("beta", beta)

    def forward(self, X, graph):
        if _fused_attention_ok(X):
            return _CosAttention.apply(graph, X, self.beta)
        Xn = torch.nn.functional.normalize(X, p=2.0, dim=1)
        p = row_softmax(graph, self.beta * sddmm(graph, Xn))
        return spmm(graph, X, p)


class GCN(torch.nn.Module):
    """The paper's GCN benchmark model: two GCNConv layers (16 hidden features in the evaluation)."""

    def __init__(self, in_dim, hidden_dim, out_dim):
        super().__init__()
        self.layer1 = GCNConv(in_dim, hidden_dim)
        self.layer2 = GCNConv(hidden_dim, out_dim)

    def forward(self, X, graph, edge_values=None):
        H = torch.relu(self.layer1(X, graph, edge_values))
        return torch.log_softmax(self.layer2(H, graph, edge_values), dim=1)


class AGNN(torch.nn.Module):
    """The paper's AGNN benchmark model: linear embedding, n_layers attention propagations (4 layers of
    32 hidden features in the evaluation), linear read-out."""

    def __init__(self, in_dim, hidden_dim, out_dim, n_layers=4):
        super().__init__()
        self.embed = NodeLinear(in_dim, hidden_dim)
        self.props = torch.nn.ModuleList([AGNNConv() for _ in range(n_layers)])
        self.readout = NodeLinear(hidden_dim, out_dim)

    def forward(self, X, graph):
        H = torch.relu(self.embed(X))
        for prop in self.props:
            H = prop(H, graph)
        return torch.log_softmax(self.readout(H), dim=1)
