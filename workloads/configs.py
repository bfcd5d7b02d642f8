"""The five benchmark workloads, by number (1-based, as listed in the baseline description).

`make_config(k)` returns a dict:
  csr      CSR structure (int32)
  X        float32 [N, D] (bf16-exact values when 'x_dtype' == 'bf16')
  x_dtype  'f32' or 'bf16' -- the storage type the GPU library is given
  w        float32 [nnz] edge weights in CSR order, or None (unit weights)
  ops      tuple of the operations the workload runs
  name     short label
`n` overrides the node count (same recipe, smaller graph) for parity tests.
"""
from . import graphs, features

CONFIGS = {
    1: "er2k_d16_f32",
    2: "chunglu20k_d64_f32",
    3: "rmat100k_d32_f32_attention",
    4: "rmat1m_d128",
    5: "clustered200k_d256_bf16",
}


def make_config(k, n=None, x_dtype=None, seed=0, permute=True, d=None):
    if k == 1:
        n = n or 2048
        d = d or 16
        csr = graphs.erdos_renyi_gnm(n, 2 * n, seed, self_loops=True)
        X = features.features_uniform(n, d, seed)
        w = graphs.sym_norm_weights(csr)
        xd = x_dtype or "f32"
        ops = ("sgt", "spmm")
    elif k == 2:
        n = n or 20000
        d = d or 64
        csr = graphs.chung_lu_powerlaw(n, seed, 2.1, 5.0, 500.0, self_loops=True)
        X = features.features_normal(n, d, seed)
        w = graphs.sym_norm_weights(csr)
        xd = x_dtype or "f32"
        ops = ("sgt", "spmm")
    elif k == 3:
        n = n or 100000
        d = d or 32
        scale = max(1, (n - 1).bit_length())
        csr = graphs.rmat(n, scale, 20 * n, seed)
        X = features.features_normal(n, d, seed)
        w = None
        xd = x_dtype or "f32"
        ops = ("sgt", "sddmm", "row_softmax", "spmm")
    elif k == 4:
        n = n or 1000000
        d = d or 128
        scale = max(1, (n - 1).bit_length())
        csr = graphs.rmat(n, scale, 10 * n, seed)
        X = features.features_uniform(n, d, seed)
        w = None
        xd = x_dtype or "f32"
        ops = ("sgt", "spmm")
    elif k == 5:
        n = n or 200000
        d = d or 256
        assert n % 64 == 0
        csr = graphs.clustered_communities(n // 64, 64, 0.3, 0.01, seed, permute=permute)
        X = features.features_normal(n, d, seed)
        w = None
        xd = x_dtype or "bf16"
        ops = ("sgt", "sddmm", "spmm")
    else:
        raise ValueError("config must be 1..5")
    if xd == "bf16":
        X = features.round_to_bf16(X)
    name = CONFIGS[k] + ("" if k != 5 or permute else "_unpermuted")
    return dict(csr=csr, X=X, x_dtype=xd, w=w, ops=ops, name=name, config=k)
