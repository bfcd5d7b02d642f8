"""MI355X-native neighbour aggregation (SGT + SpMM + SDDMM) -- Python face of libtcgnn.so.

The functions mirror the C ABI in include/tcgnn.h one to one; all computation happens in the
library's HIP kernels."""
from .binding import (  # noqa: F401
    EXPORTED, POLICY_AUTO, POLICY_GATHER, POLICY_TILE, TCG_BF16, TCG_F16, TCG_F32, Meta, TcgError,
    attention, attention_cos, row_rnorm, row_unit_grad, csr_permute, csr_transpose, edge_gather, reorder_rows, load_library, release_cached_memory, row_softmax, row_softmax_backward, sddmm, sddmm_pq, sgt_build, sgt_build_clustered, sgt_export, sgt_plan_stats, sgt_reserve, sgt_set_policy, sgt_tile_stats, spmm, spmm_noalloc,
)
