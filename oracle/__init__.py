"""CPU oracle for the Chipmunk hot path.  Test infrastructure only.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  The GPU library never does.
"""
from .chipmunk_oracle import (  # noqa: F401
    build,
    num_threads,
    voxel_perm,
    reorder_rows,
    topk_cols,
    mask_to_indices,
    indices_to_mask,
    attn_dense,
    attn_sparse_delta,
    attn_row_stats,
    attn_colsum_stale,
    mlp_dense,
    mlp_tile_scores,
    mlp_sparse_delta,
)
