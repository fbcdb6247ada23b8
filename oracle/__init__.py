"""CPU oracle for the HyLRA decode-attention step (test infrastructure only).

Only tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import
this package.  It shares nothing with the HIP library.
"""
from .binding import (  # noqa: F401
    append_rows,
    build,
    decode_step,
    full_attn_topk,
    full_attn_topk_blocks,
    gather_blocks,
    gather_rows,
    reuse_block_attn,
    overlap,
    overlap_counts,
    policy_search,
    similarity_matrix,
    reuse_sparse_attn,
    threads,
)
