"""Slow, plain CPU definition of the GR forward.  Test infrastructure: see gr_oracle.py."""
from .gr_oracle import (  # noqa: F401
    silu, layernorm, bucket_scalar, bucket_table, bucket_matrix, positions, allow_mask,
    merged_token_offsets, forward_request, forward, forward_request_loops,
    masked_softmax, sigmoid, block_slices, fuse_and_score, climber_request,
)
