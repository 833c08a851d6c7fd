"""fp64 CPU checker of the STA + GSTA forward pass. Test infrastructure only:
imported by tests/, by the smoke check and by the benchmark's CPU-baseline leg."""
from .laser_oracle import (num_segments, segment_counts, sigmoid, sta_segment, sta_pair, sta_pair_global, sta_pair_heads, sta_pair_softmax,
                           gsta_pair, sta_forward, gsta_forward, laser_forward, laser_forward_ragged, multires_pair, multires_forward,
                           segment_ffn_vector, segment_ffn_forward, project_rows, project_qkv, fold_query_weights, project_heads,
                           sta_folded_forward, sta_backward, gsta_pair_backward, gsta_backward)

__all__ = ["num_segments", "segment_counts", "sigmoid", "sta_segment", "sta_pair", "sta_pair_global", "sta_pair_heads", "sta_pair_softmax",
           "gsta_pair", "sta_forward", "gsta_forward", "laser_forward", "laser_forward_ragged", "multires_pair", "multires_forward",
           "segment_ffn_vector", "segment_ffn_forward", "project_rows", "project_qkv", "fold_query_weights", "project_heads",
           "sta_folded_forward", "sta_backward", "gsta_pair_backward", "gsta_backward"]
