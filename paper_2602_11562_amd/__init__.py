"""MI355X-native STA + GSTA forward path of LASER (arxiv 2602.11562).

The product is `liblaser.so` (HIP kernels behind a C ABI, see include/laser.h);
this package holds its sources (`csrc/`), the build step and a ctypes binding.
"""
from .binding import (LaserError, laser_forward, laser_forward_fused, laser_multires_forward, laser_forward_multires,
                      laser_gsta_forward_multires,
                      laser_segment_ffn_forward, laser_ffn_gsta_forward, FFN_AUTO, FFN_GENERIC, FFN_MFMA, laser_project_q_forward,
                      laser_project_kv_forward, laser_fold_query_weights, laser_project_heads_forward,
                      laser_sta_folded_forward, laser_forward_ragged, laser_multires_forward_ragged, laser_segment_ffn_forward_ragged,
                      laser_sta_backward, laser_sta_backward_static, laser_gsta_backward, PROJECT_AUTO, PROJECT_GENERIC, PROJECT_MFMA, laser_gsta_forward, laser_sta_forward, laser_sta_kernel_name,
                      laser_gsta_kernel_name, laser_version, load_library, status_string,
                      LASER_F32, LASER_BF16, STA_AUTO, STA_GENERIC, STA_MFMA, STA_STREAM,
                      GSTA_AUTO, GSTA_GENERIC, GSTA_TILED, GSTA_SPLIT)

__all__ = ["LaserError", "laser_forward", "laser_forward_fused", "laser_multires_forward", "laser_forward_multires", "laser_gsta_forward_multires", "laser_segment_ffn_forward", "laser_ffn_gsta_forward",
           "FFN_AUTO", "FFN_GENERIC", "FFN_MFMA", "laser_project_q_forward", "laser_project_kv_forward",
           "laser_fold_query_weights", "laser_project_heads_forward", "laser_sta_folded_forward", "laser_forward_ragged", "laser_multires_forward_ragged",
           "laser_segment_ffn_forward_ragged", "laser_sta_backward", "laser_sta_backward_static", "laser_gsta_backward",
           "PROJECT_AUTO", "PROJECT_GENERIC", "PROJECT_MFMA", "laser_gsta_forward", "laser_sta_forward", "laser_sta_kernel_name",
           "laser_gsta_kernel_name", "laser_version", "load_library", "status_string",
           "LASER_F32", "LASER_BF16", "STA_AUTO", "STA_GENERIC", "STA_MFMA", "STA_STREAM",
           "GSTA_AUTO", "GSTA_GENERIC", "GSTA_TILED", "GSTA_SPLIT"]
