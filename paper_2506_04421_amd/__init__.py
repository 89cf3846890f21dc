"""MI355X-native Markovian next-scale attention (HMAR, paper Sec. "Efficient Markovian
Next-Scale Prediction"): Python face of libhmar_attn.so."""
from .binding import (HMAR_MASK_BLOCK_CAUSAL, HMAR_MASK_MARKOV, HMAR_SCALE_COUNTS, KERNEL_NAMES, HmarError,
                      hmar_attn_bwd, hmar_attn_bwd_masked, hmar_attn_bwd_noalloc, hmar_attn_bwd_workspace_bytes,
                      hmar_attn_bwd_workspace_bytes_masked, hmar_attn_fwd, hmar_attn_fwd_masked,
                      hmar_attn_step_fwd, hmar_attn_step_fwd_rows, hmar_attn_steps_fwd, hmar_calibration_copy,
                      hmar_profile_begin, hmar_profile_end, hmar_schedule_describe, hmar_schedule_tiles,
                      load_library, status_string)

__all__ = ["HmarError", "HMAR_MASK_MARKOV", "HMAR_MASK_BLOCK_CAUSAL", "HMAR_SCALE_COUNTS", "KERNEL_NAMES",
           "hmar_attn_fwd", "hmar_attn_fwd_masked", "hmar_attn_step_fwd", "hmar_attn_steps_fwd",
           "hmar_attn_step_fwd_rows", "hmar_attn_bwd", "hmar_attn_bwd_masked", "hmar_attn_bwd_noalloc", "hmar_attn_bwd_workspace_bytes",
           "hmar_attn_bwd_workspace_bytes_masked", "hmar_calibration_copy", "hmar_schedule_describe",
           "hmar_schedule_tiles", "hmar_profile_begin", "hmar_profile_end", "load_library", "status_string"]
