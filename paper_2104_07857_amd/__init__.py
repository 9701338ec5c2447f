"""MI355X-native optimizer hot path for offloaded, partitioned mixed-precision training.

A thin binding over libzi.so (hand-written HIP for gfx950 behind a C ABI, see
include/zi.h).  PyTorch is used by callers for device memory and streams only.
"""
from .binding import *  # noqa: F401,F403
from .binding import (EXPORTS, LIB_PATH, ZiError, lib, make_config, make_file_tensors, make_tensors,
                      zi_adamw_config, zi_file_tensor,
                      zi_chunk_segment, zi_norm_result, zi_step_plan_item, zi_stream_stats, zi_tensor)
