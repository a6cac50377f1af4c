"""MI355X-native forward pass of the MeteoRA linear layer (paper Sec. 3.1, Eq. 2).

The compute lives in libmeteora.so (hand-written HIP for gfx950, C ABI in
include/meteora.h).  This package is only the argument-marshalling binding.
"""
from .binding import (MeteoraError, base_gemm, bucket_tokens, bucket_tokens_noalloc, gate_backward, gate_backward_workspace_bytes,  # noqa: F401
                      gate_topk, group_workspace_bytes, init, workspace_regions,
                      library_path, linear_forward, linear_forward_group, load_library, lora_forward, pack_weights,
                      packed_bytes, stage_timing_enable, stage_timing_read, workspace_bytes,
                      BMM_GATHER, LOOP_ORIGINAL, variant_forward, variant_workspace_bytes)
