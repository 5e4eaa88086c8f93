"""MI355X-native ParallelComp hot path: a C-ABI HIP library (csrc/, include/parallelcomp.h)
and its thin Python binding.  Importing the package does not load the library; the first call
does, and raises if the library has not been built (there is no CPU fallback)."""
from .binding import (lib, make_shape, alloc_workspace, pc_shape, PcError, SYMBOLS,
                      pc_chunk_prefill_attn, pc_chunk_prefill_workspace_bytes,
                      pc_chunk_query_scores, pc_chunk_query_scores_workspace_bytes,
                      pc_chunk_self_information, pc_select_chunks_topk, pc_chunk_queue_update, pc_select_tokens_topk, pc_select_tokens_calibrated,
                      pc_gather_kv, pc_gather_kv_amax, pc_kv_append, pc_kv_quantize_fp8, pc_kv_quantize_fp8_amax, pc_parallel_attn_fp8,
                      pc_parallel_attn_fp8_workspace_bytes,
                      pc_parallel_attn, pc_parallel_attn_workspace_bytes,
                      pc_parallel_attn_static, pc_parallel_attn_static_max_bytes,
                      pc_profile_begin, pc_profile_end, pc_profile_records, pc_mfma_ceiling, pc_copy_ceiling)
