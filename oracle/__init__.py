"""fp64 CPU oracle of the ParallelComp hot path.  Test infrastructure only: see parallelcomp.py."""
from .parallelcomp import (rope, rope_angles, local_attention, query_scores, select_chunks, chunk_self_information,
                           select_tokens, select_tokens_calibrated, gather_kv, global_attention_concat,
                           global_attention_merged, lse_merge, parallelcomp_layer, decode_steps,
                           fp8_e4m3_decode, fp8_e4m3_encode, quantize_kv_fp8, dequantize_kv_fp8,
                           chunk_queue_stream)
