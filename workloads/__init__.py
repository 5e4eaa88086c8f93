"""Seeded synthetic workloads (shapes and input generators) shared by the oracle and the HIP path."""
from .configs import (PrefillConfig, DecodeConfig, CFG0, CFG1, CFG2, CFG3, CFG4, CFG0U, CFG1U, CFG1P, CFG2P, CFG3P,
                      CFG1_SMALL, CFG2_SMALL, CFG4_SMALL, PREFILL_CONFIGS, DECODE_CONFIGS)
from .gen import (f32_to_bf16_bits, bf16_bits_to_f32, bf16_bits_to_f64, prefill_chunk,
                  prefill_inputs, decode_inputs, gather_inputs, relevant_chunks, lm_logits_inputs, v_offsets)
