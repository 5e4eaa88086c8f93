"""Named workload shapes for the chunked-prefill / parallel-attention path.

Shapes only: no arithmetic of the method lives here.  Notation follows the paper's
section 3.1 ("Parallel attention"): C chunks of w context rows, each concatenated with the
same w_q query rows, L = w + w_q rows per chunk sequence, position id = row index.
The chunk+query = pre-training window rule (7680+512 = 8192, 3584+512 = 4096) is the one the
paper's hyperparameter appendix states.
"""
from dataclasses import dataclass, field, replace
from typing import Tuple


@dataclass(frozen=True)
class PrefillConfig:
    name: str
    n_chunks: int          # C
    chunk_len: int         # w
    query_len: int         # w_q
    n_q_heads: int         # H_q
    n_kv_heads: int        # H_kv
    head_dim: int          # D
    rope_base: float
    keep_chunks: int       # k_c (0: selection not part of this workload)
    keep_tokens: int       # k_t
    obs_window: int        # w_obs: last query rows that vote
    entry_scale: float     # std of the Gaussian entries of q, k, v
    n_relevant: int = 0    # chunks whose keys get the planted query direction
    relevant_fixed: Tuple[int, ...] = ()   # fixed relevant chunk ids (else drawn from the seed)
    plant_gain: float = 0.5
    sink_gain: float = 4.0           # norm multiplier of key 0 of every chunk (1 = none)
    key_lognormal_sigma: float = 0.0  # >0: key norms are log-normal with this sigma
    recency_rows: int = 0            # last context rows of each chunk with boosted key norm
    recency_gain: float = 1.0
    q_gain: float = 1.0              # extra multiplier on the query-side entries (q): logit std
    v_offset: float = 0.0            # >0: a constant drawn per (chunk, KV head) from [-v_offset, v_offset] is added to V
    key_norm: float = 1.0            # median key norm when key_lognormal_sigma > 0
    cfg_id: int = 0                  # enters the seed

    @property
    def seq_len(self) -> int:        # L
        return self.chunk_len + self.query_len

    @property
    def group(self) -> int:          # G = H_q / H_kv
        return self.n_q_heads // self.n_kv_heads

    @property
    def context_tokens(self) -> int:
        return self.n_chunks * self.chunk_len


@dataclass(frozen=True)
class DecodeConfig:
    name: str
    batch: int             # B sequences
    n_seg: int             # retained chunks (segments) per sequence
    keep_tokens: int       # k_t rows per KV head per segment
    n_q: int               # new query tokens per step
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    src_rows: int          # rows per source chunk for the gather (2x compression)
    entry_scale: float
    cfg_id: int = 4


_S64 = 1.0 / 8.0
_S128 = 1.0 / (128.0 ** 0.5)

CFG0 = PrefillConfig("cfg0_tiny_mha", 4, 512, 64, 8, 8, 64, 1.0e4, 2, 128, 32, _S64,
                     n_relevant=1, relevant_fixed=(2,), cfg_id=0)
CFG1 = PrefillConfig("cfg1_llama3_8b_128k", 16, 7680, 512, 32, 8, 128, 5.0e5, 8, 2048, 32, _S128,
                     n_relevant=3, cfg_id=1)
CFG2 = PrefillConfig("cfg2_llama2_7b_128k", 36, 3584, 512, 32, 32, 128, 1.0e4, 12, 1024, 32, _S128,
                     sink_gain=1.0, key_lognormal_sigma=0.5, recency_rows=64, recency_gain=2.0,
                     cfg_id=2)
CFG3 = PrefillConfig("cfg3_llama3_8b_512k_stress", 64, 8192, 512, 32, 8, 128, 5.0e5, 0, 0, 32, _S128,
                     sink_gain=1.0, cfg_id=3)
CFG4 = DecodeConfig("cfg4_decode_llama3_8b", 16, 32, 2048, 1, 32, 8, 128, 4096, _S128)

# "u" variants: unit-variance entries, so logits have std ~ 1 and selection gaps are real.
# The planted direction is scaled by sqrt(D) too, so it keeps its size relative to a key.
CFG0U = replace(CFG0, name="cfg0u_tiny_mha_unit", entry_scale=1.0, plant_gain=0.5 * 8.0, cfg_id=10)
CFG1U = replace(CFG1, name="cfg1u_llama3_8b_128k_unit", entry_scale=1.0,
                plant_gain=0.5 * 128.0 ** 0.5, cfg_id=11)

# "p" variants: inputs on which the attention outputs carry signal at the full sizes.  With the
# 1/sqrt(D) entries above, logits have std ~ 1/D: the softmax is flat and an output row is the
# mean of thousands of zero-mean values, far below any tolerance.  Here entries have unit
# variance, q carries a gain (logit std ~ 2: a row's weight sits on a few dozen keys, which fall
# in different key tiles for different rows), and V carries a constant per (chunk, KV head), so
# that a tile taken from another chunk or head shows in the output.  The gains are the largest
# for which bf16 operands (rotated q and k rounded to bf16, probabilities rounded to bf16) stay
# within about 0.6 of the outputs' tolerance when emulated on the CPU; at logit std 3 that
# rounding alone reaches the tolerance on the heaviest rows (the sink key, the log-normal norms).
CFG1P = replace(CFG1U, name="cfg1p_llama3_8b_128k_peaked", q_gain=2.0, v_offset=2.0, sink_gain=1.5,
                cfg_id=41)
CFG2P = replace(CFG2, name="cfg2p_llama2_7b_128k_peaked", entry_scale=1.0, q_gain=0.45,
                key_norm=128.0 ** 0.5, recency_gain=1.25, v_offset=2.0, cfg_id=42)
CFG3P = replace(CFG3, name="cfg3p_llama3_8b_512k_stress_peaked", entry_scale=1.0, q_gain=2.0,
                v_offset=2.0, cfg_id=43)

# Reduced shapes with the same structure as cfg 1 / cfg 2 / cfg 4: several tiles plus a ragged
# tail, small enough for the oracle to finish in seconds.
CFG1_SMALL = replace(CFG1, name="cfg1_small", n_chunks=5, chunk_len=600, query_len=104,
                     keep_chunks=3, keep_tokens=200, n_relevant=2, cfg_id=21)
CFG2_SMALL = replace(CFG2, name="cfg2_small", n_chunks=6, chunk_len=459, query_len=72,
                     n_q_heads=8, n_kv_heads=8, keep_chunks=3, keep_tokens=150, cfg_id=22)
CFG4_SMALL = replace(CFG4, name="cfg4_small", batch=3, n_seg=5, keep_tokens=333, src_rows=700,
                     cfg_id=24)

PREFILL_CONFIGS = {c.name: c for c in (CFG0, CFG1, CFG2, CFG3, CFG0U, CFG1U, CFG1P, CFG2P, CFG3P,
                                       CFG1_SMALL, CFG2_SMALL)}
DECODE_CONFIGS = {c.name: c for c in (CFG4, CFG4_SMALL)}
