"""Seeded synthetic inputs for the chunked-prefill / parallel-attention path.

These generators serve both the CPU oracle and the HIP path and contain none of the method's
arithmetic: only Gaussian draws, norm scaling, an added direction, and one rounding to bf16.
Every tensor is returned as raw bf16 bits (uint16) so both sides consume identical values.

The structure planted here stands in for what the paper observes in trained models (its
empirical study of attention bias): a sink at the first key of a chunk, a recency bump at the
chunk tail, and chunks that are relevant to the query.
"""
from concurrent.futures import ThreadPoolExecutor
import numpy as np

from .configs import PrefillConfig, DecodeConfig

BASE_SEED = 2502

# stream ids inside one config's seed space
_STREAM_QUERY = 1_000_000
_STREAM_RELEVANT = 1_000_001
_STREAM_DECODE_Q = 1_000_002
_STREAM_GATHER_IDX = 1_000_003
_STREAM_V_OFFSET = 1_000_004


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (round-to-nearest-even), return the 16-bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(b).astype(np.float64)


def _rng(cfg_id: int, stream: int) -> np.random.Generator:
    return np.random.default_rng([BASE_SEED, int(cfg_id), int(stream)])


def _normal(rng, shape, scale):
    a = rng.standard_normal(shape, dtype=np.float32)
    if scale != 1.0:
        a *= np.float32(scale)
    return a


def relevant_chunks(cfg: PrefillConfig) -> np.ndarray:
    """Sorted ids of the chunks that carry the planted query direction."""
    if cfg.n_relevant == 0:
        return np.zeros(0, dtype=np.int64)
    if cfg.relevant_fixed:
        return np.array(sorted(cfg.relevant_fixed), dtype=np.int64)
    rng = _rng(cfg.cfg_id, _STREAM_RELEVANT)
    return np.sort(rng.choice(cfg.n_chunks, size=cfg.n_relevant, replace=False))


def _key_norm_structure(cfg: PrefillConfig, rng, k_rows: np.ndarray, first_row: int):
    """Log-normal key norms (direction kept, norm replaced)."""
    if cfg.key_lognormal_sigma > 0.0:
        nrm = np.linalg.norm(k_rows, axis=-1, keepdims=True)
        z = rng.standard_normal(nrm.shape, dtype=np.float32)
        k_rows *= np.float32(cfg.key_norm) * np.exp(np.float32(cfg.key_lognormal_sigma) * z) / np.maximum(nrm, 1e-20)
    return k_rows


def v_offsets(cfg: PrefillConfig) -> np.ndarray:
    """[C + 1, H_kv] constants added to V: row c for chunk c's context rows, row C for the query
    rows.  Zeros when the config has no offset."""
    if cfg.v_offset <= 0.0:
        return np.zeros((cfg.n_chunks + 1, cfg.n_kv_heads), dtype=np.float32)
    rng = _rng(cfg.cfg_id, _STREAM_V_OFFSET)
    return (rng.uniform(-1.0, 1.0, size=(cfg.n_chunks + 1, cfg.n_kv_heads)) * cfg.v_offset).astype(np.float32)


def query_rows_f32(cfg: PrefillConfig):
    """The w_q query rows (q, k, v), identical in every chunk, before rounding."""
    rng = _rng(cfg.cfg_id, _STREAM_QUERY)
    q = _normal(rng, (cfg.query_len, cfg.n_q_heads, cfg.head_dim), cfg.entry_scale * cfg.q_gain)
    k = _normal(rng, (cfg.query_len, cfg.n_kv_heads, cfg.head_dim), cfg.entry_scale)
    v = _normal(rng, (cfg.query_len, cfg.n_kv_heads, cfg.head_dim), cfg.entry_scale)
    k = _key_norm_structure(cfg, rng, k, cfg.chunk_len)
    if cfg.v_offset > 0.0:
        v += v_offsets(cfg)[cfg.n_chunks][None, :, None]
    return q, k, v


def mean_query_direction(cfg: PrefillConfig, q_query: np.ndarray) -> np.ndarray:
    """Unit vector per KV head: mean of the group's query heads over all query rows."""
    m = q_query.astype(np.float64).reshape(cfg.query_len, cfg.n_kv_heads, cfg.group, cfg.head_dim)
    m = m.mean(axis=(0, 2))
    m /= np.linalg.norm(m, axis=-1, keepdims=True)
    return m.astype(np.float32)


def prefill_chunk(cfg: PrefillConfig, c: int, _cache=None):
    """bf16 bits of chunk sequence c: q [L,H_q,D], k [L,H_kv,D], v [L,H_kv,D]."""
    if _cache is None:
        _cache = _prefill_shared(cfg)
    qq, kq, vq, u, rel = _cache
    rng = _rng(cfg.cfg_id, c)
    w = cfg.chunk_len
    q = _normal(rng, (w, cfg.n_q_heads, cfg.head_dim), cfg.entry_scale * cfg.q_gain)
    k = _normal(rng, (w, cfg.n_kv_heads, cfg.head_dim), cfg.entry_scale)
    v = _normal(rng, (w, cfg.n_kv_heads, cfg.head_dim), cfg.entry_scale)
    k = _key_norm_structure(cfg, rng, k, 0)
    if cfg.v_offset > 0.0:
        v += v_offsets(cfg)[c][None, :, None]
    if cfg.recency_rows > 0:
        k[w - cfg.recency_rows:] *= np.float32(cfg.recency_gain)
    if c in rel:
        k += np.float32(cfg.plant_gain) * u[None, :, :]
    if cfg.sink_gain != 1.0:
        k[0] *= np.float32(cfg.sink_gain)
    qb = np.concatenate([f32_to_bf16_bits(q), f32_to_bf16_bits(qq)], axis=0)
    kb = np.concatenate([f32_to_bf16_bits(k), f32_to_bf16_bits(kq)], axis=0)
    vb = np.concatenate([f32_to_bf16_bits(v), f32_to_bf16_bits(vq)], axis=0)
    return qb, kb, vb


def _prefill_shared(cfg: PrefillConfig):
    qq, kq, vq = query_rows_f32(cfg)
    u = mean_query_direction(cfg, qq)
    rel = set(int(x) for x in relevant_chunks(cfg))
    return qq, kq, vq, u, rel


def prefill_inputs(cfg: PrefillConfig, threads: int = 8):
    """bf16 bits of the whole batch: q [C,L,H_q,D], k,v [C,L,H_kv,D]."""
    C, L = cfg.n_chunks, cfg.seq_len
    q = np.empty((C, L, cfg.n_q_heads, cfg.head_dim), dtype=np.uint16)
    k = np.empty((C, L, cfg.n_kv_heads, cfg.head_dim), dtype=np.uint16)
    v = np.empty((C, L, cfg.n_kv_heads, cfg.head_dim), dtype=np.uint16)
    shared = _prefill_shared(cfg)

    def fill(c):
        q[c], k[c], v[c] = prefill_chunk(cfg, c, shared)

    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        list(ex.map(fill, range(C)))
    return q, k, v


def decode_inputs(cfg: DecodeConfig, threads: int = 8):
    """bf16 bits: q [B,n_q,H_q,D]; kc, vc [B,S,H_kv,k_t,D] (already rotated, compacted)."""
    B, S = cfg.batch, cfg.n_seg
    rq = _rng(cfg.cfg_id, _STREAM_DECODE_Q)
    q = f32_to_bf16_bits(_normal(rq, (B, cfg.n_q, cfg.n_q_heads, cfg.head_dim), cfg.entry_scale))
    kc = np.empty((B, S, cfg.n_kv_heads, cfg.keep_tokens, cfg.head_dim), dtype=np.uint16)
    vc = np.empty_like(kc)

    def fill(b):
        rng = _rng(cfg.cfg_id, b)
        shp = kc.shape[1:]
        kc[b] = f32_to_bf16_bits(_normal(rng, shp, cfg.entry_scale))
        vc[b] = f32_to_bf16_bits(_normal(rng, shp, cfg.entry_scale))

    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        list(ex.map(fill, range(B)))
    return q, kc, vc


def gather_inputs(cfg: DecodeConfig, threads: int = 8):
    """Gather workload of the decode config: source K,V [B,S,rows,H_kv,D] bf16 bits,
    chunk_idx [S] (identity) and tok_idx [B,S,H_kv,k_t]: sorted random k_t-subsets of the rows."""
    B, S, R = cfg.batch, cfg.n_seg, cfg.src_rows
    ks = np.empty((B, S, R, cfg.n_kv_heads, cfg.head_dim), dtype=np.uint16)
    vs = np.empty_like(ks)
    idx = np.empty((B, S, cfg.n_kv_heads, cfg.keep_tokens), dtype=np.int32)

    def fill(b):
        rng = _rng(cfg.cfg_id, 10_000 + b)
        shp = ks.shape[1:]
        ks[b] = f32_to_bf16_bits(_normal(rng, shp, cfg.entry_scale))
        vs[b] = f32_to_bf16_bits(_normal(rng, shp, cfg.entry_scale))
        for s in range(S):
            for g in range(cfg.n_kv_heads):
                idx[b, s, g] = np.sort(rng.choice(R, size=cfg.keep_tokens, replace=False))

    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        list(ex.map(fill, range(B)))
    chunk_idx = np.arange(S, dtype=np.int32)
    return ks, vs, chunk_idx, idx


def lm_logits_inputs(n_chunks: int, n_tokens: int, vocab: int, relevant=(), boost: float = 1.5,
                     cfg_id: int = 31):
    """Synthetic language-model logits for the query tokens after every chunk (stand-in for an LM
    head's output: no trained weights here).  logits [C, n_tokens, vocab] as bf16 bit patterns,
    N(0, 2^2) entries; targets [n_tokens] int32, the query's own token ids (the same for every
    chunk).  For the chunks listed in `relevant`, the target token's logit is raised by `boost`
    at every position: the query is more predictable after a relevant chunk."""
    rng = _rng(cfg_id, 0)
    targets = rng.integers(0, vocab, size=n_tokens).astype(np.int32)
    logits = np.empty((n_chunks, n_tokens, vocab), dtype=np.uint16)
    for c in range(n_chunks):
        x = _normal(_rng(cfg_id, 1 + c), (n_tokens, vocab), 2.0)
        if c in set(int(r) for r in relevant):
            x[np.arange(n_tokens), targets] += np.float32(boost)
        logits[c] = f32_to_bf16_bits(x)
    return logits, targets
