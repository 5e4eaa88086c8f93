"""CPU oracle for the ParallelComp chunked-prefill / parallel-attention path.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain fp64 statement of what the path
computes, written from the paper's method section (3.1).  Only the tests, the smoke check
and the benchmark's CPU-baseline leg may import it; the product path never does, and this
module imports nothing from the product package.  It shares no code with the HIP kernels.

Every function works on float64 numpy arrays (bf16 inputs are widened exactly by the caller)
and follows the paper's order of steps:

  rope                  position reuse: positions restart in every chunk (sec. 3.1, "Parallel
                        attention"; related work on reusing position encodings)
  local_attention       Eq. 1-2: A = Softmax(Q K^T / sqrt(d)), F = A V, inside one chunk
  query_scores          Eq. 5-6: cumulative query->key attention, summed over voting rows
  select_chunks         Eq. 3-4 mechanics: fixed number of best chunks (see readings below)
  chunk_queue_stream    sec. 3.1 "Chunk eviction": the fixed-size priority queue, chunks arriving
                        a batch at a time; an evicted chunk frees its KV slot for a later entrant
  chunk_self_information  Eq. 3: I_c = -log P(X^q | X^c) from given language-model logits
  select_tokens         Eq. 7: retained token set per head per chunk
  select_tokens_calibrated  Eq. 8 then Eq. 7: evict the tokens of one position class whose score
                        exceeds lambda (R_H), keep the best of the rest
  gather_kv             Eq. 7: compressed KV cache K_r = K_x[.], V_r = V_x[.]
  global_attention_*    Eq. 9-11: the query attends over [K^1 .. K^C, K^q]
  decode_steps          decoding stage: one new token per step attends over the compressed
                        segments, the query block and the tokens generated so far
  fp8_e4m3_*, quantize_kv_fp8, dequantize_kv_fp8
                        an 8-bit storage format for the compressed cache of the decoding stage
                        (not in the paper, which leaves the cache precision open): the
                        published OCP 8-bit float E4M3 encoding with one scale per (segment,
                        KV head); attention then runs on the dequantised values unchanged

Readings of the paper taken here (the paper is silent or ambiguous on each):
  * Eq. 1 carries a causal mask (decoder LLMs): key j is visible to row r iff j <= r.
  * The scale is 1/sqrt(head_dim) unless the caller passes another.
  * RoPE pairs dimension i with i + D/2 ("rotate-half"), theta_i = base^(-2i/D).
  * Each chunk sequence is [w context rows ; w_q query rows] under one causal mask.
  * A(i, j) in Eq. 5 is the post-softmax probability of row i of Eq. 1, normalised over the
    row's whole causal key set (chunk keys and the query's own keys).
  * Only the last obs_window query rows vote (the appendix's "last 8 tokens"; a parameter).
  * Scores cover chunk keys j < w only; query keys are always kept (Eq. 9 keeps K^q whole).
  * The kept set of Eq. 7 is the top-k by score; ties go to the lower index.
  * GQA: a KV head's score is the sum over the query heads that read it.
  * Chunk criterion: the query's attention mass on the chunk (sum of its token scores),
    larger is better.  This replaces Eq. 3's self-information inside the layer, which needs a
    language-model head and trained weights: selection against the paper's own criterion on
    real text is PARITY UNPINNED.  chunk_self_information computes Eq. 3 itself from given
    logits (synthetic ones here); select_chunks(-I, k) is then Eq. 4's "lowest I_c, fixed count"
    (Eq. 4 as printed compares the index c with a threshold: read as I_c <= epsilon).
  * In global attention keys keep their chunk-local rotation and query row t sits at w + t.
  * Attention calibration (Eq. 8): the text evicts R_H although the equation indexes the
    retained cache with it (as Eq. 7 does with R_L); R_H = tokens of ONE position class (a
    contiguous index range [lo, hi): the appendix's first 100 / last 100 / the rest) whose
    cumulative score is strictly above lambda; lambda is never given (a parameter).  Combined
    with compression, R_H is evicted first and the top-k of the remaining tokens is kept, so a
    head keeps min(k, w - |R_H|) tokens.  A NaN score is not above lambda.

  * 8-bit cache (extension, the paper has none): scale = amax / 448 per (segment, KV head)
    over the valid rows, in float32 (1 if amax = 0); code = E4M3(float32(x) / scale), round to
    nearest, ties to the even code, saturating at +-448; rows behind seg_len get code 0.  The
    division and the rounding decide an integer, so both are taken in float32 on both sides.
    PARITY UNPINNED against the paper (it has no such format); pinned to the format's definition.

Pins (tests/test_oracle_pins.py): brute-force softmax in pure Python loops; closed forms
(K = 0, V = 1, position 0, norm preservation, shift invariance); a library attention routine
for one chunk without eviction; one softmax over concatenated keys versus the logsumexp merge;
planted relevance with selections known by construction; gather as a pure permutation.
"""
import numpy as np


# --------------------------------------------------------------------------- RoPE
def rope_angles(positions, head_dim, base):
    """angle[p, i] = position_p * theta_i, theta_i = base^(-2 i / D), i in [0, D/2)."""
    i = np.arange(head_dim // 2, dtype=np.float64)
    theta = np.power(np.float64(base), -2.0 * i / np.float64(head_dim))
    return np.asarray(positions, dtype=np.float64)[:, None] * theta[None, :]


def rope(x, positions, base):
    """Rotate x [rows, heads, D] at the given integer positions (one per row).

    Pair (i, i + D/2) is rotated by angle position * theta_i.
    """
    x = np.asarray(x, dtype=np.float64)
    half = x.shape[-1] // 2
    ang = rope_angles(positions, x.shape[-1], base)[:, None, :]
    c, s = np.cos(ang), np.sin(ang)
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


# --------------------------------------------------------------------------- Eq. 1-2
def local_attention(q_rot, k_rot, v, scale=None, rows=None, return_probs=False):
    """Causal softmax attention inside one chunk sequence (Eq. 1-2).

    q_rot [L, H_q, D], k_rot [L, H_kv, D], v [L, H_kv, D] (q, k already rotated).
    Query head h reads KV head h // (H_q / H_kv).  rows: which rows to compute (default all).
    Returns o [n_rows, H_q, D], lse [n_rows, H_q] and, if asked, P [n_rows, H_q, L].
    """
    L, Hq, D = q_rot.shape
    Hkv = k_rot.shape[1]
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / np.sqrt(np.float64(D))
    rows = np.arange(L) if rows is None else np.asarray(rows, dtype=np.int64)
    n = rows.shape[0]
    o = np.zeros((n, Hq, D), dtype=np.float64)
    lse = np.zeros((n, Hq), dtype=np.float64)
    P_all = np.zeros((n, Hq, L), dtype=np.float64) if return_probs else None
    visible = np.arange(L)[None, :] <= rows[:, None]          # j <= r
    for h in range(Hq):
        g = h // G
        s = (q_rot[rows, h, :] @ k_rot[:, g, :].T) * scale       # [n, L]
        s = np.where(visible, s, -np.inf)
        m = s.max(axis=1, keepdims=True)
        e = np.exp(s - m)
        z = e.sum(axis=1, keepdims=True)
        P = e / z
        o[:, h, :] = P @ v[:, g, :]
        lse[:, h] = (m + np.log(z))[:, 0]
        if return_probs:
            P_all[:, h, :] = P
    return (o, lse, P_all) if return_probs else (o, lse)


# --------------------------------------------------------------------------- Eq. 5-6
def query_scores(q_rot, k_rot, chunk_len, obs_window, n_kv_heads, scale=None):
    """Cumulative attention of the voting query rows to every chunk key (Eq. 5-6).

    Voting rows R = the last obs_window rows of the sequence.  Returns
    tok_score [H_kv, w] = sum over the group's query heads and over R of P[r, j], j < w,
    and chunk_score = sum of tok_score (the query's attention mass on the chunk).
    """
    L, Hq, D = q_rot.shape
    G = Hq // n_kv_heads
    R = np.arange(L - obs_window, L)
    v_dummy = np.zeros((L, n_kv_heads, 1), dtype=np.float64)
    _, _, P = local_attention(q_rot, k_rot, v_dummy, scale=scale, rows=R, return_probs=True)
    col = P.sum(axis=0)                                          # [H_q, L]
    tok = col.reshape(n_kv_heads, G, L).sum(axis=1)[:, :chunk_len]
    return tok, tok.sum()


# --------------------------------------------------------------------------- Eq. 3
def chunk_self_information(logits, targets):
    """Self-information of the query tokens given each chunk (Eq. 3).

    logits [C, n_t, V]: row (c, t) holds the language model's logits for query token t after
    chunk c and the query tokens before t; targets [n_t]: the query's token ids.  By the chain
    rule  I_c = -log P(X^q | X^c) = sum_t ( log sum_v exp(logits[c, t, v]) - logits[c, t, targets[t]] ).
    Returns (I [C], nll [C, n_t]) in nats.  Lower I = more relevant chunk (Eq. 4 keeps those).
    """
    logits = np.asarray(logits, dtype=np.float64)
    targets = np.asarray(targets, dtype=np.int64)
    m = logits.max(axis=2)
    lse = m + np.log(np.exp(logits - m[..., None]).sum(axis=2))
    tgt = np.take_along_axis(logits, targets[None, :, None], axis=2)[..., 0]
    nll = lse - tgt
    return nll.sum(axis=1), nll


# --------------------------------------------------------------------------- selection
def _top_k_lower_index_wins(score, k):
    """Indices of the k largest scores under the total order (score desc, index asc)."""
    score = np.asarray(score, dtype=np.float64)
    order = np.lexsort((np.arange(score.shape[0]), -score))      # primary: -score, then index
    return order[:k]


def select_chunks(chunk_score, k_c):
    """Kept chunk ids in rank order (best first); ties go to the lower id (Eq. 3-4 mechanics)."""
    return _top_k_lower_index_wins(chunk_score, k_c).astype(np.int32)


def chunk_queue_stream(chunk_score, batch, capacity):
    """The fixed-size priority queue of sec. 3.1 ("Chunk eviction"), fed a batch of chunks at a
    time (the chunks are encoded in memory-sized batches; only the chunks in the queue keep their
    compressed KV).  After each batch the queue holds the `capacity` best chunks seen so far under
    the order (score descending, earlier chunk first; NaN below every number), and every chunk in
    the queue owns one of `capacity` KV slots: a chunk keeps its slot while it stays in the queue,
    a chunk that enters takes a free slot (entrants in rank order take the free slots in ascending
    order), an evicted chunk frees its slot.

    chunk_score [C]; returns a list with one entry per batch: (queue ids in rank order,
    slot of each queue entry, list of (chunk id, slot) of the batch's entrants).
    """
    score = np.asarray(chunk_score, dtype=np.float64)
    key = np.where(np.isnan(score), -np.inf, score)
    nan_last = np.isnan(score)                                  # NaN ranks below -inf too
    queue, slot_of, out = [], {}, []
    for c0 in range(0, score.shape[0], batch):
        cand = queue + list(range(c0, min(c0 + batch, score.shape[0])))
        cand.sort(key=lambda c: (bool(nan_last[c]), -key[c], c))
        new_queue = cand[:capacity]
        for c in queue:
            if c not in new_queue:
                del slot_of[c]
        free = [s for s in range(capacity) if s not in slot_of.values()]
        entrants = []
        for c in new_queue:                                     # rank order
            if c not in slot_of:
                slot_of[c] = free.pop(0)
                entrants.append((c, slot_of[c]))
        queue = new_queue
        out.append((list(queue), [slot_of[c] for c in queue], entrants))
    return out


def select_tokens(tok_score, k_t):
    """Kept token ids per row of tok_score [..., w], ascending; ties go to the lower id (Eq. 7)."""
    tok_score = np.asarray(tok_score, dtype=np.float64)
    flat = tok_score.reshape(-1, tok_score.shape[-1])
    out = np.empty((flat.shape[0], k_t), dtype=np.int32)
    for i in range(flat.shape[0]):
        out[i] = np.sort(_top_k_lower_index_wins(flat[i], k_t))
    return out.reshape(tok_score.shape[:-1] + (k_t,))


def select_tokens_calibrated(tok_score, k_t, lam, class_lo, class_hi, valid_len=None):
    """Eq. 8 followed by Eq. 7 per row of tok_score [..., w].

    R_H = {j in [class_lo, class_hi) : score_j > lam} is evicted; of the remaining tokens the
    k_t best are kept (ties to the lower id), ascending.  valid_len [...] (optional): only
    tokens j < valid_len exist (a chunk shorter than w).  Returns (idx [..., k_t] int32 padded
    with -1, cnt [...] int32 = number kept = min(k_t, valid_len - |R_H|)).
    """
    tok_score = np.asarray(tok_score, dtype=np.float64)
    w = tok_score.shape[-1]
    flat = tok_score.reshape(-1, w)
    vlen = np.full(flat.shape[0], w) if valid_len is None else np.asarray(valid_len).reshape(-1)
    idx = np.full((flat.shape[0], k_t), -1, dtype=np.int32)
    cnt = np.zeros(flat.shape[0], dtype=np.int32)
    for i in range(flat.shape[0]):
        evicted = np.zeros(w, dtype=bool)
        evicted[vlen[i]:] = True
        for j in range(max(class_lo, 0), min(class_hi, w)):
            if flat[i, j] > lam:
                evicted[j] = True
        rest = np.nonzero(~evicted)[0]
        keep = rest[_top_k_lower_index_wins(flat[i, rest], min(k_t, rest.shape[0]))]
        cnt[i] = keep.shape[0]
        idx[i, :cnt[i]] = np.sort(keep)
    return idx.reshape(tok_score.shape[:-1] + (k_t,)), cnt.reshape(tok_score.shape[:-1])


# --------------------------------------------------------------------------- Eq. 7
def gather_kv(k_src, v_src, chunk_idx, tok_idx):
    """Compressed cache: dst[s, g, t, :] = src[chunk_idx[s], tok_idx[s, g, t], g, :].

    k_src, v_src [C, rows, H_kv, D] (any dtype: this is a pure copy);
    chunk_idx [n_sel]; tok_idx [n_sel, H_kv, k_t], a negative id gives a zero row.
    Returns [n_sel, H_kv, k_t, D] each.
    """
    n_sel, Hkv, kt = tok_idx.shape
    kd = np.zeros((n_sel, Hkv, kt) + k_src.shape[3:], dtype=k_src.dtype)
    vd = np.zeros_like(kd)
    for s in range(n_sel):
        for g in range(Hkv):
            ok = tok_idx[s, g] >= 0
            kd[s, g, ok] = k_src[chunk_idx[s], tok_idx[s, g, ok], g]
            vd[s, g, ok] = v_src[chunk_idx[s], tok_idx[s, g, ok], g]
    return kd, vd


# --------------------------------------------------------------------------- Eq. 9-11
def _masked_softmax_rows(s, visible=None):
    """Row softmax of a logit matrix; returns (P, lse).  visible: boolean mask or None."""
    if visible is not None:
        s = np.where(visible, s, -np.inf)
    m = s.max(axis=1, keepdims=True)
    e = np.exp(s - m)
    z = e.sum(axis=1, keepdims=True)
    return e / z, (m + np.log(z))[:, 0]


def global_attention_concat(q_rot, kc, vc, k_self=None, v_self=None, seg_len=None, scale=None):
    """Eq. 9-11 as printed: one softmax over the concatenation [K^1 .. K^S, K^q].

    q_rot [n_q, H_q, D] rotated query rows; kc, vc [S, H_kv, k_t, D] compressed segments
    (keys rotated); optional causal self segment k_self, v_self [n_q, H_kv, D]: query row t
    sees self keys 0..t.  seg_len [S] or [S, H_kv]: valid rows per segment (and KV head);
    default all k_t.  Returns o [n_q, H_q, D], lse [n_q, H_q].
    """
    nq, Hq, D = q_rot.shape
    S, Hkv, kt, _ = kc.shape
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / np.sqrt(np.float64(D))
    seg_len = _seg_len_per_head(seg_len, S, Hkv, kt)
    o = np.zeros((nq, Hq, D))
    lse = np.zeros((nq, Hq))
    for h in range(Hq):
        g = h // G
        K = [kc[s, g, :seg_len[s, g]] for s in range(S)]
        V = [vc[s, g, :seg_len[s, g]] for s in range(S)]
        visible = np.ones((nq, int(seg_len[:, g].sum())), dtype=bool)
        if k_self is not None:
            K.append(k_self[:, g])
            V.append(v_self[:, g])
            causal = np.arange(nq)[None, :] <= np.arange(nq)[:, None]
            visible = np.concatenate([visible, causal], axis=1)
        K = np.concatenate(K, axis=0)
        V = np.concatenate(V, axis=0)
        P, lse[:, h] = _masked_softmax_rows((q_rot[:, h] @ K.T) * scale, visible)
        o[:, h] = P @ V
    return o, lse


def _seg_len_per_head(seg_len, S, Hkv, kt):
    """seg_len None / [S] / [S, H_kv] -> int64 [S, H_kv]."""
    if seg_len is None:
        return np.full((S, Hkv), kt, dtype=np.int64)
    seg_len = np.asarray(seg_len, dtype=np.int64)
    return np.repeat(seg_len[:, None], Hkv, axis=1) if seg_len.ndim == 1 else seg_len


def lse_merge(o_parts, lse_parts):
    """Exact merge of per-segment softmax partials (leading axis = segment):
    LSE = log sum_s exp(lse_s), o = sum_s exp(lse_s - LSE) o_s.  A segment with no visible key
    carries lse = -inf and weight 0."""
    lse_parts = np.asarray(lse_parts, dtype=np.float64)
    m = lse_parts.max(axis=0)
    wgt = np.exp(lse_parts - m)
    z = wgt.sum(axis=0)
    o = (wgt[..., None] * np.asarray(o_parts)).sum(axis=0) / z[..., None]
    return o, m + np.log(z)


def global_attention_merged(q_rot, kc, vc, k_self=None, v_self=None, seg_len=None, scale=None):
    """Same quantity as global_attention_concat, computed the "parallel" way: an independent
    softmax per segment (and a causal one over the self segment), merged by lse_merge."""
    nq, Hq, D = q_rot.shape
    S, Hkv, kt, _ = kc.shape
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / np.sqrt(np.float64(D))
    seg_len = _seg_len_per_head(seg_len, S, Hkv, kt)
    n_parts = S + (1 if k_self is not None else 0)
    o_p = np.zeros((n_parts, nq, Hq, D))
    l_p = np.full((n_parts, nq, Hq), -np.inf)
    causal = np.arange(nq)[None, :] <= np.arange(nq)[:, None]
    for h in range(Hq):
        g = h // G
        for s in range(S):
            if seg_len[s, g] > 0:
                Ks, Vs = kc[s, g, :seg_len[s, g]], vc[s, g, :seg_len[s, g]]
                P, l_p[s, :, h] = _masked_softmax_rows((q_rot[:, h] @ Ks.T) * scale)
                o_p[s, :, h] = P @ Vs
        if k_self is not None:
            P, l_p[S, :, h] = _masked_softmax_rows((q_rot[:, h] @ k_self[:, g].T) * scale, causal)
            o_p[S, :, h] = P @ v_self[:, g]
    return lse_merge(o_p, l_p)


# --------------------------------------------------------------------------- decoding stage
def decode_steps(q_new, k_new, v_new, kc, vc, k_tail, v_tail, pos0, rope_base, seg_len=None,
                 scale=None, store=None):
    """Token-by-token generation after the prefill (sec. 3.1, decoding stage of Eq. 9-11).

    Step t: the new token's q and k [H, D] are rotated at position pos0 + t (positions continue
    behind the query block), its k and v are appended to the tail (k_tail, v_tail [n0, H_kv, D]:
    the query block's rotated keys / values), and the token attends, in one softmax, over the
    compressed segments kc, vc [S, H_kv, k_t, D] (seg_len rows each) and the whole tail, itself
    included.  q_new [T, H_q, D], k_new, v_new [T, H_kv, D] before RoPE.  Returns o [T, H_q, D],
    lse [T, H_q] and the final tail (k, v).
    store: the cache's storage format, a function applied once to the rotated key row before it
    enters the tail (the paper does not state a precision; a 16-bit cache rounds the rotated key
    there, as the prefill's cache does).  Default: the row is kept in float64."""
    T = q_new.shape[0]
    Hkv = k_new.shape[1]
    kt = kc.shape[2]
    o = np.zeros_like(np.asarray(q_new, dtype=np.float64))
    lse = np.zeros(o.shape[:2])
    k_tail, v_tail = np.array(k_tail, dtype=np.float64), np.array(v_tail, dtype=np.float64)
    for t in range(T):
        q_rot = rope(q_new[t:t + 1], [pos0 + t], rope_base)
        k_rot = rope(k_new[t:t + 1], [pos0 + t], rope_base)
        if store is not None:
            k_rot = np.asarray(store(k_rot), dtype=np.float64)
        k_tail = np.concatenate([k_tail, k_rot], axis=0)
        v_tail = np.concatenate([v_tail, np.asarray(v_new[t:t + 1], dtype=np.float64)], axis=0)
        n = k_tail.shape[0]
        pad = max(kt, n)
        kc_t = np.zeros((kc.shape[0] + 1, Hkv, pad, kc.shape[3])); vc_t = np.zeros_like(kc_t)
        kc_t[:-1, :, :kt] = kc; vc_t[:-1, :, :kt] = vc
        kc_t[-1, :, :n] = k_tail.transpose(1, 0, 2); vc_t[-1, :, :n] = v_tail.transpose(1, 0, 2)
        sl = np.full(kc.shape[0], kt) if seg_len is None else np.asarray(seg_len)
        o[t:t + 1], lse[t:t + 1] = global_attention_concat(q_rot, kc_t, vc_t, seg_len=np.append(sl, n),
                                                          scale=scale)
    return o, lse, (k_tail, v_tail)


# --------------------------------------------------------------------------- 8-bit cache
def fp8_e4m3_decode(codes):
    """OCP 8-bit float E4M3 (finite-only variant): 1 sign, 4 exponent (bias 7), 3 mantissa bits.
    Exponent field 0 is subnormal (m / 8 * 2^-6); exponent 15 with mantissa 7 is NaN; there are
    no infinities, the largest magnitude is 1.75 * 2^8 = 448.  uint8 -> float64."""
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    sign = np.where(c & 0x80, -1.0, 1.0)
    e = (c >> 3) & 0xF
    m = (c & 0x7).astype(np.float64)
    val = np.where(e == 0, m / 8.0 * 2.0 ** -6, (1.0 + m / 8.0) * 2.0 ** (e.astype(np.float64) - 7.0))
    val = np.where((e == 15) & ((c & 0x7) == 7), np.nan, val)
    return sign * val


def fp8_e4m3_encode(x):
    """Nearest E4M3 code of every finite float32 x: the representable value closest to x, the
    one with the even code on a tie, +-448 beyond the range (saturating); the sign of x is
    kept (-0.0 -> 0x80).  Written as the definition: a search over all 127 finite magnitudes."""
    x = np.asarray(x, dtype=np.float32)
    mags = fp8_e4m3_decode(np.arange(0x7F, dtype=np.uint8))            # codes 0x00..0x7E ascending
    a = np.abs(x.astype(np.float64))
    hi = np.searchsorted(mags, a, side="left").clip(1, 0x7E)            # first magnitude >= |x|
    lo = hi - 1
    d_lo, d_hi = a - mags[lo], mags[hi] - a
    code = np.where(d_lo < d_hi, lo, np.where(d_hi < d_lo, hi, np.where(lo % 2 == 0, lo, hi)))
    code = np.where(a >= mags[0x7E], 0x7E, code)
    return (code | np.where(np.signbit(x), 0x80, 0)).astype(np.uint8)


def quantize_kv_fp8(kc, vc, seg_len=None):
    """kc, vc [S, H_kv, k_t, D] (values exactly representable in float32) -> codes uint8 of the
    same shape and scales float32 [S, H_kv] for each: scale = max |x| over the segment's valid
    rows / 448 (1 where that maximum is 0), code = E4M3(float32(x) / scale) in float32
    arithmetic; rows behind seg_len ([S] or [S, H_kv]) get code 0."""
    S, Hkv, kt, D = kc.shape
    seg_len = _seg_len_per_head(seg_len, S, Hkv, kt)
    out = []
    for x in (kc, vc):
        x32 = np.asarray(x, dtype=np.float32)
        codes = np.zeros(x32.shape, dtype=np.uint8)
        scale = np.ones((S, Hkv), dtype=np.float32)
        for s_ in range(S):
            for g in range(Hkv):
                n = int(seg_len[s_, g])
                if n == 0:
                    continue
                amax = np.abs(x32[s_, g, :n]).max()
                if amax > 0:
                    scale[s_, g] = amax / np.float32(448.0)
                codes[s_, g, :n] = fp8_e4m3_encode(x32[s_, g, :n] / scale[s_, g])
        out += [codes, scale]
    return tuple(out)            # k_codes, k_scale, v_codes, v_scale


def dequantize_kv_fp8(codes, scale):
    """codes uint8 [S, H_kv, k_t, D], scale [S, H_kv] -> float64 values code * scale (exact)."""
    return fp8_e4m3_decode(codes) * np.asarray(scale, dtype=np.float64)[:, :, None, None]


# --------------------------------------------------------------------------- the whole layer
def parallelcomp_layer(q, k, v, chunk_len, obs_window, keep_chunks, keep_tokens, rope_base,
                       scale=None, attn_rows=None, calibration=None, chunk_lens=None):
    """One layer of the method on C chunk sequences, in the paper's order of steps.

    q [C, L, H_q, D], k, v [C, L, H_kv, D] in float64, before RoPE; every chunk's last
    L - chunk_len rows are the query rows.  attn_rows: rows of every chunk for which the local
    attention output is computed (default all).  calibration = (lambda, class_lo, class_hi)
    switches the token selection to Eq. 8 + Eq. 7 (select_tokens_calibrated).  Returns a dict
    with every intermediate result.
    chunk_lens [C] (optional): chunk c has only chunk_lens[c] <= chunk_len context rows ("at
    most w tokens" per chunk, sec. 3.1) and its sequence is rows [0, chunk_lens[c] + w_q) of
    q[c], k[c], v[c]: the query rows follow the context directly, at positions chunk_lens[c] + t.
    Rows behind a short sequence are padding: outputs and rotated keys there stay zero, the
    token scores of the missing tokens are zero and they are never selected (a head of a short
    chunk may keep fewer than keep_tokens tokens; per-head counts are returned as tok_cnt).
    """
    C, L, Hq, D = q.shape
    Hkv = k.shape[2]
    w = chunk_len
    wq = L - w
    lens = np.full(C, w, dtype=np.int64) if chunk_lens is None else np.asarray(chunk_lens, dtype=np.int64)
    rows = np.arange(L) if attn_rows is None else np.asarray(attn_rows)
    out = {"o": np.zeros((C, rows.shape[0], Hq, D)), "lse": np.zeros((C, rows.shape[0], Hq)),
           "k_rope": np.zeros_like(k), "tok_score": np.zeros((C, Hkv, w)),
           "chunk_score": np.zeros(C), "attn_rows": rows}
    q_rot_query = None
    for c in range(C):
        Lc = int(lens[c]) + wq
        pos = np.arange(Lc)
        q_rot = rope(q[c, :Lc], pos, rope_base)
        k_rot = rope(k[c, :Lc], pos, rope_base)
        out["k_rope"][c, :Lc] = k_rot
        sel = np.nonzero(rows < Lc)[0]
        out["o"][c, sel], out["lse"][c, sel] = local_attention(q_rot, k_rot, v[c, :Lc], scale, rows[sel])
        tok, out["chunk_score"][c] = query_scores(q_rot, k_rot, int(lens[c]), obs_window, Hkv, scale)
        out["tok_score"][c, :, :lens[c]] = tok
        if c == 0:
            q_rot_query = q_rot[lens[0]:]
    if keep_chunks <= 0:
        return out
    chunk_idx = select_chunks(out["chunk_score"], keep_chunks)
    if calibration is None and chunk_lens is None:
        tok_idx, tok_cnt = select_tokens(out["tok_score"][chunk_idx], keep_tokens), None
    else:
        lam, lo, hi = (np.inf, 0, 0) if calibration is None else calibration
        vlen = np.repeat(lens[chunk_idx][:, None], Hkv, axis=1)
        tok_idx, tok_cnt = select_tokens_calibrated(out["tok_score"][chunk_idx], keep_tokens,
                                                    lam, lo, hi, valid_len=vlen)
    kc, vc = gather_kv(out["k_rope"], v, chunk_idx, tok_idx)
    k_self, v_self = out["k_rope"][0, lens[0]:lens[0] + wq], v[0, lens[0]:lens[0] + wq]
    og, lg = global_attention_merged(q_rot_query, kc, vc, k_self, v_self, seg_len=tok_cnt,
                                     scale=scale)
    out.update({"chunk_idx": chunk_idx, "tok_idx": tok_idx, "tok_cnt": tok_cnt, "kc": kc, "vc": vc,
                "global_o": og, "global_lse": lg, "q_rot_query": q_rot_query})
    return out
