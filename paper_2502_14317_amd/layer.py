"""Host orchestration of one ParallelComp layer over the C-ABI calls (section 3.1 of the paper):
chunk-batched local attention with fused query scores -> chunk selection -> per-head token
selection -> KV compaction -> global attention of the query over the surviving KV.
All arithmetic happens inside the library's kernels; this class only owns buffers."""
import torch

from . import binding as B


class ParallelCompLayer:
    def __init__(self, n_chunks, chunk_len, query_len, n_q_heads, n_kv_heads, head_dim,
                 obs_window, rope_base, keep_chunks, keep_tokens, softmax_scale=0.0,
                 device="cuda", calibration=None):
        self.C, self.w, self.wq = n_chunks, chunk_len, query_len
        self.L = chunk_len + query_len
        self.Hq, self.Hkv, self.D = n_q_heads, n_kv_heads, head_dim
        self.kc_n, self.kt_n = keep_chunks, keep_tokens
        self.rope_base, self.scale = rope_base, softmax_scale
        self.calibration = calibration          # None or (lambda, class_lo, class_hi) of Eq. 8
        self.chunk_lens = None                  # set by chunk_prefill for ragged chunks
        self.first_len = chunk_len
        self.shape = B.make_shape(n_chunks, chunk_len, query_len, n_q_heads, n_kv_heads, head_dim,
                                  obs_window, rope_base, softmax_scale)
        dev, bf, f32, i32 = device, torch.bfloat16, torch.float32, torch.int32
        C, L, Hq, Hkv, D = self.C, self.L, self.Hq, self.Hkv, self.D
        self.o = torch.empty((C, L, Hq, D), dtype=bf, device=dev)
        self.lse = torch.empty((C, Hq, L), dtype=f32, device=dev)
        self.k_rope = torch.empty((C, L, Hkv, D), dtype=bf, device=dev)
        self.tok_score = torch.empty((C, Hkv, chunk_len), dtype=f32, device=dev)
        self.chunk_score = torch.empty((C,), dtype=f32, device=dev)
        ws = B.pc_chunk_prefill_workspace_bytes(self.shape)
        if keep_chunks > 0:
            self.chunk_idx = torch.empty((keep_chunks,), dtype=i32, device=dev)
            self.chunk_top = torch.empty((keep_chunks,), dtype=f32, device=dev)
            self.tok_idx = torch.empty((keep_chunks, Hkv, keep_tokens), dtype=i32, device=dev)
            self.tok_cnt = torch.empty((keep_chunks, Hkv), dtype=i32, device=dev)
            self.kc = torch.empty((1, keep_chunks, Hkv, keep_tokens, D), dtype=bf, device=dev)
            self.vc = torch.empty_like(self.kc)
            self.global_o = torch.empty((1, query_len, Hq, D), dtype=bf, device=dev)
            self.global_lse = torch.empty((1, Hq, query_len), dtype=f32, device=dev)
            ws = max(ws, B.pc_parallel_attn_workspace_bytes(1, query_len, keep_chunks, keep_tokens,
                                                            Hq, Hkv, D, True))
        self.ws = B.alloc_workspace(ws, dev)

    def chunk_prefill(self, q, k, v, with_scores=True, chunk_lens=None, first_len=None):
        """Eq. 1-2 and 5-6 for all chunks: fills o, lse, k_rope, tok_score, chunk_score.
        chunk_lens [C] int32 (device): ragged chunks, see pc_chunk_prefill_attn; first_len is
        chunk_lens[0] as a host integer (where chunk 0's query rows sit; default w)."""
        self.chunk_lens = chunk_lens
        self.first_len = self.w if first_len is None else int(first_len)
        B.pc_chunk_prefill_attn(self.shape, q, k, v, self.o, self.lse, self.k_rope,
                                self.tok_score if with_scores else None,
                                self.chunk_score if with_scores else None, self.ws,
                                chunk_lens=chunk_lens)

    def evict_and_attend(self, q, v):
        """Eq. 3-4 mechanics, Eq. 7 (after Eq. 8 when calibration is set) and Eq. 9-11 on the
        results of chunk_prefill."""
        C, L, w = self.C, self.L, self.w
        B.pc_select_chunks_topk(self.chunk_score, C, self.kc_n, self.chunk_idx, self.chunk_top)
        if self.calibration is None and self.chunk_lens is None:
            B.pc_select_tokens_topk(self.tok_score, self.chunk_idx, self.kc_n, self.Hkv, w,
                                    self.kt_n, self.tok_idx)
            seg_len, per_head = None, 0
        else:
            lam, lo, hi = self.calibration if self.calibration is not None else (float("inf"), 0, 0)
            B.pc_select_tokens_calibrated(self.tok_score, self.chunk_idx, self.kc_n, self.Hkv, w,
                                          self.kt_n, lam, lo, hi, self.tok_idx, self.tok_cnt,
                                          chunk_lens=self.chunk_lens)
            seg_len, per_head = self.tok_cnt, 1
        B.pc_gather_kv(self.k_rope, v, self.chunk_idx, self.tok_idx, 1, C, L, self.kc_n, self.Hkv,
                       self.kt_n, self.D, self.kc, self.vc)
        w0 = self.first_len
        B.pc_parallel_attn(q[0, w0:w0 + self.wq], self.kc, self.vc, seg_len,
                           self.k_rope[0, w0:w0 + self.wq], v[0, w0:w0 + self.wq], 1,
                           self.wq, self.kc_n, self.kt_n, self.Hq, self.Hkv, self.D, w0,
                           self.rope_base, self.scale, self.global_o, self.global_lse, self.ws,
                           seg_len_per_head=per_head)

    def forward(self, q, k, v, chunk_lens=None, first_len=None):
        self.chunk_prefill(q, k, v, with_scores=True, chunk_lens=chunk_lens, first_len=first_len)
        if self.kc_n > 0:
            self.evict_and_attend(q, v)
        return self.global_o if self.kc_n > 0 else self.o


class StreamingParallelComp:
    """The same layer with the chunks arriving in memory-sized batches (sec. 3.1: chunks are
    encoded a batch at a time and a fixed-size priority queue keeps the best ones).  After each
    batch the queue holds the top keep_chunks of all chunks seen so far (score descending, earlier
    chunk first on ties, i.e. the offline top-k of the prefix); only the compacted KV of the chunks
    in the queue stays resident, an evicted chunk's slot is reused.  The final queue equals the
    offline selection, whatever the batch size.  The queue and its slot table live on the device
    (pc_chunk_queue_update), and the token selection and the gather of a batch's entrants are one
    launch each, driven by the device-side slot table: no host round trip between batches.  Host
    code here only owns buffers; every computation is a library call."""

    def __init__(self, n_chunks, batch_chunks, chunk_len, query_len, n_q_heads, n_kv_heads,
                 head_dim, obs_window, rope_base, keep_chunks, keep_tokens, softmax_scale=0.0,
                 device="cuda"):
        self.C, self.bc = n_chunks, min(batch_chunks, n_chunks)
        self.w, self.wq, self.L = chunk_len, query_len, chunk_len + query_len
        self.Hq, self.Hkv, self.D = n_q_heads, n_kv_heads, head_dim
        self.obs, self.rope_base, self.scale = obs_window, rope_base, softmax_scale
        self.kc_n, self.kt_n = min(keep_chunks, n_chunks), keep_tokens
        bf, f32, i32 = torch.bfloat16, torch.float32, torch.int32
        bc, L, Hq, Hkv, D = self.bc, self.L, n_q_heads, n_kv_heads, head_dim
        self.o = torch.empty((bc, L, Hq, D), dtype=bf, device=device)
        self.lse = torch.empty((bc, Hq, L), dtype=f32, device=device)
        self.k_rope = torch.empty((bc, L, Hkv, D), dtype=bf, device=device)
        self.tok_score = torch.empty((bc, Hkv, chunk_len), dtype=f32, device=device)
        self.chunk_score = torch.empty((n_chunks,), dtype=f32, device=device)     # all chunks seen
        # the device-side queue: ids in rank order, their scores and KV slots; entrants per slot
        self.queue_id = torch.full((self.kc_n,), -1, dtype=i32, device=device)
        self.queue_score = torch.zeros((self.kc_n,), dtype=f32, device=device)
        self.queue_slot = torch.zeros((self.kc_n,), dtype=i32, device=device)
        self.slot_src = torch.full((self.kc_n,), -1, dtype=i32, device=device)
        self.tok_idx = torch.empty((self.kc_n, Hkv, keep_tokens), dtype=i32, device=device)   # by slot
        self.kc = torch.empty((1, self.kc_n, Hkv, keep_tokens, D), dtype=bf, device=device)   # by slot
        self.vc = torch.empty_like(self.kc)
        self.q_query = torch.empty((query_len, Hq, D), dtype=bf, device=device)
        self.k_self = torch.empty((query_len, Hkv, D), dtype=bf, device=device)
        self.v_self = torch.empty_like(self.k_self)
        self.global_o = torch.empty((1, query_len, Hq, D), dtype=bf, device=device)
        self.global_lse = torch.empty((1, Hq, query_len), dtype=f32, device=device)
        shape = B.make_shape(bc, chunk_len, query_len, Hq, Hkv, D, obs_window, rope_base, softmax_scale)
        ws = max(B.pc_chunk_prefill_workspace_bytes(shape),
                 B.pc_parallel_attn_workspace_bytes(1, query_len, self.kc_n, keep_tokens, Hq, Hkv, D, True))
        self.ws = B.alloc_workspace(ws, device)

    def forward(self, q, k, v, after_batch=None):
        """q [C, L, H_q, D], k, v [C, L, H_kv, D] (any device-resident source; only one batch is
        touched at a time).  Returns the global attention output of the query rows.
        after_batch(first chunk id, chunks in the batch): optional callback after each batch's
        launches (tests read the queue there; it is not part of the path)."""
        self.queue_id.fill_(-1)                                  # an empty queue (plain fill)
        for c0 in range(0, self.C, self.bc):
            c1 = min(c0 + self.bc, self.C)
            nb = c1 - c0
            shape = B.make_shape(nb, self.w, self.wq, self.Hq, self.Hkv, self.D, self.obs,
                                 self.rope_base, self.scale)
            B.pc_chunk_prefill_attn(shape, q[c0:c1], k[c0:c1], v[c0:c1], self.o[:nb], self.lse[:nb],
                                    self.k_rope[:nb], self.tok_score[:nb], self.chunk_score[c0:c1],
                                    self.ws)
            if c0 == 0:              # the query rows of chunk 0 are the self segment (plain copies)
                self.q_query.copy_(q[0, self.w:]); self.k_self.copy_(self.k_rope[0, self.w:])
                self.v_self.copy_(v[0, self.w:])
            # merge the batch into the queue; then select and gather its entrants, slot by slot
            B.pc_chunk_queue_update(self.chunk_score[c0:c1], nb, c0, self.kc_n, self.queue_id,
                                    self.queue_score, self.queue_slot, self.slot_src)
            B.pc_select_tokens_topk(self.tok_score, self.slot_src, self.kc_n, self.Hkv, self.w,
                                    self.kt_n, self.tok_idx)
            B.pc_gather_kv(self.k_rope, v[c0:c1], self.slot_src, self.tok_idx, 1, nb, self.L, self.kc_n,
                           self.Hkv, self.kt_n, self.D, self.kc, self.vc)
            if after_batch is not None:
                after_batch(c0, nb)
        # every slot is filled once keep_chunks chunks have been seen (keep_chunks <= C)
        B.pc_parallel_attn(self.q_query, self.kc, self.vc, None, self.k_self, self.v_self, 1, self.wq,
                           self.kc_n, self.kt_n, self.Hq, self.Hkv, self.D, self.w, self.rope_base,
                           self.scale, self.global_o, self.global_lse, self.ws)
        return self.global_o


class DecodeCache:
    """The decoding stage (sec. 3.1, Eq. 9-11 token by token): the compressed segments of B
    sequences plus one tail segment that starts as the query block's keys / values and grows by
    one row per generated token.  Segment lengths live on the device and are advanced by
    pc_kv_append, so a run of decode steps is a run of library calls with no host round trip.
    A step = pc_kv_append (rotate and store the new token's K, V) + pc_parallel_attn (the new
    token's query over [segments ; tail], itself included)."""

    def __init__(self, batch, n_seg, keep_tokens, n_q_heads, n_kv_heads, head_dim, rope_base,
                 softmax_scale=0.0, device="cuda"):
        self.B, self.S, self.kt = batch, n_seg + 1, keep_tokens          # last segment = tail
        self.Hq, self.Hkv, self.D = n_q_heads, n_kv_heads, head_dim
        self.rope_base, self.scale = rope_base, softmax_scale
        bf, i32 = torch.bfloat16, torch.int32
        self.kc = torch.zeros((batch, self.S, n_kv_heads, keep_tokens, head_dim), dtype=bf, device=device)
        self.vc = torch.zeros_like(self.kc)
        self.seg_len = torch.zeros((batch, self.S), dtype=i32, device=device)
        self.out = torch.empty((batch, 1, n_q_heads, head_dim), dtype=bf, device=device)
        self.lse = torch.empty((batch, n_q_heads, 1), dtype=torch.float32, device=device)
        self.ws = B.alloc_workspace(B.pc_parallel_attn_workspace_bytes(
            batch, 1, self.S, keep_tokens, n_q_heads, n_kv_heads, head_dim, False), device)

    def load(self, kc, vc, seg_len, k_tail, v_tail):
        """kc, vc [B, n_seg, H_kv, k_t, D] compacted segments (plain copies into the cache),
        seg_len [B, n_seg] or None (all k_t), k_tail, v_tail [B, n0, H_kv, D] rotated keys /
        values of the query block (appended through the library as already-rotated rows)."""
        n = self.S - 1
        self.kc[:, :n].copy_(kc); self.vc[:, :n].copy_(vc)
        if seg_len is None:
            self.seg_len[:, :n].fill_(self.kt)
        else:
            self.seg_len[:, :n].copy_(seg_len)
        self.seg_len[:, n].zero_()
        B.pc_kv_append(k_tail, v_tail, self.B, k_tail.shape[1], self.S, n, self.kt, self.Hkv, self.D,
                       -1, self.rope_base, self.kc, self.vc, self.seg_len)

    def step(self, q_new, k_new, v_new, pos):
        """q_new [B, 1, H_q, D], k_new, v_new [B, 1, H_kv, D] before RoPE; pos = the token's
        position (continues behind the query block).  Returns out [B, 1, H_q, D]."""
        B.pc_kv_append(k_new, v_new, self.B, 1, self.S, self.S - 1, self.kt, self.Hkv, self.D, pos,
                       self.rope_base, self.kc, self.vc, self.seg_len)
        B.pc_parallel_attn(q_new, self.kc, self.vc, self.seg_len, None, None, self.B, 1, self.S,
                           self.kt, self.Hq, self.Hkv, self.D, pos, self.rope_base, self.scale,
                           self.out, self.lse, self.ws)
        return self.out


def fp8_rows(k_t):
    """Key rows the codes of a segment occupy: whole 32-key blocks."""
    return (k_t + 31) // 32 * 32


def fp8_alloc(batch, n_seg, n_kv_heads, k_t, head_dim, device="cuda"):
    """Zeroed buffer for the K or V codes of pc_kv_quantize_fp8 / pc_parallel_attn_fp8:
    [B, S, H_kv, ceil(k_t / 32) * 32 * D] bytes (32-key blocks laid out for the matrix cores)."""
    return torch.zeros((batch, n_seg, n_kv_heads, fp8_rows(k_t) * head_dim), dtype=torch.uint8, device=device)


class DecodeCacheFp8:
    """DecodeCache with the compressed segments stored in 8 bits (E4M3 codes + one scale per
    sequence, segment and KV head, written once by pc_kv_quantize_fp8 when the cache is loaded)
    and the growing tail kept in bf16 as a one-segment cache of its own.  A step =
    pc_kv_append on the tail + pc_parallel_attn_fp8 over [8-bit segments ; tail]."""

    def __init__(self, batch, n_seg, keep_tokens, tail_cap, n_q_heads, n_kv_heads, head_dim, rope_base,
                 softmax_scale=0.0, device="cuda"):
        self.B, self.S, self.kt, self.cap = batch, n_seg, keep_tokens, tail_cap
        self.Hq, self.Hkv, self.D = n_q_heads, n_kv_heads, head_dim
        self.rope_base, self.scale = rope_base, softmax_scale
        bf, i32, f32 = torch.bfloat16, torch.int32, torch.float32
        self.k8 = fp8_alloc(batch, n_seg, n_kv_heads, keep_tokens, head_dim, device)
        self.v8 = fp8_alloc(batch, n_seg, n_kv_heads, keep_tokens, head_dim, device)
        self.k_scale = torch.ones((batch, n_seg, n_kv_heads), dtype=f32, device=device)
        self.v_scale = torch.ones_like(self.k_scale)
        self.seg_len = torch.zeros((batch, n_seg), dtype=i32, device=device)
        self.k_tail = torch.zeros((batch, 1, n_kv_heads, tail_cap, head_dim), dtype=bf, device=device)
        self.v_tail = torch.zeros_like(self.k_tail)
        self.tail_len = torch.zeros((batch, 1), dtype=i32, device=device)
        self.out = torch.empty((batch, 1, n_q_heads, head_dim), dtype=bf, device=device)
        self.lse = torch.empty((batch, n_q_heads, 1), dtype=f32, device=device)
        self.ws = B.alloc_workspace(B.pc_parallel_attn_fp8_workspace_bytes(
            batch, 1, n_seg, keep_tokens, tail_cap, n_q_heads, n_kv_heads, head_dim), device)

    def load(self, kc, vc, seg_len, k_tail, v_tail):
        """kc, vc [B, n_seg, H_kv, k_t, D] bf16 compacted segments (quantised here), seg_len
        [B, n_seg] or None, k_tail, v_tail [B, n0, H_kv, D] rotated keys / values of the query block."""
        if seg_len is None:
            self.seg_len.fill_(self.kt)
        else:
            self.seg_len.copy_(seg_len)
        B.pc_kv_quantize_fp8(kc, vc, self.seg_len, self.B, self.S, self.kt, self.Hkv, self.D, self.k8,
                             self.v8, self.k_scale, self.v_scale)
        self.tail_len.zero_()
        B.pc_kv_append(k_tail, v_tail, self.B, k_tail.shape[1], 1, 0, self.cap, self.Hkv, self.D, -1,
                       self.rope_base, self.k_tail, self.v_tail, self.tail_len)

    def step(self, q_new, k_new, v_new, pos):
        B.pc_kv_append(k_new, v_new, self.B, 1, 1, 0, self.cap, self.Hkv, self.D, pos, self.rope_base,
                       self.k_tail, self.v_tail, self.tail_len)
        B.pc_parallel_attn_fp8(q_new, self.k8, self.v8, self.k_scale, self.v_scale, self.seg_len,
                               self.k_tail, self.v_tail, self.tail_len, self.cap, self.B, 1, self.S,
                               self.kt, self.Hq, self.Hkv, self.D, pos, self.rope_base, self.scale,
                               self.out, self.lse, self.ws)
        return self.out
