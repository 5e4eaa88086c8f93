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

    def chunk_prefill(self, q, k, v, with_scores=True):
        """Eq. 1-2 and 5-6 for all chunks: fills o, lse, k_rope, tok_score, chunk_score."""
        B.pc_chunk_prefill_attn(self.shape, q, k, v, self.o, self.lse, self.k_rope,
                                self.tok_score if with_scores else None,
                                self.chunk_score if with_scores else None, self.ws)

    def evict_and_attend(self, q, v):
        """Eq. 3-4 mechanics, Eq. 7 (after Eq. 8 when calibration is set) and Eq. 9-11 on the
        results of chunk_prefill."""
        C, L, w = self.C, self.L, self.w
        B.pc_select_chunks_topk(self.chunk_score, C, self.kc_n, self.chunk_idx, self.chunk_top)
        if self.calibration is None:
            B.pc_select_tokens_topk(self.tok_score, self.chunk_idx, self.kc_n, self.Hkv, w,
                                    self.kt_n, self.tok_idx)
            seg_len, per_head = None, 0
        else:
            lam, lo, hi = self.calibration
            B.pc_select_tokens_calibrated(self.tok_score, self.chunk_idx, self.kc_n, self.Hkv, w,
                                          self.kt_n, lam, lo, hi, self.tok_idx, self.tok_cnt)
            seg_len, per_head = self.tok_cnt, 1
        B.pc_gather_kv(self.k_rope, v, self.chunk_idx, self.tok_idx, 1, C, L, self.kc_n, self.Hkv,
                       self.kt_n, self.D, self.kc, self.vc)
        B.pc_parallel_attn(q[0, w:], self.kc, self.vc, seg_len, self.k_rope[0, w:], v[0, w:], 1,
                           self.wq, self.kc_n, self.kt_n, self.Hq, self.Hkv, self.D, w,
                           self.rope_base, self.scale, self.global_o, self.global_lse, self.ws,
                           seg_len_per_head=per_head)

    def forward(self, q, k, v):
        self.chunk_prefill(q, k, v, with_scores=True)
        if self.kc_n > 0:
            self.evict_and_attend(q, v)
        return self.global_o if self.kc_n > 0 else self.o
