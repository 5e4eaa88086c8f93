"""Thin ctypes binding of libparallelcomp.so: argument marshalling only.

Every function has the name and argument order of its C entry point (include/parallelcomp.h)
and takes torch tensors that already live on the GPU; PyTorch is used for device memory and
the current stream, nothing else.  Every step of the path runs in the library's HIP kernels.
There is no fallback: if the library is missing, loading raises.
"""
import ctypes
import os
from ctypes import POINTER, Structure, c_char_p, c_float, c_int, c_int32, c_size_t, c_void_p

import torch

# PARALLELCOMP_LIB overrides the in-tree library (e.g. to time an experimental build)
_LIB_PATH = os.environ.get("PARALLELCOMP_LIB") or os.path.join(
    os.path.dirname(os.path.abspath(__file__)), "libparallelcomp.so")

PC_OK = 0
SYMBOLS = [
    "pc_chunk_prefill_attn", "pc_chunk_prefill_workspace_bytes", "pc_chunk_query_scores",
    "pc_chunk_query_scores_workspace_bytes", "pc_select_chunks_topk", "pc_select_tokens_topk",
    "pc_select_tokens_calibrated", "pc_gather_kv", "pc_parallel_attn", "pc_parallel_attn_workspace_bytes", "pc_status_string",
    "pc_last_hip_error", "pc_version", "pc_profile_begin", "pc_profile_end", "pc_profile_count",
    "pc_profile_get", "pc_kernel_name", "pc_mfma_ceiling", "pc_chunk_self_information", "pc_kv_append",
    "pc_kv_quantize_fp8", "pc_parallel_attn_fp8", "pc_parallel_attn_fp8_workspace_bytes",
    "pc_profile_begin_kernel", "pc_parallel_attn_static", "pc_parallel_attn_static_max_bytes",
    "pc_chunk_queue_update", "pc_gather_kv_amax", "pc_kv_quantize_fp8_amax",
    "pc_copy_ceiling",
]


class pc_shape(Structure):
    _fields_ = [("n_chunks", c_int32), ("chunk_len", c_int32), ("query_len", c_int32),
                ("n_q_heads", c_int32), ("n_kv_heads", c_int32), ("head_dim", c_int32),
                ("obs_window", c_int32), ("rope_base", c_float), ("softmax_scale", c_float)]


class PcError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = lib().pc_status_string(status).decode()
        if status == -4:
            msg += f" (hipError {lib().pc_last_hip_error()})"
        super().__init__(f"{where}: {msg}")


_lib = None


def lib():
    """Load the shared library (once).  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2502_14317_amd.build` "
            "(the HIP extension is required; there is no CPU fallback)")
    L = ctypes.CDLL(_LIB_PATH)
    P = c_void_p
    L.pc_chunk_prefill_attn.argtypes = [POINTER(pc_shape), P, P, P, P, P, P, P, P, P, P, c_size_t, P]
    L.pc_chunk_prefill_attn.restype = c_int
    L.pc_chunk_prefill_workspace_bytes.argtypes = [POINTER(pc_shape)]
    L.pc_chunk_prefill_workspace_bytes.restype = c_size_t
    L.pc_chunk_query_scores.argtypes = [POINTER(pc_shape), P, P, P, P, P, P, c_size_t, P]
    L.pc_chunk_query_scores.restype = c_int
    L.pc_chunk_query_scores_workspace_bytes.argtypes = [POINTER(pc_shape)]
    L.pc_chunk_query_scores_workspace_bytes.restype = c_size_t
    L.pc_select_chunks_topk.argtypes = [P, c_int32, c_int32, P, P, P]
    L.pc_select_chunks_topk.restype = c_int
    L.pc_chunk_queue_update.argtypes = [P, c_int32, c_int32, c_int32, P, P, P, P, P]
    L.pc_chunk_queue_update.restype = c_int
    L.pc_select_tokens_topk.argtypes = [P, P, c_int32, c_int32, c_int32, c_int32, P, P]
    L.pc_select_tokens_topk.restype = c_int
    L.pc_gather_kv.argtypes = [P, P, P, P] + [c_int32] * 7 + [P, P, P]
    L.pc_gather_kv.restype = c_int
    L.pc_gather_kv_amax.argtypes = [P, P, P, P] + [c_int32] * 7 + [P, P, P, P, P]
    L.pc_gather_kv_amax.restype = c_int
    L.pc_kv_quantize_fp8_amax.argtypes = [P, P, P, P, P] + [c_int32] * 6 + [P, P, P, P, P]
    L.pc_kv_quantize_fp8_amax.restype = c_int
    L.pc_parallel_attn.argtypes = [P] * 4 + [c_int32, P, P] + [c_int32] * 8 + [c_float, c_float, P, P, P, c_size_t, P]
    L.pc_select_tokens_calibrated.argtypes = [P, P] + [c_int32] * 4 + [c_float, c_int32, c_int32, P, P, P, P]
    L.pc_select_tokens_calibrated.restype = c_int
    L.pc_parallel_attn.restype = c_int
    L.pc_parallel_attn_static.argtypes = [P] * 4 + [c_int32, P, P] + [c_int32] * 8 + [c_float, c_float, P, P, P]
    L.pc_parallel_attn_static.restype = c_int
    L.pc_parallel_attn_static_max_bytes.argtypes = []
    L.pc_parallel_attn_static_max_bytes.restype = c_size_t
    L.pc_parallel_attn_workspace_bytes.argtypes = [c_int32] * 8
    L.pc_parallel_attn_workspace_bytes.restype = c_size_t
    L.pc_status_string.argtypes = [c_int]
    L.pc_status_string.restype = c_char_p
    L.pc_last_hip_error.argtypes = []
    L.pc_last_hip_error.restype = c_int
    L.pc_version.argtypes = []
    L.pc_version.restype = c_char_p
    L.pc_profile_get.argtypes = [c_int, POINTER(c_int), POINTER(c_float)]
    L.pc_kernel_name.argtypes = [c_int]
    L.pc_kernel_name.restype = c_char_p
    L.pc_mfma_ceiling.argtypes = [c_int, c_int, c_int, P, c_size_t, POINTER(ctypes.c_double), P]
    L.pc_mfma_ceiling.restype = c_int
    L.pc_copy_ceiling.argtypes = [c_int, P, P, c_size_t, P]
    L.pc_copy_ceiling.restype = c_int
    L.pc_chunk_self_information.argtypes = [P, P, c_int32, c_int32, c_int32, c_int32, P, P, P]
    L.pc_chunk_self_information.restype = c_int
    L.pc_kv_append.argtypes = [P, P] + [c_int32] * 8 + [c_float, P, P, P, c_int32, P]
    L.pc_kv_append.restype = c_int
    L.pc_kv_quantize_fp8.argtypes = [P, P, P] + [c_int32] * 6 + [P, P, P, P, P]
    L.pc_kv_quantize_fp8.restype = c_int
    L.pc_parallel_attn_fp8.argtypes = ([P] * 6 + [c_int32] + [P] * 3 + [c_int32] + [P] * 2 + [c_int32] * 8 +
                                       [c_float, c_float, P, P, P, c_size_t, P])
    L.pc_parallel_attn_fp8.restype = c_int
    L.pc_parallel_attn_fp8_workspace_bytes.argtypes = [c_int32] * 9
    L.pc_parallel_attn_fp8_workspace_bytes.restype = c_size_t
    _lib = L
    return L


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors must be contiguous GPU tensors")
    return c_void_p(t.data_ptr())


def _stream():
    return c_void_p(torch.cuda.current_stream().cuda_stream)


def _ws(ws):
    return (_ptr(ws), c_size_t(ws.numel() * ws.element_size())) if ws is not None else (None, c_size_t(0))


def _check(rc, where):
    if rc != PC_OK:
        raise PcError(rc, where)


def make_shape(n_chunks, chunk_len, query_len, n_q_heads, n_kv_heads, head_dim, obs_window,
               rope_base, softmax_scale=0.0):
    return pc_shape(n_chunks, chunk_len, query_len, n_q_heads, n_kv_heads, head_dim, obs_window,
                    rope_base, softmax_scale)


def alloc_workspace(n_bytes, device="cuda"):
    """Device scratch for a call (torch allocations are 256-byte aligned or better)."""
    return torch.empty(max(int(n_bytes), 256), dtype=torch.uint8, device=device)


def pc_chunk_prefill_workspace_bytes(shape):
    return lib().pc_chunk_prefill_workspace_bytes(ctypes.byref(shape))


def pc_chunk_query_scores_workspace_bytes(shape):
    return lib().pc_chunk_query_scores_workspace_bytes(ctypes.byref(shape))


def pc_parallel_attn_workspace_bytes(batch, n_q, n_seg, k_t, n_q_heads, n_kv_heads, head_dim, has_self):
    return lib().pc_parallel_attn_workspace_bytes(batch, n_q, n_seg, k_t, n_q_heads, n_kv_heads,
                                                  head_dim, int(has_self))


def pc_chunk_prefill_attn(shape, q, k, v, o, lse, k_rope, tok_score, chunk_score, ws,
                          chunk_lens=None):
    p, n = _ws(ws)
    _check(lib().pc_chunk_prefill_attn(ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(v),
                                       _ptr(chunk_lens), _ptr(o), _ptr(lse), _ptr(k_rope), _ptr(tok_score), _ptr(chunk_score),
                                       p, n, _stream()), "pc_chunk_prefill_attn")


def pc_chunk_query_scores(shape, q, k, tok_score, chunk_score, ws, chunk_lens=None):
    p, n = _ws(ws)
    _check(lib().pc_chunk_query_scores(ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(chunk_lens),
                                       _ptr(tok_score),
                                       _ptr(chunk_score), p, n, _stream()), "pc_chunk_query_scores")


def pc_chunk_self_information(logits, targets, n_chunks, n_tokens, vocab, negate, token_nll, info):
    _check(lib().pc_chunk_self_information(_ptr(logits), _ptr(targets), n_chunks, n_tokens, vocab,
                                           int(bool(negate)), _ptr(token_nll), _ptr(info),
                                           _stream()), "pc_chunk_self_information")


def pc_select_chunks_topk(chunk_score, n, k, out_idx, out_score=None):
    _check(lib().pc_select_chunks_topk(_ptr(chunk_score), n, k, _ptr(out_idx), _ptr(out_score),
                                       _stream()), "pc_select_chunks_topk")


def pc_chunk_queue_update(batch_score, n_batch, chunk_id0, capacity, queue_id, queue_score, queue_slot,
                          slot_src):
    _check(lib().pc_chunk_queue_update(_ptr(batch_score), n_batch, chunk_id0, capacity, _ptr(queue_id),
                                       _ptr(queue_score), _ptr(queue_slot), _ptr(slot_src), _stream()),
           "pc_chunk_queue_update")


def pc_select_tokens_topk(tok_score, chunk_idx, n_sel, n_kv_heads, chunk_len, k, out_idx):
    _check(lib().pc_select_tokens_topk(_ptr(tok_score), _ptr(chunk_idx), n_sel, n_kv_heads,
                                       chunk_len, k, _ptr(out_idx), _stream()),
           "pc_select_tokens_topk")


def pc_select_tokens_calibrated(tok_score, chunk_idx, n_sel, n_kv_heads, chunk_len, k, lam,
                                class_lo, class_hi, out_idx, out_cnt, chunk_lens=None):
    _check(lib().pc_select_tokens_calibrated(_ptr(tok_score), _ptr(chunk_idx), n_sel, n_kv_heads,
                                             chunk_len, k, lam, class_lo, class_hi,
                                             _ptr(chunk_lens), _ptr(out_idx), _ptr(out_cnt),
                                             _stream()),
           "pc_select_tokens_calibrated")


def pc_gather_kv(k_src, v_src, chunk_idx, tok_idx, batch, n_chunks, rows_per_chunk, n_sel,
                 n_kv_heads, k, head_dim, k_dst, v_dst):
    _check(lib().pc_gather_kv(_ptr(k_src), _ptr(v_src), _ptr(chunk_idx), _ptr(tok_idx), batch,
                              n_chunks, rows_per_chunk, n_sel, n_kv_heads, k, head_dim,
                              _ptr(k_dst), _ptr(v_dst), _stream()), "pc_gather_kv")


def pc_gather_kv_amax(k_src, v_src, chunk_idx, tok_idx, batch, n_chunks, rows_per_chunk, n_sel,
                      n_kv_heads, k, head_dim, k_dst, v_dst, k_amax, v_amax):
    _check(lib().pc_gather_kv_amax(_ptr(k_src), _ptr(v_src), _ptr(chunk_idx), _ptr(tok_idx), batch,
                                   n_chunks, rows_per_chunk, n_sel, n_kv_heads, k, head_dim,
                                   _ptr(k_dst), _ptr(v_dst), _ptr(k_amax), _ptr(v_amax), _stream()),
           "pc_gather_kv_amax")


def pc_kv_quantize_fp8_amax(kc, vc, k_amax, v_amax, seg_len, batch, n_seg, k_t, n_kv_heads, head_dim,
                            k8, v8, k_scale, v_scale, seg_len_per_head=0):
    _check(lib().pc_kv_quantize_fp8_amax(_ptr(kc), _ptr(vc), _ptr(k_amax), _ptr(v_amax), _ptr(seg_len),
                                         seg_len_per_head, batch, n_seg, k_t, n_kv_heads, head_dim,
                                         _ptr(k8), _ptr(v8), _ptr(k_scale), _ptr(v_scale), _stream()),
           "pc_kv_quantize_fp8_amax")


def pc_parallel_attn(q, kc, vc, seg_len, k_self, v_self, batch, n_q, n_seg, k_t, n_q_heads,
                     n_kv_heads, head_dim, q_pos0, rope_base, softmax_scale, out, lse_out, ws,
                     seg_len_per_head=0):
    p, n = _ws(ws)
    _check(lib().pc_parallel_attn(_ptr(q), _ptr(kc), _ptr(vc), _ptr(seg_len),
                                  int(seg_len_per_head), _ptr(k_self),
                                  _ptr(v_self), batch, n_q, n_seg, k_t, n_q_heads, n_kv_heads,
                                  head_dim, q_pos0, rope_base, softmax_scale, _ptr(out),
                                  _ptr(lse_out), p, n, _stream()), "pc_parallel_attn")


def pc_parallel_attn_static(q, kc, vc, seg_len, k_self, v_self, batch, n_q, n_seg, k_t, n_q_heads,
                            n_kv_heads, head_dim, q_pos0, rope_base, softmax_scale, out, lse_out,
                            seg_len_per_head=0):
    _check(lib().pc_parallel_attn_static(_ptr(q), _ptr(kc), _ptr(vc), _ptr(seg_len),
                                         int(seg_len_per_head), _ptr(k_self), _ptr(v_self), batch,
                                         n_q, n_seg, k_t, n_q_heads, n_kv_heads, head_dim, q_pos0,
                                         rope_base, softmax_scale, _ptr(out), _ptr(lse_out),
                                         _stream()), "pc_parallel_attn_static")


def pc_parallel_attn_static_max_bytes():
    return int(lib().pc_parallel_attn_static_max_bytes())


def pc_kv_append(k_new, v_new, batch, n_new, n_seg, seg, k_t, n_kv_heads, head_dim, pos0, rope_base,
                 kc, vc, seg_len, seg_len_per_head=0):
    _check(lib().pc_kv_append(_ptr(k_new), _ptr(v_new), batch, n_new, n_seg, seg, k_t, n_kv_heads,
                              head_dim, pos0, rope_base, _ptr(kc), _ptr(vc), _ptr(seg_len),
                              seg_len_per_head, _stream()), "pc_kv_append")


def pc_kv_quantize_fp8(kc, vc, seg_len, batch, n_seg, k_t, n_kv_heads, head_dim, k8, v8, k_scale,
                       v_scale, seg_len_per_head=0):
    _check(lib().pc_kv_quantize_fp8(_ptr(kc), _ptr(vc), _ptr(seg_len), seg_len_per_head, batch, n_seg,
                                    k_t, n_kv_heads, head_dim, _ptr(k8), _ptr(v8), _ptr(k_scale),
                                    _ptr(v_scale), _stream()), "pc_kv_quantize_fp8")


def pc_parallel_attn_fp8_workspace_bytes(batch, n_q, n_seg, k_t, tail_cap, n_q_heads, n_kv_heads, head_dim,
                                         has_self=False):
    return int(lib().pc_parallel_attn_fp8_workspace_bytes(batch, n_q, n_seg, k_t, tail_cap, n_q_heads,
                                                          n_kv_heads, head_dim, int(has_self)))


def pc_parallel_attn_fp8(q, k8, v8, k_scale, v_scale, seg_len, k_tail, v_tail, tail_len, tail_cap, batch,
                         n_q, n_seg, k_t, n_q_heads, n_kv_heads, head_dim, q_pos0, rope_base,
                         softmax_scale, out, lse_out, ws, seg_len_per_head=0, k_self=None, v_self=None):
    p, n = _ws(ws)
    _check(lib().pc_parallel_attn_fp8(_ptr(q), _ptr(k8), _ptr(v8), _ptr(k_scale), _ptr(v_scale),
                                      _ptr(seg_len), seg_len_per_head, _ptr(k_tail), _ptr(v_tail),
                                      _ptr(tail_len), tail_cap, _ptr(k_self), _ptr(v_self), batch, n_q,
                                      n_seg, k_t, n_q_heads,
                                      n_kv_heads, head_dim, q_pos0, rope_base, softmax_scale,
                                      _ptr(out), _ptr(lse_out), p, n, _stream()), "pc_parallel_attn_fp8")


def pc_profile_begin(kernel=None):
    """Start recording per-kernel durations; kernel = a kernel's name: only its launches."""
    if kernel is None:
        _check(lib().pc_profile_begin(), "pc_profile_begin")
        return
    L = lib()
    ids = [i for i in range(64) if L.pc_kernel_name(i).decode() == kernel]
    if not ids:
        raise ValueError(f"unknown kernel {kernel!r}")
    _check(L.pc_profile_begin_kernel(ids[0]), "pc_profile_begin_kernel")


def pc_profile_end():
    _check(lib().pc_profile_end(), "pc_profile_end")


def pc_mfma_ceiling(mode, n_cus, iters, scratch):
    """Enqueue the MFMA ceiling kernel (mode 0 constant operands, 1 random operands, 2 random
    operands with attention's LDS-read and softmax work); returns the MFMA flops of the launch
    (time it outside)."""
    flops = ctypes.c_double(0.0)
    _check(lib().pc_mfma_ceiling(int(mode), n_cus, iters, _ptr(scratch),
                                 scratch.numel() * scratch.element_size(), ctypes.byref(flops),
                                 _stream()), "pc_mfma_ceiling")
    return flops.value


def pc_copy_ceiling(mode, src, dst):
    """Enqueue the bare copy loop (mode 0 ordinary, 1 non-temporal) from src to dst (time it outside)."""
    _check(lib().pc_copy_ceiling(int(mode), _ptr(src), _ptr(dst), src.numel() * src.element_size(),
                                 _stream()), "pc_copy_ceiling")


def pc_profile_records():
    """[(kernel name, milliseconds)] of every kernel launched between begin and end."""
    L = lib()
    out = []
    kid, ms = c_int(0), c_float(0.0)
    for i in range(L.pc_profile_count()):
        _check(L.pc_profile_get(i, ctypes.byref(kid), ctypes.byref(ms)), "pc_profile_get")
        out.append((L.pc_kernel_name(kid.value).decode(), float(ms.value)))
    return out
