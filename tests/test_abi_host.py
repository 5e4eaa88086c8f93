"""Host-side checks that need no GPU: the C-ABI library loads, exports every symbol the header
declares, and rejects bad arguments before touching the GPU."""
import ctypes
import os
import re

import pytest

import paper_2502_14317_amd as pc
from paper_2502_14317_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    inc = os.path.join(ROOT, "include")
    text = "".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pc_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = pc.lib()
    names = _declared_symbols()
    assert len(names) >= 12
    for name in names:
        assert hasattr(L, name), name
    assert set(names) == set(binding.SYMBOLS)
    assert L.pc_version().startswith(b"parallelcomp")


def test_status_strings():
    L = pc.lib()
    for code in range(-5, 1):
        assert L.pc_status_string(code)
    assert b"unknown" in L.pc_status_string(-99)


def test_null_and_shape_errors_before_any_gpu_work():
    L = pc.lib()
    one = ctypes.c_void_p(256)            # never dereferenced: validation fails first
    # select chunks
    assert L.pc_select_chunks_topk(None, 4, 2, one, None, None) == -1
    assert L.pc_select_chunks_topk(one, 4, 5, one, None, None) == -2
    assert L.pc_select_chunks_topk(one, 0, 0, one, None, None) == -2
    assert L.pc_select_chunks_topk(one, 5000, 1, one, None, None) == -2
    # ceiling kernel (measurement aid): mode, sizes and scratch are checked before the launch
    fl = ctypes.c_double(0.0)
    assert L.pc_mfma_ceiling(0, 256, 10, None, 1 << 20, ctypes.byref(fl), None) == -1
    assert L.pc_mfma_ceiling(3, 256, 10, one, 1 << 20, ctypes.byref(fl), None) == -2
    assert L.pc_mfma_ceiling(2, 0, 10, one, 1 << 20, ctypes.byref(fl), None) == -2
    assert L.pc_mfma_ceiling(2, 256, 10, one, 1024, ctypes.byref(fl), None) == -3
    # gather with maxima, one-read quantisation
    assert L.pc_gather_kv_amax(one, one, None, one, 1, 2, 8, 1, 1, 4, 128, one, one, None, one, None) == -1
    assert L.pc_gather_kv_amax(one, one, None, one, 1, 2, 8, 1, 1, 4, 96, one, one, one, one, None) == -2
    assert L.pc_kv_quantize_fp8_amax(one, one, None, one, None, 0, 1, 1, 4, 1, 128, one, one, one, one, None) == -1
    assert L.pc_kv_quantize_fp8_amax(one, one, one, one, None, 2, 1, 1, 4, 1, 128, one, one, one, one, None) == -2
    # streaming chunk queue
    assert L.pc_chunk_queue_update(None, 4, 0, 2, one, one, one, one, None) == -1
    assert L.pc_chunk_queue_update(one, 4, 0, 2, one, one, one, None, None) == -1
    assert L.pc_chunk_queue_update(one, 0, 0, 2, one, one, one, one, None) == -2
    assert L.pc_chunk_queue_update(one, 4, 0, 2000, one, one, one, one, None) == -2
    assert L.pc_chunk_queue_update(one, 4, -1, 2, one, one, one, one, None) == -2
    # select tokens
    assert L.pc_select_tokens_topk(None, None, 1, 1, 8, 2, one, None) == -1
    assert L.pc_select_tokens_topk(one, None, 1, 1, 8, 9, one, None) == -2
    assert L.pc_select_tokens_topk(one, None, 1, 1, 40000, 2, one, None) == -2
    # calibrated token selection (Eq. 8): class bounds and lambda are checked on the host
    assert L.pc_select_tokens_calibrated(one, None, 1, 1, 8, 2, 0.5, 0, 4, None, one, None, None) == -1
    assert L.pc_select_tokens_calibrated(one, None, 1, 1, 8, 2, 0.5, 5, 4, None, one, one, None) == -2
    assert L.pc_select_tokens_calibrated(one, None, 1, 1, 8, 2, 0.5, 0, 9, None, one, one, None) == -2
    assert L.pc_select_tokens_calibrated(one, None, 1, 1, 8, 2, float('nan'), 0, 4, None, one, one, None) == -2
    assert L.pc_select_tokens_calibrated(one, None, 0, 1, 8, 2, 0.5, 0, 4, None, one, one, None) == 0
    # gather
    assert L.pc_gather_kv(one, one, None, None, 1, 1, 8, 1, 1, 2, 128, one, one, None) == -1
    assert L.pc_gather_kv(one, one, None, one, 1, 1, 8, 1, 1, 2, 96, one, one, None) == -2
    # prefill
    good = pc.make_shape(2, 64, 16, 8, 2, 128, 8, 1e4)
    assert L.pc_chunk_prefill_attn(None, one, one, one, None, one, one, None, None, None, one, 1 << 30, None) == -1
    assert L.pc_chunk_prefill_attn(ctypes.byref(good), None, one, one, None, one, one, None, None, None, one, 1 << 30, None) == -1
    assert L.pc_chunk_prefill_attn(ctypes.byref(good), one, one, one, None, one, one, None, None, None, one, 16, None) == -3
    assert L.pc_chunk_prefill_attn(ctypes.byref(good), one, one, one, None, one, one, None, None, None, None, 0, None) == -3
    for field, value in (("head_dim", 96), ("n_q_heads", 7), ("n_chunks", 0), ("rope_base", 0.5)):
        bad = pc.make_shape(2, 64, 16, 8, 2, 128, 8, 1e4)
        setattr(bad, field, value)
        assert L.pc_chunk_prefill_attn(ctypes.byref(bad), one, one, one, None, one, one, None, None, None, one, 1 << 30, None) == -2
        assert pc.pc_chunk_prefill_workspace_bytes(bad) == 0
    bad = pc.make_shape(2, 64, 16, 8, 2, 128, 100, 1e4)     # obs_window too large
    assert L.pc_chunk_query_scores(ctypes.byref(bad), one, one, None, one, None, one, 1 << 30, None) == -2
    # ragged chunks: the voting window must fit the query block (a chunk may be empty)
    ragged = pc.make_shape(2, 64, 16, 8, 2, 128, 17, 1e4)
    assert L.pc_chunk_query_scores(ctypes.byref(ragged), one, one, one, one, None, one, 1 << 30, None) == -2
    assert L.pc_chunk_prefill_attn(ctypes.byref(ragged), one, one, one, one, one, one, None, one, None, one, 1 << 30, None) == -2
    assert pc.pc_chunk_query_scores_workspace_bytes(ragged) > 0       # fine with full chunks
    # chunk_score without tok_score
    assert L.pc_chunk_prefill_attn(ctypes.byref(good), one, one, one, None, one, one, None, None, one, one, 1 << 30, None) == -1
    # parallel attention
    args = (1, 1, 2, 64, 8, 2, 128, -1, 1e4, 0.0)
    assert L.pc_parallel_attn(None, one, one, None, 0, None, None, *args, one, None, one, 1 << 30, None) == -1
    assert L.pc_parallel_attn(one, one, one, None, 0, one, None, *args, one, None, one, 1 << 30, None) == -1
    assert L.pc_parallel_attn(one, one, one, None, 0, None, None, *args, one, None, one, 8, None) == -3
    assert L.pc_parallel_attn(one, one, one, one, 2, None, None, *args, one, None, one, 1 << 30, None) == -2
    bad_args = (1, 1, 2, 64, 8, 3, 128, -1, 1e4, 0.0)
    assert L.pc_parallel_attn(one, one, one, None, 0, None, None, *bad_args, one, None, one, 1 << 30, None) == -2
    # misaligned tensors and shapes beyond the kernels' 32-bit indexing are shape errors
    odd = ctypes.c_void_p(264)
    assert L.pc_parallel_attn(odd, one, one, None, 0, None, None, *args, one, None, one, 1 << 30, None) == -2
    assert L.pc_parallel_attn(one, one, odd, None, 0, None, None, *args, one, None, one, 1 << 30, None) == -2
    huge = (1 << 20, 1, 1 << 20, 64, 8, 2, 128, -1, 1e4, 0.0)
    assert L.pc_parallel_attn(one, one, one, None, 0, None, None, *huge, one, None, one, 1 << 30, None) == -2
    assert L.pc_chunk_prefill_attn(ctypes.byref(good), odd, one, one, None, one, one, None, None, None, one, 1 << 30, None) == -2
    # the variant that allocates nothing: same checks, plus its own limits (all on the host)
    assert L.pc_parallel_attn_static(None, one, one, None, 0, None, None, *args, one, None, None) == -1
    assert L.pc_parallel_attn_static(one, one, one, None, 0, None, None, *bad_args, one, None, None) == -2
    many_rows = (1, 64, 2, 64, 8, 2, 128, -1, 1e4, 0.0)     # 64 query rows: the tile path
    assert L.pc_parallel_attn_static(one, one, one, None, 0, None, None, *many_rows, one, None, None) == -5
    too_big = (4096, 1, 2, 64, 32, 8, 128, -1, 1e4, 0.0)    # partials beyond the fixed scratch
    assert pc.pc_parallel_attn_workspace_bytes(4096, 1, 2, 64, 32, 8, 128, 0) > pc.pc_parallel_attn_static_max_bytes()
    assert L.pc_parallel_attn_static(one, one, one, None, 0, None, None, *too_big, one, None, None) == -3
    # decoding stage: append to the tail segment
    ok = (2, 1, 3, 2, 64, 2, 128, 10, 1e4)          # batch, n_new, n_seg, seg, k_t, H_kv, D, pos0, base
    assert L.pc_kv_append(None, one, *ok, one, one, one, 0, None) == -1
    assert L.pc_kv_append(one, one, *ok, one, one, None, 0, None) == -1
    for i, value in ((3, 3), (3, -1), (6, 96), (8, 0.5), (4, 0), (2, 0)):   # seg, seg, D, base, k_t, n_seg
        bad = list(ok); bad[i] = value
        assert L.pc_kv_append(one, one, *bad, one, one, one, 0, None) == -2, (i, value)
    assert L.pc_kv_append(one, one, 2, 0, *ok[2:], one, one, one, 0, None) == 0    # nothing to append
    assert L.pc_kv_append(one, one, 0, 1, *ok[2:], one, one, one, 0, None) == 0
    # 8-bit cache
    qa = (0, 2, 3, 64, 2, 128)                      # seg_len_per_head, batch, n_seg, k_t, H_kv, D
    assert L.pc_kv_quantize_fp8(None, one, None, *qa, one, one, one, one, None) == -1
    assert L.pc_kv_quantize_fp8(None, None, None, 0, 2, 0, 64, 2, 128, None, None, None, None, None) == 0   # no segments
    assert L.pc_kv_quantize_fp8(one, one, None, *qa, one, one, None, one, None) == -1
    assert L.pc_kv_quantize_fp8(one, one, None, 0, 2, 3, 64, 2, 96, one, one, one, one, None) == -2
    assert L.pc_kv_quantize_fp8(one, one, None, 2, 2, 3, 64, 2, 128, one, one, one, one, None) == -2
    assert L.pc_kv_quantize_fp8(one, one, None, 0, 0, 3, 64, 2, 128, one, one, one, one, None) == 0   # empty batch
    pa = (0, 1, 1, 2, 64, 8, 2, 128, -1)            # tail_cap, batch, n_q, n_seg, k_t, H_q, H_kv, D, q_pos0
    call = lambda q, k8, tail, args, wsb, kself=None, vself=None: L.pc_parallel_attn_fp8(
        q, k8, one, one, one, None, 0, tail, tail, tail, args[0], kself, vself, *args[1:], 1e4, 0.0, one, None,
        one, wsb, None)
    assert call(None, one, None, pa, 1 << 30) == -1
    assert call(one, None, None, pa, 1 << 30) == -1
    assert call(one, one, None, pa, 8) == -3
    assert call(one, one, None, (16,) + pa[1:], 1 << 30) == -1                  # tail_cap > 0 without a tail
    assert call(one, one, None, (0, 1, 5, 2, 64, 8, 2, 128, -1), 8) == -3        # 20 query columns: the tile path
    assert call(one, one, None, (0, 1, 1, 0, 64, 8, 2, 128, -1), 1 << 30) == -2  # nothing to attend to
    assert call(one, one, None, pa, 1 << 30, kself=one) == -1                   # k_self without v_self
    a8 = pc.pc_parallel_attn_fp8_workspace_bytes(1, 1, 2, 4096, 0, 8, 2, 128)
    assert 0 < a8 < pc.pc_parallel_attn_fp8_workspace_bytes(1, 1, 2, 4096, 512, 8, 2, 128)
    # a query block widens the segments into the workspace: much larger, larger still with a self segment
    t8 = pc.pc_parallel_attn_fp8_workspace_bytes(1, 64, 2, 4096, 0, 8, 2, 128)
    assert a8 < t8 < pc.pc_parallel_attn_fp8_workspace_bytes(1, 64, 2, 4096, 0, 8, 2, 128, True)


def test_workspace_sizes_are_positive_and_monotone():
    s1 = pc.make_shape(2, 64, 16, 8, 2, 128, 8, 1e4)
    s2 = pc.make_shape(4, 64, 16, 8, 2, 128, 8, 1e4)
    assert 0 < pc.pc_chunk_prefill_workspace_bytes(s1) < pc.pc_chunk_prefill_workspace_bytes(s2)
    assert pc.pc_chunk_query_scores_workspace_bytes(s1) > 0
    a = pc.pc_parallel_attn_workspace_bytes(1, 1, 4, 256, 8, 2, 128, 0)
    b = pc.pc_parallel_attn_workspace_bytes(2, 1, 4, 256, 8, 2, 128, 0)
    assert 0 < a < b
    assert pc.pc_parallel_attn_workspace_bytes(1, 64, 4, 256, 8, 2, 128, 1) > a


def test_header_compiles_as_c_and_links_from_a_c_program(tmp_path):
    """The boundary is a C ABI: a plain C program (gcc, -std=c99 -pedantic) includes both headers,
    links against the library and gets status codes for bad arguments, all without a GPU."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    src = os.path.join(ROOT, "tests", "c_abi", "host_check.c")
    exe = str(tmp_path / "host_check")
    lib_dir = os.path.join(ROOT, "paper_2502_14317_amd")
    subprocess.run([gcc, "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), src,
                    "-o", exe, "-L", lib_dir, "-l:libparallelcomp.so", "-Wl,-rpath," + lib_dir,
                    "-Wl,-rpath,/opt/rocm/lib"], check=True)
    out = subprocess.run([exe], capture_output=True, text=True)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "c abi ok" in out.stdout
