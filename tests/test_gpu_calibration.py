"""GPU parity of attention calibration (Eq. 8 then Eq. 7) and of per-head segment lengths in the
global attention, against the fp64 CPU oracle on the same seeded inputs."""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2502_14317_amd as pc
from paper_2502_14317_amd.layer import ParallelCompLayer
from workloads import CFG0U, CFG1_SMALL, prefill_inputs, bf16_bits_to_f64, f32_to_bf16_bits
from helpers import (O_ATOL, O_RTOL, LSE_ATOL, bits_to_dev, dev_to_bits, dev_bf16_to_f64,
                     assert_close, assert_selection_matches)

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("n,k", [(37, 9), (512, 128), (7680, 2048), (3000, 3000)])
def test_select_tokens_calibrated_bit_exact(n, k):
    """Integer work on given fp32 scores: indices, padding and counts must equal the oracle's."""
    _say(f"calibrated select n={n} k={k}")
    r = np.random.default_rng([41, n, k])
    C, H = 3, 2
    score = r.standard_normal((C, H, n)).astype(np.float32)
    score[0, 0, : n // 2] = np.float32(0.5)                    # a long run of ties
    score[1, 1, 3] = np.nan
    score[2, 0, 5] = np.inf
    score[2, 1, 7] = -np.inf
    cidx = np.array([2, 0, 1], dtype=np.int32)
    lam = float(np.float32(0.3))
    cases = [(lam, 0, min(100, n)), (lam, max(n - 100, 0), n), (lam, min(100, n), max(n - 100, min(100, n))),
             (-math.inf, 0, n - min(n, 5)), (math.inf, 0, n), (lam, 4, 4), (0.5, 0, n)]
    dscore, dcidx = torch.from_numpy(score).cuda(), torch.from_numpy(cidx).cuda()
    for lam_, lo, hi in cases:
        idx = torch.full((C, H, k), 12345, dtype=torch.int32, device="cuda")
        cnt = torch.full((C, H), -7, dtype=torch.int32, device="cuda")
        pc.pc_select_tokens_calibrated(dscore, dcidx, C, H, n, k, lam_, lo, hi, idx, cnt)
        torch.cuda.synchronize()
        ridx, rcnt = oracle.select_tokens_calibrated(score[cidx].astype(np.float64), k, lam_, lo, hi)
        assert np.array_equal(cnt.cpu().numpy(), rcnt), (lam_, lo, hi)
        assert np.array_equal(idx.cpu().numpy(), ridx), (lam_, lo, hi)
    # an empty class or lambda = +inf is Eq. 7 itself
    plain = torch.empty((C, H, k), dtype=torch.int32, device="cuda")
    pc.pc_select_tokens_topk(dscore, dcidx, C, H, n, k, plain)
    idx = torch.empty_like(plain); cnt = torch.empty((C, H), dtype=torch.int32, device="cuda")
    pc.pc_select_tokens_calibrated(dscore, dcidx, C, H, n, k, math.inf, 0, n, idx, cnt)
    torch.cuda.synchronize()
    assert torch.equal(idx, plain) and bool((cnt == k).all())


def _parallel_attn_per_head(name, B, n_q, S, kt, Hq, Hkv, D, with_self, seed):
    _say(f"parallel_attn per-head lengths {name}")
    r = np.random.default_rng([43, seed])
    def mk(shape, s=1.0):
        return f32_to_bf16_bits((r.standard_normal(shape) * s).astype(np.float32))
    q, kc, vc = mk((B, n_q, Hq, D), 3.0), mk((B, S, Hkv, kt, D)), mk((B, S, Hkv, kt, D))
    ks = mk((B, n_q, Hkv, D)) if with_self else None
    vs = mk((B, n_q, Hkv, D)) if with_self else None
    sl = r.integers(0, kt + 1, size=(B, S, Hkv)).astype(np.int32)
    sl[0, 0, 0] = kt; sl[0, 0, Hkv - 1] = 0; sl[B - 1, S - 1, 0] = 1
    # rows past a head's length hold garbage that must not matter
    for b in range(B):
        for s_ in range(S):
            for g in range(Hkv):
                kc[b, s_, g, sl[b, s_, g]:] = 0x7f00      # large finite bf16
    out = torch.empty((B, n_q, Hq, D), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((B, Hq, n_q), dtype=torch.float32, device="cuda")
    ws = pc.alloc_workspace(pc.pc_parallel_attn_workspace_bytes(B, n_q, S, kt, Hq, Hkv, D, with_self))
    pc.pc_parallel_attn(bits_to_dev(q), bits_to_dev(kc), bits_to_dev(vc), torch.from_numpy(sl).cuda(),
                        bits_to_dev(ks) if with_self else None, bits_to_dev(vs) if with_self else None,
                        B, n_q, S, kt, Hq, Hkv, D, -1, 1.0e4, 0.0, out, lse, ws, seg_len_per_head=1)
    torch.cuda.synchronize()
    for b in range(B):
        if not with_self and (sl[b].sum(axis=0) == 0).any():
            continue                                    # a head with no key at all has no softmax
        ro, rl = oracle.global_attention_concat(
            bf16_bits_to_f64(q[b]), bf16_bits_to_f64(kc[b]), bf16_bits_to_f64(vc[b]),
            bf16_bits_to_f64(ks[b]) if with_self else None, bf16_bits_to_f64(vs[b]) if with_self else None,
            seg_len=sl[b])
        assert_close(dev_bf16_to_f64(out[b]), ro, O_ATOL, O_RTOL, f"{name} out[b={b}]")
        assert_close(lse[b].cpu().numpy().T, rl, LSE_ATOL, 1e-3, f"{name} lse[b={b}]")


def test_parallel_attn_per_head_lengths_decode_and_block():
    _parallel_attn_per_head("decode", 2, 1, 4, 300, 8, 2, 128, True, 1)
    _parallel_attn_per_head("decode-mha64", 2, 2, 3, 97, 4, 4, 64, True, 2)
    _parallel_attn_per_head("block", 1, 104, 3, 200, 8, 2, 128, True, 3)
    _parallel_attn_per_head("block-64", 2, 150, 2, 130, 4, 4, 64, True, 4)


def _layer_with_calibration(cfg, calibration, what):
    _say(f"layer {cfg.name} with calibration {what}")
    q, k, v = prefill_inputs(cfg)
    qf, kf, vf = (bf16_bits_to_f64(x) for x in (q, k, v))
    ref = oracle.parallelcomp_layer(qf, kf, vf, cfg.chunk_len, cfg.obs_window, cfg.keep_chunks,
                                    cfg.keep_tokens, cfg.rope_base, attn_rows=np.arange(cfg.chunk_len, cfg.seq_len),
                                    calibration=calibration)
    layer = ParallelCompLayer(cfg.n_chunks, cfg.chunk_len, cfg.query_len, cfg.n_q_heads,
                              cfg.n_kv_heads, cfg.head_dim, cfg.obs_window, cfg.rope_base,
                              cfg.keep_chunks, cfg.keep_tokens, calibration=calibration)
    layer.forward(bits_to_dev(q), bits_to_dev(k), bits_to_dev(v))
    torch.cuda.synchronize()
    g_cidx = layer.chunk_idx.cpu().numpy()
    assert_selection_matches(g_cidx, ref["chunk_idx"], ref["chunk_score"], "chunk selection")
    g_tidx, g_cnt = layer.tok_idx.cpu().numpy(), layer.tok_cnt.cpu().numpy()
    # the GPU's selection on the GPU's own fp32 scores: bit-exact integer work
    own_idx, own_cnt = oracle.select_tokens_calibrated(
        layer.tok_score.cpu().numpy()[g_cidx].astype(np.float64), cfg.keep_tokens, *calibration)
    assert np.array_equal(g_cnt, own_cnt) and np.array_equal(g_tidx, own_idx)
    # against the oracle's scores: same sets outside the tie zone (eviction by lambda included:
    # lambda is placed in a gap of the oracle's scores by the caller)
    ridx, rcnt = oracle.select_tokens_calibrated(ref["tok_score"][g_cidx], cfg.keep_tokens, *calibration)
    assert np.array_equal(g_cnt, rcnt)
    n_diff = 0
    for s_ in range(cfg.keep_chunks):
        for g in range(cfg.n_kv_heads):
            c = rcnt[s_, g]
            if c:
                n_diff += assert_selection_matches(g_tidx[s_, g, :c], ridx[s_, g, :c],
                                                   ref["tok_score"][g_cidx[s_], g], f"tokens {s_},{g}")
    _say(f"  counts {sorted(set(g_cnt.ravel().tolist()))}, selection differences inside the tie zone: {n_diff}")
    rk, rv = oracle.gather_kv(dev_to_bits(layer.k_rope), v, g_cidx, g_tidx)
    assert np.array_equal(dev_to_bits(layer.kc[0]), rk) and np.array_equal(dev_to_bits(layer.vc[0]), rv)
    w = cfg.chunk_len
    kc_ref, vc_ref = oracle.gather_kv(ref["k_rope"], vf, g_cidx, g_tidx)
    og, lg = oracle.global_attention_concat(ref["q_rot_query"], kc_ref, vc_ref, ref["k_rope"][0, w:],
                                            vf[0, w:], seg_len=g_cnt)
    assert_close(dev_bf16_to_f64(layer.global_o[0]), og, O_ATOL, O_RTOL, "global_o")
    assert_close(layer.global_lse[0].cpu().numpy().T, lg, LSE_ATOL, 1e-3, "global_lse")
    return ref, layer


def _lambda_in_a_gap(tok_score, lo, hi, rank):
    """A threshold between the rank-th and (rank+1)-th largest class score of every head, placed
    in the widest relative gap near that rank so that fp32 score error cannot flip a decision."""
    cls = np.sort(tok_score[..., lo:hi].reshape(-1))[::-1]
    best, lam = -1.0, None
    for r_ in range(max(rank - 3, 0), rank + 4):
        gap = (cls[r_] - cls[r_ + 1]) / abs(cls[r_])
        if gap > best:
            best, lam = gap, 0.5 * (cls[r_] + cls[r_ + 1])
    assert best > 1e-2
    return float(np.float32(lam))


def test_layer_with_sink_eviction_and_compression():
    """R_s of the appendix: the first-100-token class; lambda sits above all but the few largest
    class scores (the planted sink tokens among them)."""
    cfg = CFG0U
    q, k, v = prefill_inputs(cfg)
    base = oracle.parallelcomp_layer(*(bf16_bits_to_f64(x) for x in (q, k, v)), cfg.chunk_len, cfg.obs_window,
                                     cfg.keep_chunks, cfg.keep_tokens, cfg.rope_base, attn_rows=np.array([cfg.seq_len - 1]))
    lam = _lambda_in_a_gap(base["tok_score"][base["chunk_idx"]], 0, 100, 6)
    ref, layer = _layer_with_calibration(cfg, (lam, 0, 100), f"R_s lambda={lam:.4g}")
    assert (ref["tok_cnt"] == cfg.keep_tokens).all()
    assert not np.array_equal(ref["tok_idx"], base["tok_idx"])            # something was evicted


def test_layer_with_whole_class_eviction_leaves_ragged_heads():
    """lambda = -inf on a class that covers most of the chunk: fewer than k tokens are left, the
    heads come out padded and the global attention must honour the per-head counts."""
    cfg = CFG1_SMALL
    lo, hi = 10, cfg.chunk_len - 20
    ref, layer = _layer_with_calibration(cfg, (-math.inf, lo, hi), "whole class")
    assert (ref["tok_cnt"] == 30).all() and cfg.keep_tokens > 30
