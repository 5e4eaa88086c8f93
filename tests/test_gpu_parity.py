"""GPU parity: every C-ABI call against the fp64 CPU oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

import oracle
import paper_2502_14317_amd as pc
from paper_2502_14317_amd.layer import ParallelCompLayer
from workloads import (CFG0, CFG0U, CFG1_SMALL, CFG2_SMALL, CFG4_SMALL, prefill_inputs,
                       decode_inputs, gather_inputs, bf16_bits_to_f64, f32_to_bf16_bits)
from helpers import (O_ATOL, O_RTOL, S_RTOL, S_ATOL, LSE_ATOL, bits_to_dev, dev_to_bits,
                     dev_bf16_to_f64, assert_close, assert_selection_matches)

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


# ------------------------------------------------------------------------------ gather (Eq. 7)
@pytest.mark.parametrize("D", [128, 64])
@pytest.mark.parametrize("with_chunk_idx", [True, False])
def test_gather_bit_exact(D, with_chunk_idx):
    _say(f"gather D={D} chunk_idx={with_chunk_idx}")
    r = np.random.default_rng([11, D, int(with_chunk_idx)])
    B, C, R, H, n_sel, k = 2, 5, 131, 3, 3, 37
    ks = r.integers(0, 2 ** 16, size=(B, C, R, H, D)).astype(np.uint16)
    vs = r.integers(0, 2 ** 16, size=(B, C, R, H, D)).astype(np.uint16)
    cidx = np.stack([r.choice(C, n_sel, replace=False) for _ in range(B)]).astype(np.int32)
    if not with_chunk_idx:
        cidx = np.broadcast_to(np.arange(n_sel, dtype=np.int32), (B, n_sel)).copy()
    tidx = r.integers(0, R, size=(B, n_sel, H, k)).astype(np.int32)
    kd = torch.empty((B, n_sel, H, k, D), dtype=torch.bfloat16, device="cuda")
    vd = torch.empty_like(kd)
    pc.pc_gather_kv(bits_to_dev(ks), bits_to_dev(vs),
                    torch.from_numpy(cidx).cuda() if with_chunk_idx else None,
                    torch.from_numpy(tidx).cuda(), B, C, R, n_sel, H, k, D, kd, vd)
    torch.cuda.synchronize()
    for b in range(B):
        rk, rv = oracle.gather_kv(ks[b], vs[b], cidx[b], tidx[b])
        assert np.array_equal(dev_to_bits(kd[b]), rk)
        assert np.array_equal(dev_to_bits(vd[b]), rv)


def test_gather_out_of_range_indices_give_zero_rows_and_empty_is_ok():
    _say("gather out-of-range / empty")
    r = np.random.default_rng(12)
    C, R, H, k, D = 2, 9, 2, 4, 128
    ks = r.integers(1, 2 ** 15, size=(1, C, R, H, D)).astype(np.uint16)
    tidx = np.array([[[0, 8, 9, -1], [3, 100000, 2, 1]]], dtype=np.int32)[None]   # [1,1,H,k]
    kd = torch.full((1, 1, H, k, D), 7.0, dtype=torch.bfloat16, device="cuda")
    vd = torch.full_like(kd, 7.0)
    src = bits_to_dev(ks)
    pc.pc_gather_kv(src, src, None, torch.from_numpy(tidx).cuda(), 1, C, R, 1, H, k, D, kd, vd)
    pc.pc_gather_kv(src, src, None, torch.from_numpy(tidx).cuda(), 1, C, R, 0, H, k, D, kd, vd)
    torch.cuda.synchronize()
    out = dev_to_bits(kd)[0, 0]
    assert np.array_equal(out[0, 0], ks[0, 0, 0, 0]) and np.array_equal(out[0, 1], ks[0, 0, 8, 0])
    assert not out[0, 2].any() and not out[0, 3].any() and not out[1, 1].any()
    assert np.array_equal(out[1, 0], ks[0, 0, 3, 1])


def test_gather_decode_workload_shape():
    cfg = CFG4_SMALL
    _say(f"gather {cfg.name}")
    ks, vs, cidx, tidx = gather_inputs(cfg)
    B, S, R, H, D = ks.shape
    kd = torch.empty((B, S, H, cfg.keep_tokens, D), dtype=torch.bfloat16, device="cuda")
    vd = torch.empty_like(kd)
    pc.pc_gather_kv(bits_to_dev(ks), bits_to_dev(vs), None, torch.from_numpy(tidx).cuda(), B, S, R,
                    S, H, cfg.keep_tokens, D, kd, vd)
    torch.cuda.synchronize()
    for b in range(B):
        rk, rv = oracle.gather_kv(ks[b], vs[b], cidx, tidx[b])
        assert np.array_equal(dev_to_bits(kd[b]), rk) and np.array_equal(dev_to_bits(vd[b]), rv)


# ------------------------------------------------------------------------------ selection
@pytest.mark.parametrize("n,k", [(1, 1), (4, 2), (64, 8), (64, 64), (777, 100), (4096, 300)])
def test_select_chunks_exact(n, k):
    _say(f"select_chunks n={n} k={k}")
    r = np.random.default_rng([13, n, k])
    s = np.round(r.standard_normal(n), 1).astype(np.float32)        # many ties
    if n >= 64:
        s[5] = np.nan; s[6] = -np.inf; s[7] = np.inf; s[8] = -0.0; s[9] = 0.0
    out = torch.empty(k, dtype=torch.int32, device="cuda")
    outs = torch.empty(k, dtype=torch.float32, device="cuda")
    pc.pc_select_chunks_topk(torch.from_numpy(s).cuda(), n, k, out, outs)
    torch.cuda.synchronize()
    # NaN orders below everything, -inf included: the reference ranks it last
    ref_in = np.where(np.isnan(s), -np.inf, s).astype(np.float64)
    order = np.lexsort((np.arange(n), -ref_in))
    if n >= 64:
        order = np.concatenate([order[order != 5], [5]])
    order = order[:k]
    if n < 64:
        np.testing.assert_array_equal(order, oracle.select_chunks(ref_in, k))
    got = out.cpu().numpy()
    np.testing.assert_array_equal(got, order)
    np.testing.assert_array_equal(np.nan_to_num(outs.cpu().numpy(), nan=-1e30),
                                  np.nan_to_num(s[got], nan=-1e30))


@pytest.mark.parametrize("n,k", [(512, 128), (600, 200), (7680, 2048), (3584, 1024), (8192, 1),
                                 (1000, 1000), (32768, 4097), (65, 64)])
def test_select_tokens_exact(n, k):
    _say(f"select_tokens n={n} k={k}")
    r = np.random.default_rng([14, n, k])
    C, H = 5, 3
    s = r.random((C, H, n)).astype(np.float32)
    s[0] = np.round(s[0], 2)                  # heavy ties
    s[1, 0] = 0.25                            # all equal: lowest indices win
    s[2, 1, ::2] = 1.0                        # half at the maximum
    cidx = np.array([3, 0, 2, 1], dtype=np.int32)
    out = torch.empty((4, H, k), dtype=torch.int32, device="cuda")
    pc.pc_select_tokens_topk(torch.from_numpy(s).cuda(), torch.from_numpy(cidx).cuda(), 4, H, n, k, out)
    torch.cuda.synchronize()
    ref = oracle.select_tokens(s[cidx].astype(np.float64), k)
    np.testing.assert_array_equal(out.cpu().numpy(), ref)
    out2 = torch.empty((C, H, k), dtype=torch.int32, device="cuda")
    pc.pc_select_tokens_topk(torch.from_numpy(s).cuda(), None, C, H, n, k, out2)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out2.cpu().numpy(), oracle.select_tokens(s.astype(np.float64), k))


# ------------------------------------------------------------------------------ Eq. 9-11
def _parallel_attn_case(name, B, n_q, S, kt, Hq, Hkv, D, with_self, q_pos0, ragged, seed, scale=0.0):
    _say(f"parallel_attn {name}: B={B} n_q={n_q} S={S} kt={kt} H={Hq}/{Hkv} D={D} self={with_self} "
         f"pos0={q_pos0} ragged={ragged}")
    r = np.random.default_rng([15, seed])
    # q entries have std 3: logits with std ~ 3, a peaked softmax
    def mk(shape, s=1.0):
        return f32_to_bf16_bits((r.standard_normal(shape) * s).astype(np.float32))
    q, kc, vc = mk((B, n_q, Hq, D), 3.0), mk((B, S, Hkv, kt, D)), mk((B, S, Hkv, kt, D))
    ks = mk((B, n_q, Hkv, D)) if with_self else None
    vs = mk((B, n_q, Hkv, D)) if with_self else None
    seg_len = None
    if ragged:
        seg_len = r.integers(1, kt + 1, size=(B, S)).astype(np.int32)
        seg_len[0, 0] = kt
        if S > 1:
            seg_len[0, 1] = 0
        if S > 2:
            seg_len[-1, 2] = 1
    out = torch.empty((B, n_q, Hq, D), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((B, Hq, n_q), dtype=torch.float32, device="cuda")
    ws = pc.alloc_workspace(pc.pc_parallel_attn_workspace_bytes(B, n_q, S, kt, Hq, Hkv, D, with_self))
    pc.pc_parallel_attn(bits_to_dev(q), bits_to_dev(kc), bits_to_dev(vc),
                        torch.from_numpy(seg_len).cuda() if ragged else None,
                        bits_to_dev(ks) if with_self else None, bits_to_dev(vs) if with_self else None,
                        B, n_q, S, kt, Hq, Hkv, D, q_pos0, 1.0e4, scale, out, lse, ws)
    torch.cuda.synchronize()
    eff = scale if scale > 0 else 1.0 / np.sqrt(D)
    for b in range(B):
        qf = bf16_bits_to_f64(q[b])
        if q_pos0 >= 0:
            qf = oracle.rope(qf, q_pos0 + np.arange(n_q), 1.0e4)
        ro, rl = oracle.global_attention_concat(
            qf, bf16_bits_to_f64(kc[b]), bf16_bits_to_f64(vc[b]),
            bf16_bits_to_f64(ks[b]) if with_self else None,
            bf16_bits_to_f64(vs[b]) if with_self else None,
            seg_len=seg_len[b] if ragged else None, scale=eff)
        assert_close(dev_bf16_to_f64(out[b]), ro, O_ATOL, O_RTOL, f"{name} out[b={b}]")
        assert_close(lse[b].cpu().numpy().T, rl, LSE_ATOL, 1e-3, f"{name} lse[b={b}]")


def test_parallel_attn_decode_gqa():
    _parallel_attn_case("decode", 3, 1, 5, 333, 32, 8, 128, False, -1, False, 1)


def test_parallel_attn_decode_ragged_self_rope():
    _parallel_attn_case("decode-ragged", 2, 1, 4, 1100, 8, 2, 128, True, 4000, True, 2)
    _parallel_attn_case("decode-nq2-mha64", 2, 2, 3, 97, 4, 4, 64, True, 10, True, 3, scale=0.2)
    _parallel_attn_case("decode-nq4-g4", 1, 4, 2, 2048, 8, 2, 128, True, -1, False, 4)
    _parallel_attn_case("decode-self-only", 1, 3, 0, 64, 4, 2, 64, True, -1, False, 5)


def _drawn_attn_cases(n):
    r = np.random.default_rng([2502, 98])
    out = []
    for i in range(n):
        D = int(r.choice([64, 128]))
        Hkv = int(r.choice([1, 2, 3]))
        G = int(r.choice([1, 2, 4, 8]))
        n_q = int(r.choice([1, 2, 3, 5, 17, 70, 131]))
        with_self = bool(r.integers(0, 2))
        S = int(r.integers(0 if with_self else 1, 6))
        out.append((int(r.integers(1, 4)), n_q, S, int(r.integers(1, 300)), Hkv * G, Hkv, D, with_self,
                    int(r.choice([-1, 0, 777])), bool(r.integers(0, 2)) and S > 0, 100 + i))
    return out


@pytest.mark.parametrize("case", _drawn_attn_cases(12), ids=lambda c: "x".join(str(int(x)) for x in c[:10]))
def test_parallel_attn_drawn_shapes(case):
    """Twelve calls drawn from a fixed seed: the single-row path (n_q * G <= 16) and the tile path,
    with and without the causal self segment, rotated or not, ragged or full segments."""
    B, n_q, S, kt, Hq, Hkv, D, with_self, q_pos0, ragged, seed = case
    _parallel_attn_case("drawn", B, n_q, S, kt, Hq, Hkv, D, with_self, q_pos0, ragged, seed)


def test_parallel_attn_decode_many_ragged_groups():
    """Enough (sequence, KV head, segment) groups that a workgroup takes several consecutive
    segments, with ragged lengths (empty segments in the middle and at the end of a group)."""
    B, S, kt, Hq, Hkv, D = 64, 8, 48, 16, 8, 64
    _say(f"parallel_attn many groups: B={B} S={S} kt={kt} H={Hq}/{Hkv} D={D}")
    r = np.random.default_rng([15, 99])
    mk = lambda shape, sc=1.0: f32_to_bf16_bits((r.standard_normal(shape) * sc).astype(np.float32))
    q, kc, vc = mk((B, 1, Hq, D), 3.0), mk((B, S, Hkv, kt, D)), mk((B, S, Hkv, kt, D))
    seg_len = r.integers(0, kt + 1, size=(B, S)).astype(np.int32)
    seg_len[0] = [kt, 0, 0, 5, 0, kt, 0, 0]
    seg_len[1] = [0, 0, 0, 0, 0, 0, 0, 1]
    seg_len[2] = 0                                           # nothing to attend to: zeros, lse = -inf
    out = torch.empty((B, 1, Hq, D), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((B, Hq, 1), dtype=torch.float32, device="cuda")
    ws = pc.alloc_workspace(pc.pc_parallel_attn_workspace_bytes(B, 1, S, kt, Hq, Hkv, D, 0))
    pc.pc_parallel_attn(bits_to_dev(q), bits_to_dev(kc), bits_to_dev(vc), torch.from_numpy(seg_len).cuda(), None, None,
                        B, 1, S, kt, Hq, Hkv, D, -1, 1.0e4, 0.0, out, lse, ws)
    torch.cuda.synchronize()
    assert (dev_bf16_to_f64(out[2]) == 0).all() and torch.isneginf(lse[2]).all()
    for b in (0, 1, 3, 17, 63):
        ro, rl = oracle.global_attention_concat(bf16_bits_to_f64(q[b]), bf16_bits_to_f64(kc[b]), bf16_bits_to_f64(vc[b]),
                                                seg_len=seg_len[b])
        assert_close(dev_bf16_to_f64(out[b]), ro, O_ATOL, O_RTOL, f"out[b={b}]")
        assert_close(lse[b].cpu().numpy().T, rl, LSE_ATOL, 1e-3, f"lse[b={b}]")


@pytest.mark.parametrize("per_head", [0, 1])
def test_parallel_attn_decode_more_segments_than_lanes(per_head):
    """150 short segments per group: the kernel's search for a wavefront's first block walks the
    segment lengths 64 at a time; ragged lengths with many empty segments, blocks of fewer than 32
    keys, and (per_head) a different length for every KV head."""
    B, S, kt, Hq, Hkv, D = 2, 150, 40, 8, 2, 128
    _say(f"parallel_attn 150 segments: B={B} S={S} kt={kt} H={Hq}/{Hkv} D={D} per_head={per_head}")
    r = np.random.default_rng([15, 150, per_head])
    mk = lambda shape, sc=1.0: f32_to_bf16_bits((r.standard_normal(shape) * sc).astype(np.float32))
    q, kc, vc = mk((B, 1, Hq, D), 2.0), mk((B, S, Hkv, kt, D)), mk((B, S, Hkv, kt, D))
    shape = (B, S, Hkv) if per_head else (B, S)
    seg_len = r.integers(0, kt + 1, size=shape).astype(np.int32)
    seg_len[r.random(shape) < 0.4] = 0
    seg_len[0, :70] = 0                                      # the first round of 64 lengths holds no key
    seg_len[1, 60:] = 0                                      # ... and here the later rounds hold none
    out = torch.empty((B, 1, Hq, D), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((B, Hq, 1), dtype=torch.float32, device="cuda")
    ws = pc.alloc_workspace(pc.pc_parallel_attn_workspace_bytes(B, 1, S, kt, Hq, Hkv, D, 0))
    pc.pc_parallel_attn(bits_to_dev(q), bits_to_dev(kc), bits_to_dev(vc), torch.from_numpy(seg_len).cuda(), None, None,
                        B, 1, S, kt, Hq, Hkv, D, -1, 1.0e4, 0.0, out, lse, ws, seg_len_per_head=per_head)
    torch.cuda.synchronize()
    for b in range(B):
        ro, rl = oracle.global_attention_concat(bf16_bits_to_f64(q[b]), bf16_bits_to_f64(kc[b]), bf16_bits_to_f64(vc[b]),
                                                seg_len=seg_len[b])
        assert_close(dev_bf16_to_f64(out[b]), ro, O_ATOL, O_RTOL, f"out[b={b}]")
        assert_close(lse[b].cpu().numpy().T, rl, LSE_ATOL, 1e-3, f"lse[b={b}]")


def test_parallel_attn_query_block():
    _parallel_attn_case("block", 1, 104, 3, 200, 8, 2, 128, True, 600, False, 6)
    _parallel_attn_case("block-ragged64", 2, 300, 2, 130, 4, 4, 64, True, -1, True, 7)
    _parallel_attn_case("block-noself", 1, 40, 2, 64, 8, 8, 128, False, -1, False, 8)


def test_parallel_attn_decode_workload():
    cfg = CFG4_SMALL
    _say(f"parallel_attn {cfg.name}")
    q, kc, vc = decode_inputs(cfg)
    B, S, Hkv, kt, D = kc.shape
    out = torch.empty((B, 1, cfg.n_q_heads, D), dtype=torch.bfloat16, device="cuda")
    ws = pc.alloc_workspace(pc.pc_parallel_attn_workspace_bytes(B, 1, S, kt, cfg.n_q_heads, Hkv, D, 0))
    pc.pc_parallel_attn(bits_to_dev(q), bits_to_dev(kc), bits_to_dev(vc), None, None, None, B, 1, S,
                        kt, cfg.n_q_heads, Hkv, D, -1, 1.0e4, 0.0, out, None, ws)
    torch.cuda.synchronize()
    for b in range(B):
        ro, _ = oracle.global_attention_concat(bf16_bits_to_f64(q[b]), bf16_bits_to_f64(kc[b]),
                                               bf16_bits_to_f64(vc[b]))
        rm, _ = oracle.global_attention_merged(bf16_bits_to_f64(q[b]), bf16_bits_to_f64(kc[b]),
                                               bf16_bits_to_f64(vc[b]))
        np.testing.assert_allclose(ro, rm, rtol=1e-10, atol=1e-12)
        assert_close(dev_bf16_to_f64(out[b]), ro, O_ATOL, O_RTOL, f"{cfg.name} out[b={b}]")


# ------------------------------------------------------------------------------ Eq. 1-2, 5-6
def _oracle_layer(cfg, q, k, v, rows=None):
    qf, kf, vf = (bf16_bits_to_f64(x) for x in (q, k, v))
    return oracle.parallelcomp_layer(qf, kf, vf, cfg.chunk_len, cfg.obs_window, cfg.keep_chunks,
                                     cfg.keep_tokens, cfg.rope_base, attn_rows=rows)


@pytest.mark.parametrize("cfg", [CFG0, CFG0U, CFG1_SMALL, CFG2_SMALL], ids=lambda c: c.name)
def test_chunk_prefill_and_layer(cfg):
    _say(f"layer {cfg.name}")
    q, k, v = prefill_inputs(cfg)
    ref = _oracle_layer(cfg, q, k, v)
    layer = ParallelCompLayer(cfg.n_chunks, cfg.chunk_len, cfg.query_len, cfg.n_q_heads,
                              cfg.n_kv_heads, cfg.head_dim, cfg.obs_window, cfg.rope_base,
                              cfg.keep_chunks, cfg.keep_tokens)
    qd, kd, vd = bits_to_dev(q), bits_to_dev(k), bits_to_dev(v)
    layer.forward(qd, kd, vd)
    torch.cuda.synchronize()
    # Eq. 1-2
    assert_close(dev_bf16_to_f64(layer.o), ref["o"], O_ATOL, O_RTOL, "o")
    assert_close(layer.lse.cpu().numpy().transpose(0, 2, 1), ref["lse"], LSE_ATOL, 1e-3, "lse")
    assert_close(dev_bf16_to_f64(layer.k_rope), ref["k_rope"], 1e-5, 2.0 ** -8, "k_rope")
    # Eq. 5-6
    assert_close(layer.tok_score.cpu().numpy(), ref["tok_score"], S_ATOL, S_RTOL, "tok_score")
    assert_close(layer.chunk_score.cpu().numpy(), ref["chunk_score"], S_ATOL, S_RTOL, "chunk_score")
    # standalone score call == fused result, bit for bit
    ts = torch.empty_like(layer.tok_score); cs = torch.empty_like(layer.chunk_score)
    ws = pc.alloc_workspace(pc.pc_chunk_query_scores_workspace_bytes(layer.shape))
    pc.pc_chunk_query_scores(layer.shape, qd, kd, ts, cs, ws)
    torch.cuda.synchronize()
    assert torch.equal(ts, layer.tok_score) and torch.equal(cs, layer.chunk_score)
    # Eq. 3-4 mechanics / Eq. 7: selections
    g_cidx = layer.chunk_idx.cpu().numpy()
    n_diff = assert_selection_matches(g_cidx, ref["chunk_idx"], ref["chunk_score"], "chunk selection")
    g_tidx = layer.tok_idx.cpu().numpy()
    ref_tidx = oracle.select_tokens(ref["tok_score"][g_cidx], cfg.keep_tokens)
    for s_ in range(cfg.keep_chunks):
        for g in range(cfg.n_kv_heads):
            assert list(g_tidx[s_, g]) == sorted(g_tidx[s_, g])
            n_diff += assert_selection_matches(g_tidx[s_, g], ref_tidx[s_, g],
                                               ref["tok_score"][g_cidx[s_], g],
                                               f"token selection chunk {g_cidx[s_]} head {g}")
    _say(f"  selection differences inside the tie zone: {n_diff}")
    # Eq. 7 gather: bit-exact copy of the GPU's own rotated keys / values at the GPU's indices
    rk, rv = oracle.gather_kv(dev_to_bits(layer.k_rope), v, g_cidx, g_tidx)
    assert np.array_equal(dev_to_bits(layer.kc[0]), rk) and np.array_equal(dev_to_bits(layer.vc[0]), rv)
    # Eq. 9-11: global attention over the kept KV (oracle evaluated on the GPU's valid selection)
    w = cfg.chunk_len
    kc_ref, vc_ref = oracle.gather_kv(ref["k_rope"], bf16_bits_to_f64(v), g_cidx, g_tidx)
    og, lg = oracle.global_attention_concat(ref["q_rot_query"], kc_ref, vc_ref, ref["k_rope"][0, w:],
                                            bf16_bits_to_f64(v)[0, w:])
    assert_close(dev_bf16_to_f64(layer.global_o[0]), og, O_ATOL, O_RTOL, "global_o")
    assert_close(layer.global_lse[0].cpu().numpy().T, lg, LSE_ATOL, 1e-3, "global_lse")
    if list(g_cidx) == list(ref["chunk_idx"]) and np.array_equal(g_tidx, ref["tok_idx"]):
        assert_close(dev_bf16_to_f64(layer.global_o[0]), ref["global_o"], O_ATOL, O_RTOL, "global_o (oracle sel)")


def test_layer_keeping_everything_is_one_softmax_over_all_chunks():
    """The degenerate case of the method: every chunk and every token kept.  The global attention
    of the query block is then one softmax over all rotated context keys and the query's own
    (the identity behind Eq. 9-11), whatever order the chunks were ranked in."""
    import dataclasses
    cfg = dataclasses.replace(CFG1_SMALL, keep_chunks=CFG1_SMALL.n_chunks, keep_tokens=CFG1_SMALL.chunk_len)
    _say(f"layer keeping everything {cfg.name}")
    q, k, v = prefill_inputs(cfg)
    layer = ParallelCompLayer(cfg.n_chunks, cfg.chunk_len, cfg.query_len, cfg.n_q_heads, cfg.n_kv_heads,
                              cfg.head_dim, cfg.obs_window, cfg.rope_base, cfg.keep_chunks, cfg.keep_tokens)
    layer.forward(bits_to_dev(q), bits_to_dev(k), bits_to_dev(v))
    torch.cuda.synchronize()
    assert sorted(layer.chunk_idx.cpu().tolist()) == list(range(cfg.n_chunks))
    assert (layer.tok_idx.cpu().numpy() == np.arange(cfg.chunk_len)).all()
    qf, kf, vf = (bf16_bits_to_f64(x) for x in (q, k, v))
    w, pos = cfg.chunk_len, np.arange(cfg.seq_len)
    k_rot = np.stack([oracle.rope(kf[c], pos, cfg.rope_base) for c in range(cfg.n_chunks)])
    q_rot = oracle.rope(qf[0], pos, cfg.rope_base)[w:]
    kc = k_rot[:, :w].transpose(0, 2, 1, 3)                   # [C, H_kv, w, D]
    vc = vf[:, :w].transpose(0, 2, 1, 3)
    og, lg = oracle.global_attention_concat(q_rot, kc, vc, k_rot[0, w:], vf[0, w:])
    assert_close(dev_bf16_to_f64(layer.global_o[0]), og, O_ATOL, O_RTOL, "global_o")
    assert_close(layer.global_lse[0].cpu().numpy().T, lg, LSE_ATOL, 1e-3, "global_lse")


def _drawn_shapes(n):
    """n layer shapes drawn from a fixed seed: chunk and query lengths that are no multiple of any
    tile, every group size 1 to 8, both head dimensions, voting windows from one row to more than
    the query block, and keep counts from 1 to everything."""
    r = np.random.default_rng([2502, 99])
    out = []
    for _ in range(n):
        D = int(r.choice([64, 128]))
        Hkv = int(r.choice([1, 2, 3]))
        G = int(r.choice([1, 2, 4, 8]))
        C = int(r.integers(1, 5))
        w = int(r.integers(1, 420))
        wq = int(r.integers(1, 150))
        w_obs = int(r.integers(1, w + wq + 1))
        out.append((C, w, wq, Hkv * G, Hkv, D, w_obs, int(r.integers(1, C + 1)), int(r.integers(1, w + 1)),
                    float(r.choice([1.0, 1.25]))))
    return out


_FIXED_SHAPES = [(1, 1, 1, 1, 1, 64, 1, 1, 1, 1.0), (3, 65, 3, 2, 1, 128, 2, 2, 64, 1.0),
                 (2, 127, 130, 4, 4, 64, 64, 1, 127, 1.0), (2, 700, 40, 8, 2, 128, 32, 1, 256, 1.25)]
_DRAWN_SHAPES = _drawn_shapes(10)


@pytest.mark.parametrize("C,w,wq,Hq,Hkv,D,w_obs,kc_n,kt_n,gain", _FIXED_SHAPES + _DRAWN_SHAPES,
                         ids=["one-token", "just-over-a-tile", "long-query", "wider-logits"]
                         + ["drawn-" + "x".join(str(x) for x in sh[:9]) for sh in _DRAWN_SHAPES])
def test_layer_tiny_and_ragged_tail_shapes(C, w, wq, Hq, Hkv, D, w_obs, kc_n, kt_n, gain):
    """Smallest possible shapes, sizes just past a tile boundary and ten shapes drawn from a fixed
    seed, unit-variance entries; where the gain is 1.25 the logits have a standard deviation of
    1.6 (q and k entries x 1.25)."""
    _say(f"tiny layer C={C} w={w} wq={wq} H={Hq}/{Hkv} D={D} gain={gain}")
    r = np.random.default_rng([16, C, w, wq])
    L = w + wq
    mk = lambda h: f32_to_bf16_bits(r.standard_normal((C, L, h, D)).astype(np.float32) * gain)
    q, k, v = mk(Hq), mk(Hkv), mk(Hkv)
    q[:, w:] = q[0, w:]; k[:, w:] = k[0, w:]; v[:, w:] = v[0, w:]          # same query rows in every chunk
    qf, kf, vf = (bf16_bits_to_f64(x) for x in (q, k, v))
    ref = oracle.parallelcomp_layer(qf, kf, vf, w, w_obs, kc_n, kt_n, 1.0e4)
    layer = ParallelCompLayer(C, w, wq, Hq, Hkv, D, w_obs, 1.0e4, kc_n, kt_n)
    layer.forward(bits_to_dev(q), bits_to_dev(k), bits_to_dev(v))
    torch.cuda.synchronize()
    assert_close(dev_bf16_to_f64(layer.o), ref["o"], O_ATOL, O_RTOL, "o")
    assert_close(layer.lse.cpu().numpy().transpose(0, 2, 1), ref["lse"], LSE_ATOL, 1e-3, "lse")
    assert_close(layer.tok_score.cpu().numpy(), ref["tok_score"], S_ATOL, S_RTOL, "tok_score")
    g_cidx, g_tidx = layer.chunk_idx.cpu().numpy(), layer.tok_idx.cpu().numpy()
    assert_selection_matches(g_cidx, ref["chunk_idx"], ref["chunk_score"], "chunk selection")
    ref_tidx = oracle.select_tokens(ref["tok_score"][g_cidx], kt_n)
    for s_ in range(kc_n):
        for g in range(Hkv):
            assert_selection_matches(g_tidx[s_, g], ref_tidx[s_, g], ref["tok_score"][g_cidx[s_], g], "tokens")
    kc_ref, vc_ref = oracle.gather_kv(ref["k_rope"], vf, g_cidx, g_tidx)
    og, lg = oracle.global_attention_concat(ref["q_rot_query"], kc_ref, vc_ref, ref["k_rope"][0, w:], vf[0, w:])
    assert_close(dev_bf16_to_f64(layer.global_o[0]), og, O_ATOL, O_RTOL, "global_o")
    assert_close(layer.global_lse[0].cpu().numpy().T, lg, LSE_ATOL, 1e-3, "global_lse")


def test_running_softmax_rescale_keeps_output_and_row_sum_consistent():
    """Logits with a standard deviation of 9 behind 64 nearly silent keys: the reference of the
    running softmax starts near 0 and is overtaken again and again, so the rare rescale path
    runs in most steps.  With identical value rows the output must be that row whatever the
    probabilities are (logits this large are beyond what bf16 operands resolve to the output
    tolerance, the normalisation is not), so O and the row sum must have been rescaled together."""
    C, w, wq, Hq, Hkv, D = 2, 700, 40, 8, 2, 128
    _say(f"rescale consistency C={C} w={w} wq={wq}")
    r = np.random.default_rng([17])
    L = w + wq
    qf = r.standard_normal((C, L, Hq, D)).astype(np.float32) * 3
    kf = r.standard_normal((C, L, Hkv, D)).astype(np.float32) * 3
    kf[:, :64] *= 0.01
    v0 = r.standard_normal((C, 1, Hkv, D)).astype(np.float32)
    q, k, v = f32_to_bf16_bits(qf), f32_to_bf16_bits(kf), f32_to_bf16_bits(np.repeat(v0, L, axis=1))
    shape = pc.make_shape(C, w, wq, Hq, Hkv, D, 32, 1.0e4)
    o = torch.empty((C, L, Hq, D), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((C, Hq, L), dtype=torch.float32, device="cuda")
    ws = pc.alloc_workspace(pc.pc_chunk_prefill_workspace_bytes(shape))
    pc.pc_chunk_prefill_attn(shape, bits_to_dev(q), bits_to_dev(k), bits_to_dev(v), o, lse, None, None, None, ws)
    torch.cuda.synchronize()
    want = np.repeat(bf16_bits_to_f64(v)[:, :, :, None, :], Hq // Hkv, axis=3).reshape(C, L, Hq, D)
    assert_close(dev_bf16_to_f64(o), want, O_ATOL, O_RTOL, "o with identical value rows")
    # the row logsumexp against the oracle on sampled rows: a probability-weighted mean of logit
    # errors, which grow with the logits (2^-8 relative per rounded operand pair)
    rows = np.array([0, 63, 64, 100, 333, 699, 700, 739])
    for c in range(C):
        pos = np.arange(L)
        q_rot = oracle.rope(bf16_bits_to_f64(q[c]), pos, 1.0e4)
        k_rot = oracle.rope(bf16_bits_to_f64(k[c]), pos, 1.0e4)
        _, rl = oracle.local_attention(q_rot, k_rot, bf16_bits_to_f64(v[c]), rows=rows)
        gl = lse[c].cpu().numpy().T[rows]
        assert np.all(np.abs(gl - rl) <= 2.0 ** -8 * np.abs(rl) + LSE_ATOL), np.abs(gl - rl).max()


def test_chunk_prefill_without_scores_and_without_k_rope_out():
    cfg = CFG1_SMALL
    _say(f"prefill only {cfg.name}")
    q, k, v = prefill_inputs(cfg)
    ref = _oracle_layer(cfg, q, k, v, rows=np.arange(0, cfg.seq_len, 7))
    shape = pc.make_shape(cfg.n_chunks, cfg.chunk_len, cfg.query_len, cfg.n_q_heads, cfg.n_kv_heads,
                          cfg.head_dim, cfg.obs_window, cfg.rope_base)
    o = torch.empty((cfg.n_chunks, cfg.seq_len, cfg.n_q_heads, cfg.head_dim), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((cfg.n_chunks, cfg.n_q_heads, cfg.seq_len), dtype=torch.float32, device="cuda")
    ws = pc.alloc_workspace(pc.pc_chunk_prefill_workspace_bytes(shape))
    pc.pc_chunk_prefill_attn(shape, bits_to_dev(q), bits_to_dev(k), bits_to_dev(v), o, lse, None, None, None, ws)
    torch.cuda.synchronize()
    assert_close(dev_bf16_to_f64(o)[:, ::7], ref["o"], O_ATOL, O_RTOL, "o")


def test_scores_obs_window_variants():
    """w_obs = 8 (the paper's appendix), smaller and larger windows, w_obs = w_q = 104 (Eq. 6 as
    printed: every query row votes) and a window reaching into the context (200 > w_q)."""
    cfg = CFG1_SMALL
    q, k, v = prefill_inputs(cfg)
    qf, kf = bf16_bits_to_f64(q), bf16_bits_to_f64(k)
    qd, kd = bits_to_dev(q), bits_to_dev(k)
    pos = np.arange(cfg.seq_len)
    for w_obs in (8, 1, 16, 64, cfg.query_len, 200):   # 1, 1, 2, 8, 13 and 25 blocks of 32 (row, head) columns
        _say(f"scores w_obs={w_obs}")
        shape = pc.make_shape(cfg.n_chunks, cfg.chunk_len, cfg.query_len, cfg.n_q_heads,
                              cfg.n_kv_heads, cfg.head_dim, w_obs, cfg.rope_base)
        ts = torch.empty((cfg.n_chunks, cfg.n_kv_heads, cfg.chunk_len), dtype=torch.float32, device="cuda")
        cs = torch.empty((cfg.n_chunks,), dtype=torch.float32, device="cuda")
        ws = pc.alloc_workspace(pc.pc_chunk_query_scores_workspace_bytes(shape))
        pc.pc_chunk_query_scores(shape, qd, kd, ts, cs, ws)
        torch.cuda.synchronize()
        for c in (0, cfg.n_chunks - 1):
            tok, chunk = oracle.query_scores(oracle.rope(qf[c], pos, cfg.rope_base),
                                             oracle.rope(kf[c], pos, cfg.rope_base),
                                             cfg.chunk_len, w_obs, cfg.n_kv_heads)
            assert_close(ts[c].cpu().numpy(), tok, S_ATOL, S_RTOL, f"tok_score w_obs={w_obs} c={c}")
            assert_close(cs[c].cpu().numpy(), chunk, S_ATOL, S_RTOL, f"chunk_score w_obs={w_obs}")
