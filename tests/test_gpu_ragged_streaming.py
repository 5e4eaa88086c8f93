"""GPU parity of ragged chunks (chunk_lens) and of the streaming chunk priority queue against the
fp64 CPU oracle, and of the streaming result against the all-chunks-at-once result."""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
import paper_2502_14317_amd as pc
from paper_2502_14317_amd.layer import ParallelCompLayer, StreamingParallelComp
from workloads import CFG1_SMALL, CFG2_SMALL, prefill_inputs, bf16_bits_to_f64
from helpers import (O_ATOL, O_RTOL, S_RTOL, S_ATOL, LSE_ATOL, bits_to_dev, dev_to_bits,
                     dev_bf16_to_f64, assert_close, assert_selection_matches)

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _ragged_inputs(cfg, lens):
    """The generator's chunks cut to lens[c] context rows, the query rows moved right behind them
    and the rest of every sequence filled with a finite pattern nothing may read."""
    q, k, v = prefill_inputs(cfg)
    w, wq = cfg.chunk_len, cfg.query_len
    out = []
    for x in (q, k, v):
        y = np.full_like(x, 0x4080)                 # bf16 4.0 everywhere, then the real rows
        for c, n in enumerate(lens):
            y[c, :n] = x[c, :n]
            y[c, n:n + wq] = x[c, w:]
        out.append(y)
    return out


@pytest.mark.parametrize("cfg,lens", [(CFG1_SMALL, [600, 600, 431, 256, 77]),
                                      (CFG2_SMALL, [459, 64, 459, 300, 1, 459]),
                                      # chunks of 0 and 1 tokens, every query row voting (w_obs = w_q,
                                      # Eq. 6 as printed): the voting window is the whole sequence of
                                      # an empty chunk
                                      (dataclasses.replace(CFG1_SMALL, obs_window=CFG1_SMALL.query_len),
                                       [600, 0, 1, 256, 77])],
                         ids=["cfg1_small", "cfg2_small", "cfg1_small_empty_chunks_all_rows_vote"])
def test_ragged_chunks_layer(cfg, lens):
    _say(f"ragged layer {cfg.name} lens={lens}")
    lens = np.array(lens, dtype=np.int32)
    q, k, v = _ragged_inputs(cfg, lens)
    qf, kf, vf = (bf16_bits_to_f64(x) for x in (q, k, v))
    ref = oracle.parallelcomp_layer(qf, kf, vf, cfg.chunk_len, cfg.obs_window, cfg.keep_chunks,
                                    cfg.keep_tokens, cfg.rope_base, chunk_lens=lens)
    layer = ParallelCompLayer(cfg.n_chunks, cfg.chunk_len, cfg.query_len, cfg.n_q_heads,
                              cfg.n_kv_heads, cfg.head_dim, cfg.obs_window, cfg.rope_base,
                              cfg.keep_chunks, cfg.keep_tokens)
    layer.o.fill_(7.0); layer.lse.fill_(7.0)
    qd, kd, vd = bits_to_dev(q), bits_to_dev(k), bits_to_dev(v)
    dlens = torch.from_numpy(lens).cuda()
    layer.forward(qd, kd, vd, chunk_lens=dlens, first_len=int(lens[0]))
    torch.cuda.synchronize()
    o, lse = dev_bf16_to_f64(layer.o), layer.lse.cpu().numpy().transpose(0, 2, 1)
    wq = cfg.query_len
    for c, n in enumerate(lens):
        Lc = n + wq
        assert_close(o[c, :Lc], ref["o"][c, :Lc], O_ATOL, O_RTOL, f"o[{c}]")
        assert_close(lse[c, :Lc], ref["lse"][c, :Lc], LSE_ATOL, 1e-3, f"lse[{c}]")
        assert (o[c, Lc:] == 7.0).all() and (lse[c, Lc:] == 7.0).all()      # padding rows untouched
        assert_close(dev_bf16_to_f64(layer.k_rope[c, :Lc]), ref["k_rope"][c, :Lc], 1e-5, 2.0 ** -8, f"k_rope[{c}]")
    ts = layer.tok_score.cpu().numpy()
    assert_close(ts, ref["tok_score"], S_ATOL, S_RTOL, "tok_score")
    for c, n in enumerate(lens):
        assert not ts[c, :, n:].any()
    assert_close(layer.chunk_score.cpu().numpy(), ref["chunk_score"], S_ATOL, S_RTOL, "chunk_score")
    # standalone score call == fused result, bit for bit
    ts2 = torch.empty_like(layer.tok_score); cs2 = torch.empty_like(layer.chunk_score)
    ws = pc.alloc_workspace(pc.pc_chunk_query_scores_workspace_bytes(layer.shape))
    pc.pc_chunk_query_scores(layer.shape, qd, kd, ts2, cs2, ws, chunk_lens=dlens)
    torch.cuda.synchronize()
    assert torch.equal(ts2, layer.tok_score) and torch.equal(cs2, layer.chunk_score)
    # selections: chunk set, per-head counts, token sets
    g_cidx = layer.chunk_idx.cpu().numpy()
    assert_selection_matches(g_cidx, ref["chunk_idx"], ref["chunk_score"], "chunk selection")
    g_tidx, g_cnt = layer.tok_idx.cpu().numpy(), layer.tok_cnt.cpu().numpy()
    vlen = np.repeat(lens[g_cidx][:, None], cfg.n_kv_heads, axis=1)
    ridx, rcnt = oracle.select_tokens_calibrated(ref["tok_score"][g_cidx], cfg.keep_tokens, np.inf, 0, 0, valid_len=vlen)
    assert np.array_equal(g_cnt, rcnt) and np.array_equal(g_cnt, np.minimum(cfg.keep_tokens, vlen))
    n_diff = 0
    for s_ in range(cfg.keep_chunks):
        for g in range(cfg.n_kv_heads):
            c_ = rcnt[s_, g]
            assert (g_tidx[s_, g, c_:] == -1).all() and (g_tidx[s_, g, :c_] < lens[g_cidx[s_]]).all()
            n_diff += assert_selection_matches(g_tidx[s_, g, :c_], ridx[s_, g, :c_],
                                               ref["tok_score"][g_cidx[s_], g], f"tokens {s_},{g}")
    _say(f"  kept counts {sorted(set(g_cnt.ravel().tolist()))}, differences inside the tie zone: {n_diff}")
    # global attention on the GPU's (valid) selection
    kc_ref, vc_ref = oracle.gather_kv(ref["k_rope"], vf, g_cidx, g_tidx)
    n0 = int(lens[0])
    og, lg = oracle.global_attention_concat(ref["q_rot_query"], kc_ref, vc_ref, ref["k_rope"][0, n0:n0 + wq],
                                            vf[0, n0:n0 + wq], seg_len=g_cnt)
    assert_close(dev_bf16_to_f64(layer.global_o[0]), og, O_ATOL, O_RTOL, "global_o")
    assert_close(layer.global_lse[0].cpu().numpy().T, lg, LSE_ATOL, 1e-3, "global_lse")


@pytest.mark.parametrize("cfg,batches", [(CFG1_SMALL, [1, 2, 3, 5]), (CFG2_SMALL, [4])],
                         ids=["cfg1_small", "cfg2_small"])
def test_streaming_queue_against_oracle(cfg, batches):
    """The streaming layer (device-side priority queue, sec. 3.1 "Chunk eviction") against the
    oracle: the queue and its slot table after every batch equal the oracle's streaming queue run
    on the oracle's own scores (checked wherever the oracle's ranking is not inside the tie zone of
    its scores), the per-slot token sets are valid selections of the oracle's scores, the
    compacted KV is a bit-exact gather, and the global attention output equals the oracle's
    evaluated on the selection the GPU made; also the streaming result equals the GPU's own
    all-chunks-at-once result."""
    _say(f"streaming {cfg.name} batches={batches}")
    q, k, v = prefill_inputs(cfg)
    qd, kd, vd = bits_to_dev(q), bits_to_dev(k), bits_to_dev(v)
    args = (cfg.chunk_len, cfg.query_len, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
            cfg.obs_window, cfg.rope_base, cfg.keep_chunks, cfg.keep_tokens)
    off = ParallelCompLayer(cfg.n_chunks, *args)
    off.forward(qd, kd, vd)
    torch.cuda.synchronize()
    off_cidx = off.chunk_idx.cpu().numpy()
    off_tidx = {int(c): off.tok_idx[s_].cpu().numpy() for s_, c in enumerate(off_cidx)}
    off_scores = off.chunk_score.cpu().numpy()
    qf, kf, vf = (bf16_bits_to_f64(x) for x in (q, k, v))
    ref = oracle.parallelcomp_layer(qf, kf, vf, cfg.chunk_len, cfg.obs_window, cfg.keep_chunks,
                                    cfg.keep_tokens, cfg.rope_base,
                                    attn_rows=np.arange(cfg.chunk_len, cfg.seq_len))
    w = cfg.chunk_len
    for bc in batches:
        st = StreamingParallelComp(cfg.n_chunks, bc, *args)
        seen = []
        st.forward(qd, kd, vd, after_batch=lambda c0, nb: seen.append(
            (st.queue_id.cpu().numpy().copy(), st.queue_slot.cpu().numpy().copy(), st.slot_src.cpu().numpy().copy())))
        torch.cuda.synchronize()
        out = st.global_o
        # the queue after every batch against the oracle's queue on the oracle's scores
        steps = oracle.chunk_queue_stream(ref["chunk_score"], bc, cfg.keep_chunks)
        assert len(seen) == len(steps)
        for i, ((g_id, g_slot, g_src), (r_id, r_slot, r_ent)) in enumerate(zip(seen, steps)):
            n = len(r_id)
            assert (g_id[n:] == -1).all()
            n_seen = min((i + 1) * bc, cfg.n_chunks)
            assert_selection_matches(g_id[:n], r_id, ref["chunk_score"][:n_seen], f"queue after batch {i}")
            assert len(set(g_slot[:n].tolist())) == n and (g_slot[:n] >= 0).all() and (g_slot[:n] < cfg.keep_chunks).all()
            if list(g_id[:n]) == r_id:
                assert list(g_slot[:n]) == r_slot, (i, g_slot, r_slot)
                want = np.full(cfg.keep_chunks, -1)
                for c, s_ in r_ent:
                    want[s_] = c - i * bc
                assert np.array_equal(g_src, want), (i, g_src, want)
        # the same scores bit for bit as the all-at-once layer, hence the same final queue
        assert np.array_equal(st.chunk_score.cpu().numpy(), off_scores)
        g_id, g_slot = st.queue_id.cpu().numpy(), st.queue_slot.cpu().numpy()
        assert np.array_equal(g_id, off_cidx)
        assert np.array_equal(st.queue_score.cpu().numpy(), off.chunk_top.cpu().numpy())
        slot_of = {int(c): int(s_) for c, s_ in zip(g_id, g_slot)}
        g_tidx = st.tok_idx.cpu().numpy()
        for c, slot in slot_of.items():
            assert np.array_equal(g_tidx[slot], off_tidx[c])
            s_off = list(off_cidx).index(c)
            assert torch.equal(st.kc[0, slot], off.kc[0, s_off]) and torch.equal(st.vc[0, slot], off.vc[0, s_off])
            for g in range(cfg.n_kv_heads):                  # a valid selection of the oracle's scores
                r_t = oracle.select_tokens(ref["tok_score"][c], cfg.keep_tokens)
                assert_selection_matches(g_tidx[slot, g], r_t[g], ref["tok_score"][c, g], f"tokens of chunk {c} head {g}")
        # global attention: segment order differs (slots), the value does not beyond rounding
        assert_close(dev_bf16_to_f64(out[0]), dev_bf16_to_f64(off.global_o[0]), 4e-3, 8e-3, f"stream vs offline bc={bc}")
        # against the oracle, unconditionally: Eq. 9-11 on the selection the GPU made (slot order)
        by_slot = sorted(slot_of, key=lambda c: slot_of[c])
        kc_ref, vc_ref = oracle.gather_kv(ref["k_rope"], vf, np.array(by_slot), g_tidx)
        og, lg = oracle.global_attention_concat(ref["q_rot_query"], kc_ref, vc_ref, ref["k_rope"][0, w:], vf[0, w:])
        assert_close(dev_bf16_to_f64(out[0]), og, O_ATOL, O_RTOL, f"stream vs oracle bc={bc}")
        assert_close(st.global_lse[0].cpu().numpy().T, lg, LSE_ATOL, 1e-3, f"stream lse vs oracle bc={bc}")


def test_chunk_queue_update_ties_nan_and_slot_reuse():
    """pc_chunk_queue_update alone on crafted scores (heavy ties, NaN, -inf, more slots than chunks)
    against the oracle's queue, bit-exact: ids, scores, slots and entrants after every batch."""
    r = np.random.default_rng(78)
    cases = [(np.array([5, 1, 7, 5, 0, 9], dtype=np.float32), 2, 2)]
    for trial in range(12):
        C, cap, bc = int(r.integers(1, 60)), int(r.integers(1, 14)), int(r.integers(1, 11))
        sc = r.integers(0, 5, size=C).astype(np.float32)
        if trial % 2 == 0:
            sc[r.integers(0, C, size=3)] = np.nan
        if trial % 3 == 0:
            sc[r.integers(0, C)] = -np.inf
        cases.append((sc, bc, cap))
    cases.append((r.standard_normal(3000).astype(np.float32), 1024, 1024))      # the limits
    for sc, bc, cap in cases:
        C = sc.shape[0]
        steps = oracle.chunk_queue_stream(sc.astype(np.float64), bc, cap)
        dsc = torch.from_numpy(sc).cuda()
        qid = torch.full((cap,), -1, dtype=torch.int32, device="cuda")
        qsc = torch.zeros((cap,), dtype=torch.float32, device="cuda")
        qsl = torch.zeros((cap,), dtype=torch.int32, device="cuda")
        src = torch.zeros((cap,), dtype=torch.int32, device="cuda")
        for i, (r_id, r_slot, r_ent) in enumerate(steps):
            c0, nb = i * bc, min(bc, C - i * bc)
            pc.pc_chunk_queue_update(dsc[c0:c0 + nb], nb, c0, cap, qid, qsc, qsl, src)
            torch.cuda.synchronize()
            n = len(r_id)
            g_id, g_sl, g_src = qid.cpu().numpy(), qsl.cpu().numpy(), src.cpu().numpy()
            assert list(g_id[:n]) == r_id and (g_id[n:] == -1).all(), (i, g_id, r_id)
            assert list(g_sl[:n]) == r_slot
            assert np.array_equal(qsc.cpu().numpy()[:n].view(np.uint32), sc[r_id].view(np.uint32))
            want = np.full(cap, -1)
            for c, s_ in r_ent:
                want[s_] = c - c0
            assert np.array_equal(g_src, want)


def test_negative_chunk_index_skips_selection_and_gather():
    """chunk_idx[s] < 0 (a queue slot with no entrant): the token selection and the gather leave
    that entry's outputs untouched; the other entries are processed as usual."""
    r = np.random.default_rng(79)
    C, Hkv, w, k, D, rows = 3, 2, 300, 40, 64, 320
    ts = torch.from_numpy(r.random((C, Hkv, w), dtype=np.float32)).cuda()
    cidx = torch.tensor([2, -1, 0], dtype=torch.int32, device="cuda")
    out = torch.full((3, Hkv, k), -7, dtype=torch.int32, device="cuda")
    pc.pc_select_tokens_topk(ts, cidx, 3, Hkv, w, k, out)
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    assert (o[1] == -7).all()
    ref = oracle.select_tokens(ts.cpu().numpy()[[2, 0]], k)
    assert np.array_equal(o[0], ref[0]) and np.array_equal(o[2], ref[1])
    ks = torch.from_numpy(r.integers(0, 65536, size=(1, C, rows, Hkv, D)).astype(np.uint16).view(np.int16)).cuda().view(torch.bfloat16)
    vs = ks.flip(2).contiguous()
    kd = torch.full((1, 3, Hkv, k, D), 9.0, dtype=torch.bfloat16, device="cuda")
    vd = torch.full_like(kd, 9.0)
    out[1] = 0
    pc.pc_gather_kv(ks, vs, cidx.view(1, 3), out, 1, C, rows, 3, Hkv, k, D, kd, vd)
    torch.cuda.synchronize()
    assert (kd[0, 1] == 9.0).all() and (vd[0, 1] == 9.0).all()
    rk, rv = oracle.gather_kv(dev_to_bits(ks[0]), dev_to_bits(vs[0]), np.array([2, 0]), o[[0, 2]])
    assert np.array_equal(dev_to_bits(kd[0, [0, 2]]), rk) and np.array_equal(dev_to_bits(vd[0, [0, 2]]), rv)
