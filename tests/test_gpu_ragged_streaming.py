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
def test_streaming_queue_equals_offline_selection(cfg, batches):
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
    ref = oracle.parallelcomp_layer(*(bf16_bits_to_f64(x) for x in (q, k, v)), cfg.chunk_len, cfg.obs_window,
                                    cfg.keep_chunks, cfg.keep_tokens, cfg.rope_base,
                                    attn_rows=np.arange(cfg.chunk_len, cfg.seq_len))
    for bc in batches:
        st = StreamingParallelComp(cfg.n_chunks, bc, *args)
        out = st.forward(qd, kd, vd)
        torch.cuda.synchronize()
        # the same scores bit for bit, hence the same queue as the offline top-k, in rank order
        assert np.array_equal(st.chunk_score.cpu().numpy(), off_scores)
        assert np.array_equal(st.chunk_idx.cpu().numpy(), off_cidx)
        assert sorted(st.slot_of) == sorted(int(c) for c in off_cidx)
        for c, slot in st.slot_of.items():
            assert np.array_equal(st.tok_idx[slot].cpu().numpy(), off_tidx[c])
            s_off = list(off_cidx).index(c)
            assert torch.equal(st.kc[0, slot], off.kc[0, s_off]) and torch.equal(st.vc[0, slot], off.vc[0, s_off])
        # global attention: segment order differs (slots), the value does not beyond rounding
        assert_close(dev_bf16_to_f64(out[0]), dev_bf16_to_f64(off.global_o[0]), 4e-3, 8e-3, f"stream vs offline bc={bc}")
        if list(off_cidx) == list(ref["chunk_idx"]) and np.array_equal(off.tok_idx.cpu().numpy(), ref["tok_idx"]):
            assert_close(dev_bf16_to_f64(out[0]), ref["global_o"], O_ATOL, O_RTOL, f"stream vs oracle bc={bc}")
