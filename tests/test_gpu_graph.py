"""The whole layer step and a decode step recorded into a HIP graph (through torch's graph
capture, which records what the library enqueues on the capturing stream) and replayed: every
replay must reproduce the eager result bit for bit, with eager work and synchronisations between
the replays and with new contents in the (static) input buffers."""
import numpy as np
import pytest
import torch

import paper_2502_14317_amd as pc
from paper_2502_14317_amd.layer import ParallelCompLayer, DecodeCache
from workloads import CFG1_SMALL, prefill_inputs, f32_to_bf16_bits
from helpers import bits_to_dev

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _layer(cfg):
    return ParallelCompLayer(cfg.n_chunks, cfg.chunk_len, cfg.query_len, cfg.n_q_heads, cfg.n_kv_heads,
                             cfg.head_dim, cfg.obs_window, cfg.rope_base, cfg.keep_chunks, cfg.keep_tokens)


def test_layer_step_in_a_hip_graph():
    cfg = CFG1_SMALL
    _say(f"graph replay of the layer step, {cfg.name}")
    q, k, v = (bits_to_dev(x) for x in prefill_inputs(cfg))
    eager, graphed = _layer(cfg), _layer(cfg)
    graphed.forward(q, k, v)                     # warm-up outside the capture (function attributes, lazy init)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        graphed.forward(q, k, v)
    r = np.random.default_rng(31)
    for rep in range(4):
        if rep:                                   # new contents in the static input buffers
            q.copy_(bits_to_dev(f32_to_bf16_bits(r.standard_normal(tuple(q.shape)).astype(np.float32) * 0.1)))
            k[:, :, :, ::2] *= -1
        graphed.global_o.fill_(0); graphed.o.fill_(0); graphed.tok_idx.fill_(-7)
        g.replay()
        eager.forward(q, k, v)                    # the program's own eager work between replays
        torch.cuda.synchronize()
        for name in ("o", "lse", "k_rope", "tok_score", "chunk_score", "chunk_idx", "tok_idx", "kc", "vc",
                     "global_o", "global_lse"):
            assert torch.equal(getattr(graphed, name), getattr(eager, name)), (rep, name)


def test_decode_step_in_a_hip_graph():
    Bn, S, kt, Hq, Hkv, D, n0 = 2, 3, 160, 8, 2, 128, 20
    _say("graph replay of a decode step")
    gen = torch.Generator(device="cuda").manual_seed(9)
    bf = torch.bfloat16
    mk = lambda *shape: torch.randn(shape, generator=gen, device="cuda").to(bf)
    kc, vc, k0, v0 = mk(Bn, S, Hkv, kt, D), mk(Bn, S, Hkv, kt, D), mk(Bn, n0, Hkv, D), mk(Bn, n0, Hkv, D)
    qn, kn, vn = mk(Bn, 1, Hq, D), mk(Bn, 1, Hkv, D), mk(Bn, 1, Hkv, D)
    eager, graphed = DecodeCache(Bn, S, kt, Hq, Hkv, D, 5.0e5), DecodeCache(Bn, S, kt, Hq, Hkv, D, 5.0e5)
    for c in (eager, graphed):
        c.load(kc, vc, None, k0, v0)
    graphed.step(qn, kn, vn, 700)                 # warm-up; both caches advance in lockstep
    eager.step(qn, kn, vn, 700)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        graphed.step(qn, kn, vn, 701)             # the position is recorded with the graph
    eager.step(qn, kn, vn, 701)                   # capture does not execute: eager catches up below
    g.replay()
    torch.cuda.synchronize()
    assert torch.equal(graphed.out, eager.out) and torch.equal(graphed.seg_len, eager.seg_len)
    for rep in range(3):                          # same position again: the tail keeps growing
        qn.copy_(mk(Bn, 1, Hq, D)); kn.copy_(mk(Bn, 1, Hkv, D))
        g.replay()
        eager.step(qn, kn, vn, 701)
        torch.cuda.synchronize()
        assert torch.equal(graphed.out, eager.out) and torch.equal(graphed.lse, eager.lse), rep
        assert torch.equal(graphed.seg_len, eager.seg_len) and torch.equal(graphed.kc, eager.kc)
