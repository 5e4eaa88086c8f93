"""Pins of the CPU oracle against things other than itself: brute force in pure Python loops,
closed forms, a library attention routine, textbook identities and planted inputs whose
selections are known by construction.  Each test names the passage of the paper it pins."""
import math

import numpy as np
import pytest
import torch

import oracle
from workloads import (CFG0, CFG0U, CFG1_SMALL, CFG2_SMALL, prefill_inputs, bf16_bits_to_f64,
                       relevant_chunks, f32_to_bf16_bits, bf16_bits_to_f32, lm_logits_inputs)


def _rng(seed):
    return np.random.default_rng([7, seed])


# ------------------------------------------------------------------ RoPE (position reuse, sec. 3.1)
def test_rope_position_zero_is_identity():
    x = _rng(0).standard_normal((3, 2, 8))
    np.testing.assert_array_equal(oracle.rope(x, np.zeros(3, dtype=np.int64), 1e4), x)


def test_rope_pairing_and_sign_closed_form():
    # D = 4: pairs are (0, 2) with theta_0 = 1 and (1, 3) with theta_1 = base^(-1/2).
    base, p = 1.0e4, 3
    th1 = 1.0 / math.sqrt(base)
    e0 = np.zeros((1, 1, 4)); e0[0, 0, 0] = 1.0
    e1 = np.zeros((1, 1, 4)); e1[0, 0, 1] = 1.0
    e2 = np.zeros((1, 1, 4)); e2[0, 0, 2] = 1.0
    r0 = oracle.rope(e0, [p], base)[0, 0]
    r1 = oracle.rope(e1, [p], base)[0, 0]
    r2 = oracle.rope(e2, [p], base)[0, 0]
    np.testing.assert_allclose(r0, [math.cos(p), 0, math.sin(p), 0], atol=1e-15)
    np.testing.assert_allclose(r1, [0, math.cos(p * th1), 0, math.sin(p * th1)], atol=1e-15)
    np.testing.assert_allclose(r2, [-math.sin(p), 0, math.cos(p), 0], atol=1e-15)


def test_rope_frequency_formula():
    # theta_i = base^(-2i/D): D = 128, base 5e5 -> theta_32 = base^(-1/2).
    ang = oracle.rope_angles([1, 10], 128, 5.0e5)
    assert ang.shape == (2, 64)
    np.testing.assert_allclose(ang[0, 0], 1.0, rtol=0, atol=0)
    np.testing.assert_allclose(ang[0, 32], 1.0 / math.sqrt(5.0e5), rtol=1e-14)
    np.testing.assert_allclose(ang[1, 63], 10.0 * 5.0e5 ** (-126.0 / 128.0), rtol=1e-14)


def test_rope_preserves_norm_and_inner_product_depends_on_distance_only():
    r = _rng(1)
    x = r.standard_normal((5, 3, 16))
    pos = np.array([0, 1, 7, 100, 4095])
    y = oracle.rope(x, pos, 1e4)
    np.testing.assert_allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-13)
    a = r.standard_normal((1, 1, 16)); b = r.standard_normal((1, 1, 16))
    d1 = (oracle.rope(a, [9], 1e4) * oracle.rope(b, [4], 1e4)).sum()
    d2 = (oracle.rope(a, [1009], 1e4) * oracle.rope(b, [1004], 1e4)).sum()
    np.testing.assert_allclose(d1, d2, rtol=1e-10)


# ------------------------------------------------------------------ Eq. 1-2 local attention
def _brute_force_causal(q, k, v, scale):
    """Pure Python loops, explicit probabilities, no running max."""
    L, Hq, D = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    o = np.zeros((L, Hq, v.shape[2]))
    lse = np.zeros((L, Hq))
    P = np.zeros((L, Hq, L))
    for r in range(L):
        for h in range(Hq):
            g = h // G
            w = []
            for j in range(r + 1):
                dot = 0.0
                for d in range(D):
                    dot += q[r, h, d] * k[j, g, d]
                w.append(math.exp(dot * scale))
            z = sum(w)
            lse[r, h] = math.log(z)
            for j in range(r + 1):
                P[r, h, j] = w[j] / z
                for d in range(v.shape[2]):
                    o[r, h, d] += P[r, h, j] * v[j, g, d]
    return o, lse, P


def test_local_attention_vs_brute_force_gqa():
    r = _rng(2)
    L, Hq, Hkv, D = 11, 4, 2, 6
    q, k, v = r.standard_normal((L, Hq, D)), r.standard_normal((L, Hkv, D)), r.standard_normal((L, Hkv, D))
    scale = 0.37
    o, lse, P = oracle.local_attention(q, k, v, scale=scale, return_probs=True)
    ob, lb, Pb = _brute_force_causal(q, k, v, scale)
    np.testing.assert_allclose(o, ob, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse, lb, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(P, Pb, rtol=1e-12, atol=1e-15)
    # a subset of rows gives the same rows
    rows = np.array([0, 5, 10])
    o2, l2 = oracle.local_attention(q, k, v, scale=scale, rows=rows)
    np.testing.assert_allclose(o2, ob[rows], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(l2, lb[rows], rtol=1e-12, atol=1e-13)


def test_local_attention_default_scale_is_inverse_sqrt_head_dim():
    r = _rng(3)
    q, k, v = r.standard_normal((5, 1, 16)), r.standard_normal((5, 1, 16)), r.standard_normal((5, 1, 16))
    o1, l1 = oracle.local_attention(q, k, v)
    ob, lb, _ = _brute_force_causal(q, k, v, 0.25)
    np.testing.assert_allclose(o1, ob, rtol=1e-12)
    np.testing.assert_allclose(l1, lb, rtol=1e-12)


def test_local_attention_closed_forms():
    r = _rng(4)
    L, H, D = 9, 2, 4
    q = r.standard_normal((L, H, D))
    k = r.standard_normal((L, H, D))
    v = r.standard_normal((L, H, D))
    # rows of P sum to one and V == 1 gives o == 1
    o, _, P = oracle.local_attention(q, k, np.ones_like(v), return_probs=True)
    np.testing.assert_allclose(P.sum(-1), 1.0, rtol=1e-14)
    np.testing.assert_allclose(o, 1.0, rtol=1e-14)
    assert np.all(np.triu(np.ones((L, L)), 1)[:, None, :].repeat(H, 1) * P == 0.0)   # causal
    # K == 0: uniform over the causal prefix
    o, lse = oracle.local_attention(q, np.zeros_like(k), v)
    for row in range(L):
        np.testing.assert_allclose(o[row], v[:row + 1].mean(axis=0), rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(lse[row], math.log(row + 1), rtol=1e-13, atol=1e-15)


def test_invariant_one_chunk_no_eviction_is_standard_causal_rope_attention():
    """Invariant A: C = 1 without eviction is ordinary causal RoPE attention; checked against
    torch's scaled_dot_product_attention (a library routine) in fp64."""
    r = _rng(5)
    L, Hq, Hkv, D, base = 70, 4, 2, 16, 1e4
    q, k, v = r.standard_normal((1, L, Hq, D)), r.standard_normal((1, L, Hkv, D)), r.standard_normal((1, L, Hkv, D))
    out = oracle.parallelcomp_layer(q, k, v, chunk_len=L - 6, obs_window=3, keep_chunks=0,
                                    keep_tokens=0, rope_base=base)
    # library route: rotate with complex multiplication (independent of the oracle's RoPE code)
    def rot(x):
        half = D // 2
        th = base ** (-2.0 * np.arange(half) / D)
        z = (x[..., :half] + 1j * x[..., half:]) * np.exp(1j * np.arange(L)[:, None, None] * th)
        return np.concatenate([z.real, z.imag], axis=-1)
    tq = torch.from_numpy(rot(q[0])).permute(1, 0, 2)[None]
    tk = torch.from_numpy(rot(k[0])).permute(1, 0, 2)[None].repeat_interleave(Hq // Hkv, dim=1)
    tv = torch.from_numpy(v[0]).permute(1, 0, 2)[None].repeat_interleave(Hq // Hkv, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)
    ref = ref[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(out["o"][0], ref, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(out["k_rope"][0], rot(k[0]), rtol=1e-12, atol=1e-14)


def test_local_attention_shift_invariance_of_positions():
    r = _rng(6)
    L = 12
    q, k, v = r.standard_normal((L, 2, 8)), r.standard_normal((L, 2, 8)), r.standard_normal((L, 2, 8))
    pos = np.arange(L)
    o1, l1 = oracle.local_attention(oracle.rope(q, pos, 1e4), oracle.rope(k, pos, 1e4), v)
    o2, l2 = oracle.local_attention(oracle.rope(q, pos + 500, 1e4), oracle.rope(k, pos + 500, 1e4), v)
    np.testing.assert_allclose(o1, o2, rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(l1, l2, rtol=1e-9, atol=1e-11)


# ------------------------------------------------------------------ Eq. 5-6 cumulative scores
def test_query_scores_vs_brute_force_and_mass_conservation():
    r = _rng(7)
    L, w, Hq, Hkv, D, wobs = 14, 9, 4, 2, 6, 3
    q, k = r.standard_normal((L, Hq, D)), r.standard_normal((L, Hkv, D))
    scale = 0.41
    tok, chunk = oracle.query_scores(q, k, w, wobs, Hkv, scale=scale)
    _, _, P = _brute_force_causal(q, k, np.zeros((L, Hkv, 1)), scale)
    ref = np.zeros((Hkv, w))
    for h in range(Hq):
        for row in range(L - wobs, L):
            for j in range(w):
                ref[h // (Hq // Hkv), j] += P[row, h, j]
    np.testing.assert_allclose(tok, ref, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(chunk, ref.sum(), rtol=1e-12)
    # every voting row's probabilities sum to 1 over ALL keys: chunk mass + self mass = H_q * w_obs
    self_mass = P[L - wobs:, :, w:].sum()
    np.testing.assert_allclose(chunk + self_mass, Hq * wobs, rtol=1e-12)
    assert chunk < Hq * wobs


def test_query_scores_closed_form_zero_keys_and_single_voter():
    r = _rng(8)
    L, w, Hq, Hkv, D, wobs = 20, 13, 6, 2, 4, 5
    q = r.standard_normal((L, Hq, D))
    tok, chunk = oracle.query_scores(q, np.zeros((L, Hkv, D)), w, wobs, Hkv)
    expect = (Hq // Hkv) * sum(1.0 / (row + 1) for row in range(L - wobs, L))
    np.testing.assert_allclose(tok, expect, rtol=1e-13)
    np.testing.assert_allclose(chunk, expect * Hkv * w, rtol=1e-13)
    # w_obs = 1, MHA: the score is the last row of P
    k = r.standard_normal((L, Hq, D))
    tok1, _ = oracle.query_scores(q, k, w, 1, Hq, scale=0.5)
    _, _, P = _brute_force_causal(q, k, np.zeros((L, Hq, 1)), 0.5)
    np.testing.assert_allclose(tok1, P[L - 1, :, :w], rtol=1e-12)


# ------------------------------------------------------------------ Eq. 3-4 / Eq. 7 selection
def _brute_topk(score, k):
    return sorted(range(len(score)), key=lambda i: (-score[i], i))[:k]


def test_select_chunks_ties_rank_order_and_bruteforce():
    s = np.array([0.5, 2.0, 2.0, -1.0, 2.0, 0.5])
    np.testing.assert_array_equal(oracle.select_chunks(s, 2), [1, 2])
    np.testing.assert_array_equal(oracle.select_chunks(s, 4), [1, 2, 4, 0])
    np.testing.assert_array_equal(oracle.select_chunks(s, 6), [1, 2, 4, 0, 5, 3])
    r = _rng(9)
    for n in (1, 2, 7, 33):
        sc = np.round(r.standard_normal(n), 1)           # many ties
        for k in {1, n // 2 or 1, n}:
            np.testing.assert_array_equal(oracle.select_chunks(sc, k), _brute_topk(list(sc), k))


def test_select_tokens_ties_ascending_identity_and_permutation():
    s = np.array([[1.0, 3.0, 3.0, 0.0, 3.0, 1.0], [0.0, 0.0, 0.0, 0.0, 0.0, 0.0]])
    out = oracle.select_tokens(s, 2)
    np.testing.assert_array_equal(out, [[1, 2], [0, 1]])
    np.testing.assert_array_equal(oracle.select_tokens(s, 6), [list(range(6))] * 2)   # k = n
    r = _rng(10)
    sc = np.round(r.random((3, 4, 50)), 2)
    out = oracle.select_tokens(sc, 17)
    assert out.shape == (3, 4, 17) and out.dtype == np.int32
    for a in range(3):
        for b in range(4):
            assert list(out[a, b]) == sorted(_brute_topk(list(sc[a, b]), 17))
    # distinct scores: permuting the input permutes the answer
    x = r.permutation(40).astype(np.float64)
    perm = r.permutation(40)
    base = set(oracle.select_tokens(x[None], 9)[0])
    moved = set(perm[i] for i in oracle.select_tokens(x[perm][None], 9)[0])
    assert base == moved


# ------------------------------------------------------------------ Eq. 7 gather
def test_gather_is_a_pure_permutation():
    r = _rng(11)
    C, rows, H, D = 3, 10, 2, 4
    k = r.integers(0, 2 ** 16, size=(C, rows, H, D)).astype(np.uint16)
    v = r.integers(0, 2 ** 16, size=(C, rows, H, D)).astype(np.uint16)
    chunk_idx = np.array([2, 0])
    tok_idx = np.stack([np.stack([np.sort(r.choice(rows, 6, replace=False)) for _ in range(H)])
                        for _ in range(2)]).astype(np.int32)
    kd, vd = oracle.gather_kv(k, v, chunk_idx, tok_idx)
    assert kd.dtype == np.uint16 and kd.shape == (2, H, 6, D)
    for s in range(2):
        for g in range(H):
            for t in range(6):
                assert np.array_equal(kd[s, g, t], k[chunk_idx[s], tok_idx[s, g, t], g])
                assert np.array_equal(vd[s, g, t], v[chunk_idx[s], tok_idx[s, g, t], g])
    # k = rows with identity indices is the transpose [C, H, rows, D] of the source
    ident = np.broadcast_to(np.arange(rows, dtype=np.int32), (C, H, rows)).copy()
    kd, _ = oracle.gather_kv(k, v, np.arange(C), ident)
    np.testing.assert_array_equal(kd, k.transpose(0, 2, 1, 3))


# ------------------------------------------------------------------ Eq. 9-11 global attention
def test_invariant_merge_equals_one_softmax_over_concatenation():
    """Invariant B: per-segment softmaxes merged by logsumexp equal one softmax over all keys;
    the concatenated form is itself checked against torch's attention with an explicit mask."""
    r = _rng(12)
    nq, Hq, Hkv, D, S, kt = 7, 4, 2, 8, 3, 11
    q = r.standard_normal((nq, Hq, D))
    kc, vc = r.standard_normal((S, Hkv, kt, D)), r.standard_normal((S, Hkv, kt, D))
    ks, vs = r.standard_normal((nq, Hkv, D)), r.standard_normal((nq, Hkv, D))
    seg_len = np.array([11, 4, 9])
    o1, l1 = oracle.global_attention_concat(q, kc, vc, ks, vs, seg_len=seg_len, scale=0.3)
    o2, l2 = oracle.global_attention_merged(q, kc, vc, ks, vs, seg_len=seg_len, scale=0.3)
    np.testing.assert_allclose(o1, o2, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(l1, l2, rtol=1e-12, atol=1e-14)
    G = Hq // Hkv
    for h in range(Hq):
        g = h // G
        K = np.concatenate([kc[s, g, :seg_len[s]] for s in range(S)] + [ks[:, g]])
        V = np.concatenate([vc[s, g, :seg_len[s]] for s in range(S)] + [vs[:, g]])
        n_ctx = int(seg_len.sum())
        mask = np.ones((nq, n_ctx + nq), dtype=bool)
        mask[:, n_ctx:] = np.tril(np.ones((nq, nq), dtype=bool))
        ref = torch.nn.functional.scaled_dot_product_attention(
            torch.from_numpy(q[:, h])[None], torch.from_numpy(K)[None], torch.from_numpy(V)[None],
            attn_mask=torch.from_numpy(mask)[None], scale=0.3)[0].numpy()
        np.testing.assert_allclose(o1[:, h], ref, rtol=1e-10, atol=1e-12)


def test_merge_invariant_to_segment_order_and_splitting():
    r = _rng(13)
    nq, H, D, S, kt = 3, 2, 4, 4, 6
    q = r.standard_normal((nq, H, D))
    kc, vc = r.standard_normal((S, H, kt, D)), r.standard_normal((S, H, kt, D))
    o, l = oracle.global_attention_merged(q, kc, vc)
    perm = np.array([2, 0, 3, 1])
    o2, l2 = oracle.global_attention_merged(q, kc[perm], vc[perm])
    np.testing.assert_allclose(o, o2, rtol=1e-12)
    np.testing.assert_allclose(l, l2, rtol=1e-12)
    # split every segment in two halves: 2S segments of k_t/2
    kc3 = kc.reshape(S, H, 2, kt // 2, D).transpose(0, 2, 1, 3, 4).reshape(2 * S, H, kt // 2, D)
    vc3 = vc.reshape(S, H, 2, kt // 2, D).transpose(0, 2, 1, 3, 4).reshape(2 * S, H, kt // 2, D)
    o3, l3 = oracle.global_attention_merged(q, kc3, vc3)
    np.testing.assert_allclose(o, o3, rtol=1e-12)
    np.testing.assert_allclose(l, l3, rtol=1e-12)
    # one segment, no self segment: plain softmax attention
    o4, l4 = oracle.global_attention_merged(q[:1], kc[:1], vc[:1], scale=1.0)
    s = kc[0, 0] @ q[0, 0]
    p = np.exp(s) / np.exp(s).sum()
    np.testing.assert_allclose(o4[0, 0], p @ vc[0, 0], rtol=1e-12)
    np.testing.assert_allclose(l4[0, 0], math.log(np.exp(s).sum()), rtol=1e-12)


def test_lse_merge_closed_form():
    o, l = oracle.lse_merge(np.array([[1.0], [3.0]])[:, None, :], np.array([[0.0], [math.log(3.0)]]))
    np.testing.assert_allclose(o, [[2.5]], rtol=1e-15)            # (1*1 + 3*3) / 4
    np.testing.assert_allclose(l, [math.log(4.0)], rtol=1e-15)
    o, l = oracle.lse_merge(np.array([[[5.0]], [[7.0]]]), np.array([[-np.inf], [1.0]]))
    np.testing.assert_allclose(o, [[7.0]])
    np.testing.assert_allclose(l, [1.0])


def test_layer_keeping_everything_is_one_softmax_over_all_chunks():
    """Invariant B at layer level: k_c = C and k_t = w (nothing evicted) makes the global
    attention one softmax over all C*w context keys plus the causal query keys."""
    r = _rng(14)
    C, w, wq, Hq, Hkv, D, base = 3, 10, 4, 4, 2, 8, 1e4
    L = w + wq
    q = r.standard_normal((C, L, Hq, D))
    k = r.standard_normal((C, L, Hkv, D))
    v = r.standard_normal((C, L, Hkv, D))
    q[:, w:], k[:, w:], v[:, w:] = q[0, w:], k[0, w:], v[0, w:]    # same query rows everywhere
    out = oracle.parallelcomp_layer(q, k, v, w, 2, C, w, base)
    assert sorted(out["chunk_idx"]) == [0, 1, 2]
    np.testing.assert_array_equal(out["tok_idx"], np.broadcast_to(np.arange(w), (C, Hkv, w)))
    pos = np.arange(L)
    G = Hq // Hkv
    for h in range(Hq):
        g = h // G
        K = np.concatenate([oracle.rope(k[c], pos, base)[:w, g] for c in out["chunk_idx"]]
                           + [oracle.rope(k[0], pos, base)[w:, g]])
        V = np.concatenate([v[c, :w, g] for c in out["chunk_idx"]] + [v[0, w:, g]])
        qh = oracle.rope(q[0], pos, base)[w:, h]
        mask = np.ones((wq, C * w + wq), dtype=bool)
        mask[:, C * w:] = np.tril(np.ones((wq, wq), dtype=bool))
        ref = torch.nn.functional.scaled_dot_product_attention(
            torch.from_numpy(qh)[None], torch.from_numpy(K)[None], torch.from_numpy(V)[None],
            attn_mask=torch.from_numpy(mask)[None])[0].numpy()
        np.testing.assert_allclose(out["global_o"][:, h], ref, rtol=1e-10, atol=1e-12)


# ------------------------------------------------------------------ planted relevance
def test_planted_relevance_selects_known_chunks_and_tokens():
    """Chunks 1 and 3 carry keys aligned with the query (1 stronger than 3) at known token
    positions; everything else is tiny noise.  The first rotary pair (theta_0 = 1) is kept
    empty and the base is huge, so rotation is numerically the identity and the answer is
    known by construction."""
    r = _rng(15)
    C, w, wq, H, D, base = 5, 24, 4, 2, 8, 1e30
    L = w + wq
    u = np.array([0, 1, 0, 0, 0, 0, 1, 0], dtype=np.float64) / math.sqrt(2)
    q = 1e-3 * r.standard_normal((C, L, H, D))
    k = 1e-3 * r.standard_normal((C, L, H, D))
    v = r.standard_normal((C, L, H, D))
    q[..., 0] = q[..., 4] = k[..., 0] = k[..., 4] = 0.0
    q[:, w:] = 6.0 * u
    k[:, w:] = k[0, w:]; v[:, w:] = v[0, w:]
    strong, weak = [3, 7, 11, 20], [2, 5, 22]
    k[1, strong] += 3.0 * u
    k[3, weak] += 2.0 * u
    out = oracle.parallelcomp_layer(q, k, v, w, wq, 2, 4, base)
    np.testing.assert_array_equal(out["chunk_idx"], [1, 3])
    np.testing.assert_array_equal(out["tok_idx"][0], [strong] * H)
    assert all(set(weak) <= set(out["tok_idx"][1, g]) for g in range(H))
    assert out["chunk_score"][1] > out["chunk_score"][3] > out["chunk_score"][[0, 2, 4]].max()


# ------------------------------------------------------------------ Eq. 8 (attention calibration)
def test_calibrated_selection_vs_brute_force_and_special_cases():
    """Eq. 8 + Eq. 7: tokens of one position class with score above lambda are evicted, the
    best k of the rest are kept.  Brute force in plain loops; lambda = +inf or an empty class
    reduces to Eq. 7; lambda = -inf evicts the whole class."""
    r = _rng(31)
    w, k = 37, 9
    score = r.standard_normal((3, 2, w))
    score[0, 0, 5] = score[0, 0, 6] = score[0, 0, 30] = 0.25        # ties inside and outside the class
    score[1, 1, 3] = np.nan                                          # a NaN is not above lambda
    lam, lo, hi = 0.1, 2, 21
    idx, cnt = oracle.select_tokens_calibrated(score, k, lam, lo, hi)
    for a in range(3):
        for g in range(2):
            cand = []
            for j in range(w):
                x = score[a, g, j]
                if lo <= j < hi and x > lam:
                    continue
                cand.append((-(x if x == x else -math.inf), j))     # NaN ranks below everything
            cand.sort()
            want = sorted(j for _, j in cand[:k])
            assert cnt[a, g] == len(want) == min(k, len(cand))
            assert list(idx[a, g, :cnt[a, g]]) == want and all(idx[a, g, cnt[a, g]:] == -1)
    plain = oracle.select_tokens(score, k)
    for args in ((math.inf, lo, hi), (lam, 7, 7), (lam, w, w + 5)):
        idx2, cnt2 = oracle.select_tokens_calibrated(score, k, *args)
        np.testing.assert_array_equal(idx2, plain)
        assert (cnt2 == k).all()
    idx3, cnt3 = oracle.select_tokens_calibrated(score, 30, -math.inf, 10, 20)
    assert (cnt3 == 27).all() and (idx3[..., 27:] == -1).all()
    assert not np.isin(idx3[..., :27], np.arange(10, 20)).any()
    keep = np.r_[0:10, 20:w]
    np.testing.assert_array_equal(idx3[..., :27], np.broadcast_to(keep, (3, 2, 27)))   # k >= rest: all of it


def test_calibration_evicts_the_planted_sink_token():
    """Config 0 plants an attention sink (key 0 of every chunk has 4x the norm).  With
    unit-variance entries it collects the largest cumulative score of the first-100 class in most
    heads; a threshold between the largest and the second largest class score evicts exactly
    that token (R_s of the appendix), and the rest of the kept set is the plain top-k of the
    other tokens."""
    cfg = CFG0U
    qb, kb, vb = prefill_inputs(cfg)
    c = 1
    pos = np.arange(cfg.seq_len)
    q_rot = oracle.rope(bf16_bits_to_f64(qb[c]), pos, cfg.rope_base)
    k_rot = oracle.rope(bf16_bits_to_f64(kb[c]), pos, cfg.rope_base)
    tok, _ = oracle.query_scores(q_rot, k_rot, cfg.chunk_len, cfg.obs_window, cfg.n_kv_heads)
    n_sink_top = 0
    for g in range(cfg.n_kv_heads):
        cls = tok[g, :100]
        order = np.argsort(-cls)
        lam = 0.5 * (cls[order[0]] + cls[order[1]])
        idx, cnt = oracle.select_tokens_calibrated(tok[g], cfg.keep_tokens, lam, 0, 100)
        assert cnt == cfg.keep_tokens and order[0] not in idx
        rest = np.delete(np.arange(cfg.chunk_len), order[0])
        want = np.sort(rest[np.argsort(-tok[g, rest], kind="stable")[:cfg.keep_tokens]])
        np.testing.assert_array_equal(idx, want)
        n_sink_top += int(order[0] == 0)
    assert n_sink_top >= cfg.n_kv_heads // 2


def test_global_attention_with_per_head_lengths_ignores_padding():
    """Per-head segment lengths (what calibration produces): rows past a head's length carry no
    weight whatever they hold, the printed one-softmax form agrees with the merged form, and a
    head whose lengths equal those of a plain [S] vector gives the same numbers."""
    r = _rng(33)
    nq, Hq, Hkv, D, S, kt = 3, 4, 2, 8, 3, 6
    q = r.standard_normal((nq, Hq, D)); kc = r.standard_normal((S, Hkv, kt, D)); vc = r.standard_normal((S, Hkv, kt, D))
    ks = r.standard_normal((nq, Hkv, D)); vs = r.standard_normal((nq, Hkv, D))
    sl = np.array([[6, 2], [0, 5], [3, 3]])
    o1, l1 = oracle.global_attention_concat(q, kc, vc, ks, vs, seg_len=sl)
    o2, l2 = oracle.global_attention_merged(q, kc, vc, ks, vs, seg_len=sl)
    np.testing.assert_allclose(o1, o2, atol=1e-12); np.testing.assert_allclose(l1, l2, atol=1e-12)
    kc2, vc2 = kc.copy(), vc.copy()
    for s_ in range(S):
        for g in range(Hkv):
            kc2[s_, g, sl[s_, g]:] = 1e3; vc2[s_, g, sl[s_, g]:] = -7.0
    o3, l3 = oracle.global_attention_merged(q, kc2, vc2, ks, vs, seg_len=sl)
    np.testing.assert_array_equal(o2, o3); np.testing.assert_array_equal(l2, l3)
    o4, l4 = oracle.global_attention_concat(q, kc, vc, ks, vs, seg_len=sl[:, 0])
    np.testing.assert_allclose(o1[:, :2], o4[:, :2], atol=1e-13)     # heads of KV head 0


def test_gather_of_padded_ids_gives_zero_rows():
    r = _rng(34)
    src = r.standard_normal((2, 5, 1, 4)); val = r.standard_normal((2, 5, 1, 4))
    kd, vd = oracle.gather_kv(src, val, np.array([1]), np.array([[[0, 3, -1]]], dtype=np.int32))
    np.testing.assert_array_equal(kd[0, 0], [src[1, 0, 0], src[1, 3, 0], np.zeros(4)])
    np.testing.assert_array_equal(vd[0, 0, 2], np.zeros(4))


# ------------------------------------------------------------------ ragged chunks, streaming queue (sec. 3.1)
def test_ragged_chunks_reduce_to_uniform_chunks_of_their_own_length():
    """A chunk with fewer context rows is the same computation as a uniform layer whose chunk
    length is that chunk's length; rows behind the short sequence are padding that nothing reads."""
    r = _rng(41)
    C, w, wq, Hq, Hkv, D, base = 3, 20, 4, 4, 2, 8, 1e4
    lens = np.array([20, 13, 7])
    L = w + wq
    q = r.standard_normal((C, L, Hq, D)); k = r.standard_normal((C, L, Hkv, D)); v = r.standard_normal((C, L, Hkv, D))
    out = oracle.parallelcomp_layer(q, k, v, w, 3, 2, 5, base, chunk_lens=lens)
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    for c in range(C):
        q2[c, lens[c] + wq:] = 1e9; k2[c, lens[c] + wq:] = -1e9; v2[c, lens[c] + wq:] = 1e9
    out2 = oracle.parallelcomp_layer(q2, k2, v2, w, 3, 2, 5, base, chunk_lens=lens)
    for key in ("o", "lse", "tok_score", "chunk_score", "global_o", "tok_idx", "tok_cnt"):
        np.testing.assert_array_equal(out[key], out2[key])
    for c in range(C):
        Lc = lens[c] + wq
        one = oracle.parallelcomp_layer(q[c:c + 1, :Lc], k[c:c + 1, :Lc], v[c:c + 1, :Lc], int(lens[c]), 3, 0, 0, base)
        np.testing.assert_array_equal(out["o"][c, :Lc], one["o"][0])
        np.testing.assert_array_equal(out["tok_score"][c, :, :lens[c]], one["tok_score"][0])
        assert not out["tok_score"][c, :, lens[c]:].any() and not out["o"][c, Lc:].any()
        assert out["chunk_score"][c] == one["chunk_score"][0]
    # the shortest kept chunk has 7 tokens < 5? no: 7 >= 5, so every head keeps 5; with k = 9 it cannot
    out9 = oracle.parallelcomp_layer(q, k, v, w, 3, 3, 9, base, chunk_lens=lens)
    for s_, c in enumerate(out9["chunk_idx"]):
        assert (out9["tok_cnt"][s_] == min(9, lens[c])).all()
        assert (out9["tok_idx"][s_][:, :min(9, lens[c])] < lens[c]).all()


def test_streaming_priority_queue_equals_offline_top_k():
    """Chunks arrive in batches; a queue of fixed size keeps the best seen so far (score
    descending, earlier chunk first on ties).  Whatever the batch size, the final queue is the
    offline top-k of all chunk scores: the reason the method may free an evicted chunk's KV."""
    r = _rng(42)
    for trial in range(20):
        n, k = int(r.integers(5, 40)), int(r.integers(1, 6))
        score = np.round(r.standard_normal(n), 1)                 # many exact ties
        want = list(oracle.select_chunks(score, min(k, n)))
        for batch in (1, 2, 3, 7, n):
            queue = []                                            # (score, global chunk id)
            for c0 in range(0, n, batch):
                queue += [(score[c], c) for c in range(c0, min(c0 + batch, n))]
                queue.sort(key=lambda t: (-t[0], t[1]))
                queue = queue[:k]
                seen = min(c0 + batch, n)
                assert [c for _, c in queue] == list(oracle.select_chunks(score[:seen], min(k, seen)))
            assert [c for _, c in queue] == want


# ------------------------------------------------------------------ Eq. 3 (chunk self-information)
def test_self_information_brute_force_and_closed_forms():
    """I_c = -log P(X^q | X^c) by the chain rule over given logits: plain loops with math.exp /
    math.log; uniform logits give n_t log V; a constant added to a row changes nothing; raising
    the target logit by a over uniform logits gives log(V - 1 + e^a) - a per token; the
    probabilities exp(-nll) of all possible targets of a row sum to one."""
    r = _rng(51)
    C, T, V = 3, 4, 7
    logits = r.standard_normal((C, T, V)) * 3
    targets = r.integers(0, V, size=T)
    I, nll = oracle.chunk_self_information(logits, targets)
    for c in range(C):
        tot = 0.0
        for t in range(T):
            z = sum(math.exp(logits[c, t, v_]) for v_ in range(V))
            p = math.exp(logits[c, t, targets[t]]) / z
            assert abs(nll[c, t] + math.log(p)) < 1e-12
            tot -= math.log(p)
        assert abs(I[c] - tot) < 1e-11
    I0, _ = oracle.chunk_self_information(np.full((2, 5, 11), 0.37), np.arange(5))
    np.testing.assert_allclose(I0, 5 * math.log(11), rtol=1e-14)
    I1, _ = oracle.chunk_self_information(logits + r.standard_normal((C, T, 1)) * 50, targets)
    np.testing.assert_allclose(I1, I, rtol=1e-12)
    a = 2.5
    x = np.zeros((1, 3, 9)); x[0, np.arange(3), [4, 0, 8]] = a
    I2, _ = oracle.chunk_self_information(x, [4, 0, 8])
    np.testing.assert_allclose(I2, 3 * (math.log(8 + math.exp(a)) - a), rtol=1e-14)
    total = np.zeros((C, T))
    for v_ in range(V):
        _, n_v = oracle.chunk_self_information(logits, np.full(T, v_))
        total += np.exp(-n_v)
    np.testing.assert_allclose(total, 1.0, rtol=1e-12)
    big = np.array([[[1000.0, 999.0, -1000.0]]])                   # no overflow
    np.testing.assert_allclose(oracle.chunk_self_information(big, [1])[0], math.log(1 + math.exp(1.0)), rtol=1e-12)


def test_self_information_ranks_planted_chunks_first():
    """Synthetic logits in which the query is more predictable after chunks 1 and 4: Eq. 4 keeps
    the chunks of lowest self-information, i.e. the top-k of -I."""
    lb, targets = lm_logits_inputs(6, 24, 512, relevant=(4, 1))
    I, _ = oracle.chunk_self_information(bf16_bits_to_f64(lb), targets)
    assert sorted(oracle.select_chunks(-I, 2)) == [1, 4]
    assert I[[1, 4]].max() < I[[0, 2, 3, 5]].min()
    lb2, t2 = lm_logits_inputs(6, 24, 512, relevant=(4, 1))
    assert np.array_equal(lb, lb2) and np.array_equal(targets, t2)


# ------------------------------------------------------------------ decoding stage
def test_incremental_decode_equals_causal_attention_in_one_shot():
    """Generating token by token with a growing tail is the textbook KV-cache identity: step t
    equals row t of one causal attention whose self segment holds all generated tokens, with the
    compressed segments and the query block fully visible."""
    r = _rng(61)
    T, Hq, Hkv, D, S, kt, n0, base, p0 = 5, 4, 2, 8, 2, 6, 3, 1e4, 40
    qn = r.standard_normal((T, Hq, D)); kn = r.standard_normal((T, Hkv, D)); vn = r.standard_normal((T, Hkv, D))
    kc = r.standard_normal((S, Hkv, kt, D)); vc = r.standard_normal((S, Hkv, kt, D))
    k0 = r.standard_normal((n0, Hkv, D)); v0 = r.standard_normal((n0, Hkv, D))
    sl = np.array([6, 4])
    o, lse, (kt_, vt_) = oracle.decode_steps(qn, kn, vn, kc, vc, k0, v0, p0, base, seg_len=sl)
    pos = p0 + np.arange(T)
    q_rot, k_rot = oracle.rope(qn, pos, base), oracle.rope(kn, pos, base)
    kc2 = np.zeros((S + 1, Hkv, kt, D)); vc2 = np.zeros_like(kc2)
    kc2[:S] = kc; vc2[:S] = vc
    kc2[S, :, :n0] = k0.transpose(1, 0, 2); vc2[S, :, :n0] = v0.transpose(1, 0, 2)
    o2, lse2 = oracle.global_attention_concat(q_rot, kc2, vc2, k_rot, vn, seg_len=np.append(sl, n0))
    np.testing.assert_allclose(o, o2, atol=1e-13); np.testing.assert_allclose(lse, lse2, atol=1e-13)
    np.testing.assert_array_equal(kt_[:n0], k0); np.testing.assert_allclose(kt_[n0:], k_rot, atol=0)
    assert kt_.shape[0] == n0 + T and np.array_equal(vt_[n0:], vn)
    # a cache storage format is applied to the rotated key once, on entry, and to nothing else
    rnd = lambda x: bf16_bits_to_f64(f32_to_bf16_bits(np.asarray(x, dtype=np.float32)))
    o3, lse3, (kt3, vt3) = oracle.decode_steps(qn, kn, vn, kc, vc, k0, v0, p0, base, seg_len=sl, store=rnd)
    np.testing.assert_array_equal(kt3[n0:], rnd(k_rot)); np.testing.assert_array_equal(kt3[:n0], k0)
    np.testing.assert_array_equal(vt3, vt_)
    o4, lse4 = oracle.global_attention_concat(q_rot, kc2, vc2, rnd(k_rot), vn, seg_len=np.append(sl, n0))
    np.testing.assert_allclose(o3, o4, atol=1e-13); np.testing.assert_allclose(lse3, lse4, atol=1e-13)
    assert np.abs(o3 - o).max() > 1e-6                      # and it is not a no-op


# ------------------------------------------------------------------ 8-bit cache format
def test_fp8_e4m3_decode_closed_forms_and_library_view():
    d = oracle.fp8_e4m3_decode
    assert d([0x00])[0] == 0.0 and d([0x38])[0] == 1.0 and d([0xC0])[0] == -2.0
    assert d([0x01])[0] == 2.0 ** -9 and d([0x07])[0] == 7 * 2.0 ** -9       # subnormals
    assert d([0x08])[0] == 2.0 ** -6 and d([0x7E])[0] == 448.0                # min normal, max
    assert np.isnan(d([0x7F])[0]) and np.isnan(d([0xFF])[0])
    assert d([0x39])[0] == 1.125 and d([0x78])[0] == 256.0
    codes = np.arange(256, dtype=np.uint8)
    lib = torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    np.testing.assert_array_equal(d(codes), lib)                              # NaNs compare equal here
    mags = d(np.arange(0x7F, dtype=np.uint8))
    assert (np.diff(mags) > 0).all()                                          # code order = value order


def test_fp8_e4m3_published_format_constants():
    """tests/golden/e4m3_format_constants.txt: the characteristic values the format's
    specification prints (bit patterns and values)."""
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "e4m3_format_constants.txt")
    seen = 0
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        name, pattern, value = line.split()
        if pattern == "-":
            continue
        code = int(pattern.replace(".", ""), 2)
        got = oracle.fp8_e4m3_decode([code])[0]
        if value == "nan":
            assert np.isnan(got), name
        else:
            assert got == float(value) and np.signbit(got) == value.startswith("-"), (name, got)
            assert oracle.fp8_e4m3_encode([np.float32(value)])[0] == code, name
        seen += 1
    assert seen == 7
    finite = oracle.fp8_e4m3_decode(np.arange(256, dtype=np.uint8))
    assert np.isfinite(finite).sum() == 254 and not np.isinf(finite).any()      # no infinities, two NaNs


def test_fp8_e4m3_encode_round_trip_ties_saturation_and_library_conversion():
    enc, dec = oracle.fp8_e4m3_encode, oracle.fp8_e4m3_decode
    finite = np.array([c for c in range(256) if c & 0x7F != 0x7F], dtype=np.uint8)
    np.testing.assert_array_equal(enc(dec(finite).astype(np.float32)), finite)     # identity on the grid
    # ties: the midpoint of two neighbours goes to the even code; brute force in plain Python
    mags = [float(v) for v in dec(np.arange(0x7F, dtype=np.uint8))]
    for c in range(0x7E):
        mid = np.float32((mags[c] + mags[c + 1]) / 2)           # exact: one more mantissa bit
        assert float(mid) == (mags[c] + mags[c + 1]) / 2
        want = c if c % 2 == 0 else c + 1
        assert enc([mid])[0] == want and enc([-mid])[0] == (want | 0x80)
        below, above = np.nextafter(mid, np.float32(0)), np.nextafter(mid, np.float32(1e9))
        assert enc([below])[0] == c and enc([above])[0] == c + 1
    assert enc([1.0625])[0] == 0x38 and enc([1.1875])[0] == 0x3A              # worked ties
    assert enc([448.0])[0] == 0x7E and enc([463.9])[0] == 0x7E and enc([1e30])[0] == 0x7E
    assert enc([-1e30])[0] == 0xFE and enc([0.0])[0] == 0x00 and enc([-0.0])[0] == 0x80
    assert enc([2.0 ** -10])[0] == 0x00 and enc([1.5 * 2.0 ** -10])[0] == 0x01   # half the smallest: tie -> 0
    # a library conversion (round to nearest even) on every bf16 value inside the range and on
    # random float32 values
    with np.errstate(invalid="ignore"):                      # the NaN patterns are dropped below
        allb = bf16_bits_to_f64(np.arange(65536, dtype=np.uint16)).astype(np.float32)
    allb = allb[np.isfinite(allb) & (np.abs(allb) <= 448)]
    r = _rng(71)
    rnd = (r.standard_normal(100000) * r.choice([1e-3, 0.02, 1, 30, 200], 100000)).astype(np.float32).clip(-448, 448)
    for x in (allb, rnd):
        lib = torch.from_numpy(x.copy()).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        np.testing.assert_array_equal(enc(x), lib)


def test_quantize_kv_fp8_scale_padding_and_error_bound():
    r = _rng(72)
    S, H, kt, D = 3, 2, 40, 16
    kc = bf16_bits_to_f64(f32_to_bf16_bits(r.standard_normal((S, H, kt, D)).astype(np.float32) * 3))
    vc = bf16_bits_to_f64(f32_to_bf16_bits(r.standard_normal((S, H, kt, D)).astype(np.float32)))
    kc[1, 1] = 0.0                                              # an all-zero segment
    kc[0, 0, 35:] = 1e6                                         # huge values in rows nobody may read
    sl = np.array([[35, 40], [40, 40], [0, 7]])
    k8, ks, v8, vs = oracle.quantize_kv_fp8(kc, vc, sl)
    assert k8.dtype == np.uint8 and ks.dtype == np.float32 and ks.shape == (S, H)
    for s_ in range(S):
        for g in range(H):
            n = sl[s_, g]
            for x, c8, sc in ((kc, k8, ks), (vc, v8, vs)):
                assert (c8[s_, g, n:] == 0).all()                              # padding rows
                amax = np.abs(x[s_, g, :n]).max() if n else 0.0
                want = np.float32(amax) / np.float32(448) if amax > 0 else np.float32(1)
                assert sc[s_, g] == want
                if amax > 0:
                    top = np.unravel_index(np.abs(x[s_, g, :n]).argmax(), (n, D))
                    assert c8[s_, g][top] & 0x7F == 0x7E                      # the largest element is +-448
                dq = oracle.dequantize_kv_fp8(c8, sc)[s_, g, :n]
                err = np.abs(dq - x[s_, g, :n])
                # half a unit in the last place: 2^-4 relative for normals, scale * 2^-10 below them
                assert (err <= np.maximum(np.abs(x[s_, g, :n]) * 2.0 ** -4, float(sc[s_, g]) * 2.0 ** -10) * (1 + 1e-6)).all()
    assert (k8[1, 1] == 0).all() and ks[1, 1] == 1.0
    # uniform seg_len forms agree
    a = oracle.quantize_kv_fp8(kc[:, :, :30], vc[:, :, :30])
    b = oracle.quantize_kv_fp8(kc[:, :, :30], vc[:, :, :30], np.full(S, 30))
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)


def test_workload_plant_makes_relevant_chunks_win():
    """The unit-variance tiny config: the planted chunk must be the top chunk of the oracle."""
    cfg = CFG0U
    q, k, v = (bf16_bits_to_f64(x) for x in prefill_inputs(cfg))
    out = oracle.parallelcomp_layer(q, k, v, cfg.chunk_len, cfg.obs_window, cfg.keep_chunks,
                                    cfg.keep_tokens, cfg.rope_base, attn_rows=[0, cfg.seq_len - 1])
    assert out["chunk_idx"][0] == 2
    # the sink (key 0, 4x norm) is kept by every head of every kept chunk
    assert np.all(out["tok_idx"][:, :, 0] == 0)


# ------------------------------------------------------------------ generators
def test_bf16_rounding_is_nearest_even_and_exact_round_trip():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, -2.5, 0.0], dtype=np.float32)
    b = f32_to_bf16_bits(x)
    np.testing.assert_array_equal(bf16_bits_to_f32(b),
                                  np.array([1.0, 1.0, 1.0 + 2 ** -7, 1.0 + 2 ** -6, -2.5, 0.0], np.float32))
    t = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(b, t)
    y = _rng(16).standard_normal(1000).astype(np.float32)
    np.testing.assert_array_equal(f32_to_bf16_bits(y),
                                  torch.from_numpy(y).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))


def test_generators_are_seeded_and_structured():
    q1, k1, v1 = prefill_inputs(CFG1_SMALL)
    q2, k2, v2 = prefill_inputs(CFG1_SMALL, threads=1)
    assert np.array_equal(q1, q2) and np.array_equal(k1, k2) and np.array_equal(v1, v2)
    w = CFG1_SMALL.chunk_len
    assert np.array_equal(q1[0, w:], q1[3, w:]) and np.array_equal(k1[0, w:], k1[4, w:])
    kf = bf16_bits_to_f64(k1)
    nrm = np.linalg.norm(kf, axis=-1)
    assert np.all(nrm[:, 0] > 3.0 * np.median(nrm))                      # sink at key 0
    assert len(relevant_chunks(CFG1_SMALL)) == 2
    k2f = bf16_bits_to_f64(prefill_inputs(CFG2_SMALL)[1])
    n2 = np.linalg.norm(k2f, axis=-1)
    w2 = CFG2_SMALL.chunk_len
    assert np.median(n2[:, w2 - 64:w2]) > 1.7 * np.median(n2[:, :w2 - 64])   # recency bump
    np.testing.assert_allclose(np.std(np.log(n2[:, :w2 - 64])), 0.5, rtol=0.1)  # log-normal sigma


def test_chunk_queue_stream_equals_offline_top_k_of_every_prefix():
    """Sec. 3.1 "Chunk eviction": the streaming queue must hold, after every batch, exactly the
    offline top-k of the chunks seen so far (select_chunks on the prefix, itself pinned by brute
    force above), whatever the batch size; slots are a permutation-free bookkeeping: distinct,
    stable while a chunk stays, and entrants reuse only freed slots."""
    r = np.random.default_rng(77)
    for trial in range(30):
        C = int(r.integers(1, 40)); cap = int(r.integers(1, 12)); batch = int(r.integers(1, 9))
        score = r.integers(0, 6, size=C).astype(np.float64)          # heavy ties
        if trial % 3 == 0:
            score[r.integers(0, C, size=2)] = np.nan
        if trial % 5 == 0:
            score[r.integers(0, C)] = -np.inf
        steps = oracle.chunk_queue_stream(score, batch, cap)
        prev_slot = {}
        for i, (queue, slots, entrants) in enumerate(steps):
            seen = min((i + 1) * batch, C)
            # offline: a stable sort of the prefix by descending score, NaN last (plain Python)
            order = sorted(range(seen), key=lambda c: (np.isnan(score[c]), -np.nan_to_num(score[c], nan=0.0), c))
            assert queue == order[:cap]
            if not np.isnan(score[:seen]).any():
                assert queue == list(oracle.select_chunks(score[:seen], min(cap, seen)))
            assert len(set(slots)) == len(slots) and all(0 <= s < cap for s in slots)
            now = dict(zip(queue, slots))
            for c, s_ in now.items():
                if c in prev_slot:
                    assert prev_slot[c] == s_                        # a resident chunk never moves
            assert [c for c, _ in entrants] == [c for c in queue if c not in prev_slot]
            freed = sorted(set(range(cap)) - set(prev_slot[c] for c in prev_slot if c in now))
            assert [s_ for _, s_ in entrants] == freed[:len(entrants)]   # ascending free slots, in rank order
            prev_slot = now
    # a worked case: capacity 2, batches of 2, scores 5 1 | 7 5 | 0 9
    steps = oracle.chunk_queue_stream([5, 1, 7, 5, 0, 9], 2, 2)
    assert steps[0] == ([0, 1], [0, 1], [(0, 0), (1, 1)])
    assert steps[1] == ([2, 0], [1, 0], [(2, 1)])                     # 1 leaves, 2 takes its slot; tie 5 = 5: chunk 0 stays
    assert steps[2] == ([5, 2], [0, 1], [(5, 0)])
