"""GPU parity of the 8-bit (E4M3) compressed cache: codes and scales bit-exact against the CPU
oracle's encoder, attention over the 8-bit segments (+ a 16-bit tail) against the oracle's
attention on the dequantised values."""
import numpy as np
import pytest
import torch

import oracle
import paper_2502_14317_amd as pc
from paper_2502_14317_amd.layer import fp8_alloc
from workloads import CFG4, f32_to_bf16_bits, bf16_bits_to_f64
from helpers import (O_ATOL, O_RTOL, LSE_ATOL, bits_to_dev, dev_to_bits, dev_bf16_to_f64, assert_close,
                     fp8_rows_view, fp8_from_rows)

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _mk(r, shape, s=1.0):
    return f32_to_bf16_bits((r.standard_normal(shape) * s).astype(np.float32))


def _quantize(kc_bits, vc_bits, seg_len, per_head):
    B, S, Hkv, kt, D = kc_bits.shape
    k8 = fp8_alloc(B, S, Hkv, kt, D).fill_(0x55)              # codes: 32-key blocks in matrix-core order
    v8 = fp8_alloc(B, S, Hkv, kt, D).fill_(0x55)
    ks = torch.empty((B, S, Hkv), dtype=torch.float32, device="cuda")
    vs = torch.empty_like(ks)
    pc.pc_kv_quantize_fp8(bits_to_dev(kc_bits), bits_to_dev(vc_bits),
                          None if seg_len is None else torch.from_numpy(seg_len).cuda(), B, S, kt, Hkv, D,
                          k8, v8, ks, vs, seg_len_per_head=per_head)
    torch.cuda.synchronize()
    # keys behind k_t in the last block must be written too (code 0): the attention kernel reads whole blocks
    for which, c8 in (("k", k8), ("v", v8)):
        assert (fp8_rows_view(which, c8, kt, D, padded=True)[..., kt:, :] == 0).all(), "codes behind k_t are not zero"
    return k8, v8, ks, vs


def test_quantize_every_bf16_value_bit_exact():
    """Scale exactly 1 (the segment's maximum is 448): the codes of all bf16 values of magnitude
    <= 448 must be the oracle's, which pins rounding, ties, subnormals and signs."""
    _say("fp8 quantize: all bf16 values")
    allb = np.arange(65536, dtype=np.uint16)
    with np.errstate(invalid="ignore"):                      # the NaN patterns are dropped below
        f = bf16_bits_to_f64(allb)
    allb = allb[np.isfinite(f) & (np.abs(f) <= 448)]
    D = 128
    kt = (allb.size + D - 1) // D
    bits = np.zeros((1, 1, 1, kt, D), dtype=np.uint16)
    bits.reshape(-1)[:allb.size] = allb
    k8, v8, ks, vs = _quantize(bits, bits[:, :, :, ::-1].copy(), None, 0)
    rk8, rks, rv8, rvs = oracle.quantize_kv_fp8(bf16_bits_to_f64(bits[0]), bf16_bits_to_f64(bits[0, :, :, ::-1]))
    assert ks.item() == 1.0 and vs.item() == 1.0 and rks[0, 0] == 1.0
    np.testing.assert_array_equal(fp8_rows_view("k", k8, kt, D).cpu().numpy()[0], rk8)
    np.testing.assert_array_equal(fp8_rows_view("v", v8, kt, D).cpu().numpy()[0], rv8)


@pytest.mark.parametrize("D,per_head", [(128, 0), (64, 1)])
def test_quantize_random_segments_bit_exact(D, per_head):
    _say(f"fp8 quantize: random segments D={D} per_head={per_head}")
    r = np.random.default_rng([51, D])
    B, S, Hkv, kt = 2, 3, 2, 100
    kc, vc = _mk(r, (B, S, Hkv, kt, D), 2.5), _mk(r, (B, S, Hkv, kt, D), 0.3)
    kc[0, 0, 0, 5] = f32_to_bf16_bits(np.full(D, 37.0, dtype=np.float32))      # an outlier row (sink-like)
    kc[1, 2, 1] = 0                                                            # an all-zero segment
    sl = r.integers(0, kt + 1, size=(B, S, Hkv) if per_head else (B, S)).astype(np.int32)
    sl[0, 0] = kt
    k8, v8, ks, vs = _quantize(kc, vc, sl, per_head)
    for b in range(B):
        rk8, rks, rv8, rvs = oracle.quantize_kv_fp8(bf16_bits_to_f64(kc[b]), bf16_bits_to_f64(vc[b]), sl[b])
        np.testing.assert_array_equal(ks[b].cpu().numpy(), rks)
        np.testing.assert_array_equal(vs[b].cpu().numpy(), rvs)
        np.testing.assert_array_equal(fp8_rows_view("k", k8[b], kt, D).cpu().numpy(), rk8)
        np.testing.assert_array_equal(fp8_rows_view("v", v8[b], kt, D).cpu().numpy(), rv8)


def _attn_case(name, B, n_q, S, kt, Hq, Hkv, D, tail_cap, q_pos0, ragged, seed, with_self=False):
    _say(f"fp8 attention {name}: B={B} n_q={n_q} S={S} kt={kt} H={Hq}/{Hkv} D={D} tail={tail_cap} ragged={ragged} self={with_self}")
    r = np.random.default_rng([52, seed])
    q = _mk(r, (B, n_q, Hq, D), 3.0)
    kc, vc = _mk(r, (B, S, Hkv, kt, D)), _mk(r, (B, S, Hkv, kt, D))
    sl = r.integers(0, kt + 1, size=(B, S)).astype(np.int32) if ragged else None
    if ragged:
        sl[0, 0] = kt
    k8, v8, ks, vs = _quantize(kc, vc, sl, 0)
    kt_bits = vt_bits = tl = None
    if tail_cap:
        kt_bits, vt_bits = _mk(r, (B, 1, Hkv, tail_cap, D)), _mk(r, (B, 1, Hkv, tail_cap, D))
        tl = r.integers(1, tail_cap + 1, size=(B,)).astype(np.int32)
    ks_bits = vs_bits = None
    if with_self:
        ks_bits, vs_bits = _mk(r, (B, n_q, Hkv, D)), _mk(r, (B, n_q, Hkv, D))
    out = torch.full((B, n_q, Hq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full((B, Hq, n_q), float("nan"), dtype=torch.float32, device="cuda")
    ws = pc.alloc_workspace(pc.pc_parallel_attn_fp8_workspace_bytes(B, n_q, S, kt, tail_cap, Hq, Hkv, D, with_self))
    pc.pc_parallel_attn_fp8(bits_to_dev(q), k8, v8, ks, vs, None if sl is None else torch.from_numpy(sl).cuda(),
                            bits_to_dev(kt_bits) if tail_cap else None, bits_to_dev(vt_bits) if tail_cap else None,
                            torch.from_numpy(tl).cuda() if tail_cap else None, tail_cap, B, n_q, S, kt, Hq, Hkv, D,
                            q_pos0, 1.0e4, 0.0, out, lse, ws,
                            k_self=bits_to_dev(ks_bits) if with_self else None,
                            v_self=bits_to_dev(vs_bits) if with_self else None)
    torch.cuda.synchronize()
    for b in range(B):
        # the oracle quantises on its own (bit-equal to the GPU's codes, tested above) and attends
        # over its dequantised values
        rk8, rks, rv8, rvs = oracle.quantize_kv_fp8(bf16_bits_to_f64(kc[b]), bf16_bits_to_f64(vc[b]),
                                                    None if sl is None else sl[b])
        kd, vd = oracle.dequantize_kv_fp8(rk8, rks), oracle.dequantize_kv_fp8(rv8, rvs)
        seg_len = np.full(S, kt) if sl is None else sl[b].astype(np.int64)
        if tail_cap:
            pad = max(kt, tail_cap)
            K = np.zeros((S + 1, Hkv, pad, D)); V = np.zeros_like(K)
            K[:S, :, :kt] = kd; V[:S, :, :kt] = vd
            K[S, :, :tail_cap] = bf16_bits_to_f64(kt_bits[b, 0]); V[S, :, :tail_cap] = bf16_bits_to_f64(vt_bits[b, 0])
            kd, vd, seg_len = K, V, np.append(seg_len, tl[b])
        qf = bf16_bits_to_f64(q[b])
        if q_pos0 >= 0:
            qf = oracle.rope(qf, q_pos0 + np.arange(n_q), 1.0e4)
        ro, rl = oracle.global_attention_concat(qf, kd, vd, seg_len=seg_len,
                                                k_self=bf16_bits_to_f64(ks_bits[b]) if with_self else None,
                                                v_self=bf16_bits_to_f64(vs_bits[b]) if with_self else None)
        assert_close(dev_bf16_to_f64(out[b]), ro, O_ATOL, O_RTOL, f"{name} out[b={b}]")
        assert_close(lse[b].cpu().numpy().T, rl, LSE_ATOL, 1e-3, f"{name} lse[b={b}]")


def test_fp8_attention_gqa_with_tail():
    _attn_case("gqa-tail", 2, 1, 4, 1100, 8, 2, 128, 70, 4000, True, 1)


def test_fp8_attention_mha64_and_two_rows():
    _attn_case("mha64", 3, 1, 3, 333, 4, 4, 64, 0, -1, True, 2)
    _attn_case("nq2-g4", 1, 2, 2, 2048, 8, 2, 128, 1500, -1, False, 3)
    _attn_case("nq4-g4", 2, 4, 3, 300, 8, 2, 128, 64, 9, True, 6)            # 16 query columns
    _attn_case("tail-only", 2, 1, 0, 64, 4, 2, 64, 40, 7, False, 4)


def test_fp8_decode_steps_match_oracle():
    """The decode loop on the 8-bit cache: segments quantised at load, bf16 tail grown on the
    device; against the oracle's decode_steps over its own dequantised segments."""
    from paper_2502_14317_amd.layer import DecodeCacheFp8
    Bn, S, kt, Hq, Hkv, D, n0, T, base, pos0, cap = 2, 3, 160, 8, 2, 128, 37, 7, 5.0e5, 700, 64
    _say(f"fp8 decode steps: B={Bn} S={S} kt={kt} H={Hq}/{Hkv} D={D} n0={n0} T={T}")
    r = np.random.default_rng([53])
    kc, vc = _mk(r, (Bn, S, Hkv, kt, D)), _mk(r, (Bn, S, Hkv, kt, D))
    k0, v0 = _mk(r, (Bn, n0, Hkv, D)), _mk(r, (Bn, n0, Hkv, D))
    qn, kn, vn = _mk(r, (Bn, T, Hq, D), 3.0), _mk(r, (Bn, T, Hkv, D)), _mk(r, (Bn, T, Hkv, D))
    sl = r.integers(1, kt + 1, size=(Bn, S)).astype(np.int32)
    cache = DecodeCacheFp8(Bn, S, kt, cap, Hq, Hkv, D, base)
    cache.load(bits_to_dev(kc), bits_to_dev(vc), torch.from_numpy(sl).cuda(), bits_to_dev(k0), bits_to_dev(v0))
    qd, kd, vd = bits_to_dev(qn), bits_to_dev(kn), bits_to_dev(vn)
    outs, lses = [], []
    for t in range(T):
        cache.step(qd[:, t:t + 1].contiguous(), kd[:, t:t + 1].contiguous(), vd[:, t:t + 1].contiguous(), pos0 + t)
        outs.append(cache.out.clone()); lses.append(cache.lse.clone())
    torch.cuda.synchronize()
    assert (cache.tail_len.cpu().numpy() == n0 + T).all()
    to_bf16 = lambda x: bf16_bits_to_f64(f32_to_bf16_bits(np.asarray(x, dtype=np.float32)))
    for b in range(Bn):
        rk8, rks, rv8, rvs = oracle.quantize_kv_fp8(bf16_bits_to_f64(kc[b]), bf16_bits_to_f64(vc[b]), sl[b])
        ro, rl, _ = oracle.decode_steps(bf16_bits_to_f64(qn[b]), bf16_bits_to_f64(kn[b]), bf16_bits_to_f64(vn[b]),
                                        oracle.dequantize_kv_fp8(rk8, rks), oracle.dequantize_kv_fp8(rv8, rvs),
                                        bf16_bits_to_f64(k0[b]), bf16_bits_to_f64(v0[b]), pos0, base,
                                        seg_len=sl[b], store=to_bf16)
        go = np.stack([dev_bf16_to_f64(o[b, 0]) for o in outs])
        gl = np.stack([l[b, :, 0].cpu().numpy() for l in lses])
        assert_close(go, ro, O_ATOL, O_RTOL, f"fp8 decode steps out[b={b}]")
        assert_close(gl, rl, LSE_ATOL, 1e-3, f"fp8 decode steps lse[b={b}]")


def test_fp8_dequantisation_is_exact_for_every_code():
    """One key per segment and scale 1: the output is the key's value row and, with unit-vector
    queries and softmax scale 1, the row logsumexp is one element of the key.  Every finite code
    (subnormals included) must come out as the value the format defines."""
    _say("fp8 attention: every code exact")
    codes = np.arange(256, dtype=np.uint8)
    codes[(codes & 0x7F) == 0x7F] = 0                       # the two NaN codes
    vals = oracle.fp8_e4m3_decode(codes)
    D, Hq = 128, 8
    one = torch.ones((1, 1, 1), dtype=torch.float32, device="cuda")
    ws = pc.alloc_workspace(pc.pc_parallel_attn_fp8_workspace_bytes(1, 1, 1, 1, 0, Hq, 1, D))
    out = torch.empty((1, 1, Hq, D), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((1, Hq, 1), dtype=torch.float32, device="cuda")
    for half in range(2):
        row = torch.from_numpy(codes[128 * half:128 * half + 128].copy()).cuda().view(1, 1, 1, 1, D)
        krow, vrow = fp8_from_rows("k", row), fp8_from_rows("v", row)   # the key as a block of K and of V
        for d0 in range(0, D, Hq):
            q = np.zeros((1, 1, Hq, D), dtype=np.float32)
            for h in range(Hq):
                q[0, 0, h, d0 + h] = 1.0
            pc.pc_parallel_attn_fp8(bits_to_dev(f32_to_bf16_bits(q)), krow, vrow, one, one, None, None, None, None, 0,
                                    1, 1, 1, 1, Hq, 1, D, -1, 1.0e4, 1.0, out, lse, ws)
            torch.cuda.synchronize()
            want = vals[128 * half:128 * half + 128]
            got_lse = lse[0, :, 0].cpu().numpy().astype(np.float64)
            np.testing.assert_allclose(got_lse, want[d0:d0 + Hq], rtol=1e-6, atol=1e-12)
            if d0 == 0:                                      # p = 1: the output is the value row, bit for bit
                np.testing.assert_array_equal(dev_bf16_to_f64(out[0, 0]), np.broadcast_to(want, (Hq, D)))


def test_fp8_attention_many_ragged_groups():
    """Enough groups that a workgroup takes several consecutive 8-bit segments, each with its own
    scales and a ragged length."""
    _attn_case("many-groups", 64, 1, 8, 48, 16, 8, 64, 0, -1, True, 5)


def test_fp8_attention_more_segments_than_lanes():
    """150 short ragged segments per group (the kernel walks the segment lengths 64 at a time to
    find a wavefront's first block), with a 16-bit tail."""
    _attn_case("150-segments", 2, 1, 150, 40, 8, 2, 128, 24, -1, True, 9)


def test_fp8_attention_query_block_over_the_8bit_cache():
    """The prefill stage of Eq. 9-11 over the 8-bit cache: a block of query rows (more than the 16
    columns of the split-KV kernel: the MFMA tile path on widened segments) attends over the
    dequantised segments, a 16-bit tail whose rows are all visible, and causally over itself."""
    _attn_case("block-self", 1, 104, 3, 200, 8, 2, 128, 0, 600, False, 11, with_self=True)
    _attn_case("block-tail-self-ragged64", 2, 70, 2, 130, 4, 4, 64, 45, -1, True, 12, with_self=True)
    _attn_case("block-noself", 1, 40, 2, 64, 8, 8, 128, 0, -1, True, 13)
    _attn_case("block-self-only", 1, 33, 0, 64, 8, 2, 128, 0, 5, False, 14, with_self=True)
    # few rows with a causal self segment: the split-KV kernel, self segment inside the merge
    _attn_case("nq3-self", 2, 3, 3, 300, 8, 2, 128, 0, 9, True, 15, with_self=True)
    _attn_case("nq2-tail-self", 1, 2, 2, 97, 4, 1, 64, 20, -1, False, 16, with_self=True)


def _drawn_fp8_cases(n):
    r = np.random.default_rng([2502, 97])
    out = []
    for i in range(n):
        D = int(r.choice([64, 128]))
        Hkv = int(r.choice([1, 2, 3]))
        G = int(r.choice([1, 2, 4, 8]))
        n_q = int(r.choice([1, 2, 3, 5, 17, 70]))
        with_self = bool(r.integers(0, 2))
        tail_cap = int(r.choice([0, 1, 33, 90]))
        S = int(r.integers(0 if (with_self or tail_cap) else 1, 5))
        out.append((int(r.integers(1, 4)), n_q, S, int(r.integers(1, 300)), Hkv * G, Hkv, D, tail_cap,
                    int(r.choice([-1, 0, 777])), bool(r.integers(0, 2)) and S > 0, 200 + i, with_self))
    return out


@pytest.mark.parametrize("case", _drawn_fp8_cases(12), ids=lambda c: "x".join(str(int(x)) for x in c[:10]) + f"x{int(c[11])}")
def test_fp8_attention_drawn_shapes(case):
    """Twelve calls over the 8-bit cache drawn from a fixed seed: the split-KV path and the tile
    path, with and without a 16-bit tail and a causal self segment, ragged or full segments."""
    B, n_q, S, kt, Hq, Hkv, D, tail_cap, q_pos0, ragged, seed, with_self = case
    _attn_case("drawn", B, n_q, S, kt, Hq, Hkv, D, tail_cap, q_pos0, ragged, seed, with_self=with_self)


def test_fp8_decode_full_size_sampled():
    """The decode config (16 sequences x 32 segments x 2048 rows x 8 KV heads) in 8 bits: sampled
    (sequence, KV group) pairs against the oracle on its own codes, and the codes themselves on
    sampled segments."""
    cfg = CFG4
    _say(f"fp8 decode {cfg.name}")
    g = torch.Generator(device="cuda").manual_seed(8)
    B, S, Hkv, kt, D, Hq = cfg.batch, cfg.n_seg, cfg.n_kv_heads, cfg.keep_tokens, cfg.head_dim, cfg.n_q_heads
    bf = torch.bfloat16
    kc = torch.empty((B, S, Hkv, kt, D), dtype=bf, device="cuda")
    vc = torch.empty_like(kc)
    for b in range(B):
        kc[b] = torch.randn(kc.shape[1:], generator=g, device="cuda").to(bf)
        vc[b] = torch.randn(kc.shape[1:], generator=g, device="cuda").to(bf)
    k8, v8 = fp8_alloc(B, S, Hkv, kt, D), fp8_alloc(B, S, Hkv, kt, D)
    ks = torch.empty((B, S, Hkv), dtype=torch.float32, device="cuda"); vs = torch.empty_like(ks)
    pc.pc_kv_quantize_fp8(kc, vc, None, B, S, kt, Hkv, D, k8, v8, ks, vs)
    q = torch.randn((B, 1, Hq, D), generator=g, device="cuda").to(bf)
    out = torch.empty((B, 1, Hq, D), dtype=bf, device="cuda")
    lse = torch.empty((B, Hq, 1), dtype=torch.float32, device="cuda")
    ws = pc.alloc_workspace(pc.pc_parallel_attn_fp8_workspace_bytes(B, 1, S, kt, 0, Hq, Hkv, D))
    pc.pc_parallel_attn_fp8(q, k8, v8, ks, vs, None, None, None, None, 0, B, 1, S, kt, Hq, Hkv, D, -1, 1.0e4,
                            0.0, out, lse, ws)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    G = Hq // Hkv
    for (b, gk) in ((0, 0), (6, 2), (15, 7)):
        kf = dev_bf16_to_f64(kc[b, :, gk])[:, None]          # [S, 1, kt, D]
        vf = dev_bf16_to_f64(vc[b, :, gk])[:, None]
        rk8, rks, rv8, rvs = oracle.quantize_kv_fp8(kf, vf)
        np.testing.assert_array_equal(fp8_rows_view("k", k8[b, :, gk], kt, D).cpu().numpy(), rk8[:, 0])
        np.testing.assert_array_equal(fp8_rows_view("v", v8[b, :, gk], kt, D).cpu().numpy(), rv8[:, 0])
        np.testing.assert_array_equal(ks[b, :, gk].cpu().numpy(), rks[:, 0])
        qf = dev_bf16_to_f64(q[b, :, gk * G:(gk + 1) * G])
        ro, rl = oracle.global_attention_concat(qf, oracle.dequantize_kv_fp8(rk8, rks),
                                                oracle.dequantize_kv_fp8(rv8, rvs))
        assert_close(dev_bf16_to_f64(out[b, :, gk * G:(gk + 1) * G]), ro, O_ATOL, O_RTOL, f"fp8 decode out[b={b},g={gk}]")
        assert_close(lse[b, gk * G:(gk + 1) * G, 0].cpu().numpy(), rl[0], LSE_ATOL, 1e-3, f"fp8 decode lse[b={b},g={gk}]")


def test_gather_amax_and_one_read_quantisation_bit_exact():
    """pc_gather_kv_amax = pc_gather_kv + the per-segment maxima of |K| and |V| (bit-exact against
    the maxima of the oracle's gathered rows); pc_kv_quantize_fp8_amax with those maxima writes the
    oracle's codes and scales (= what the two-read entry point writes).  Missing tokens (-1), a
    segment without a source chunk (skipped, keeps its contents) and a block straddling two
    segments (k not a multiple of the gather's rows per block) are all in."""
    _say("gather + amax, one-read quantisation")
    r = np.random.default_rng(57)
    B, C, rows, Hkv, S, k, D = 2, 4, 300, 2, 3, 100, 128
    ks = _mk(r, (B, C, rows, Hkv, D), 3.0); vs = _mk(r, (B, C, rows, Hkv, D), 0.2)
    ks[1, 2, 17, 1] = f32_to_bf16_bits(np.full(D, -91.0, dtype=np.float32))     # an outlier row
    cidx = np.array([[3, -1, 0], [2, 2, 1]], dtype=np.int32)
    tidx = np.sort(np.stack([np.stack([np.stack([r.choice(rows, size=k, replace=False) for _ in range(Hkv)])
                                       for _ in range(S)]) for _ in range(B)]), axis=-1).astype(np.int32)
    cnt = r.integers(1, k + 1, size=(B, S, Hkv)).astype(np.int32)
    for b in range(B):
        for s_ in range(S):
            for g in range(Hkv):
                tidx[b, s_, g, cnt[b, s_, g]:] = -1                              # a head that kept fewer tokens
    tidx[1, 1, 0, :cnt[1, 1, 0]] = np.sort(np.append(r.choice(rows, size=cnt[1, 1, 0] - 1, replace=False), 17))[:cnt[1, 1, 0]]
    bf = torch.bfloat16
    kd = torch.full((B, S, Hkv, k, D), 5.0, dtype=bf, device="cuda"); vd = torch.full_like(kd, 5.0)
    kd2 = kd.clone(); vd2 = vd.clone()
    ka = torch.full((B, S, Hkv), 123.0, dtype=torch.float32, device="cuda"); va = torch.full_like(ka, 123.0)
    dks, dvs, dc, dt = bits_to_dev(ks), bits_to_dev(vs), torch.from_numpy(cidx).cuda(), torch.from_numpy(tidx).cuda()
    pc.pc_gather_kv(dks, dvs, dc, dt, B, C, rows, S, Hkv, k, D, kd2, vd2)
    pc.pc_gather_kv_amax(dks, dvs, dc, dt, B, C, rows, S, Hkv, k, D, kd, vd, ka, va)
    torch.cuda.synchronize()
    assert torch.equal(kd.view(torch.int16), kd2.view(torch.int16)) and torch.equal(vd.view(torch.int16), vd2.view(torch.int16))
    ka_h, va_h = ka.cpu().numpy(), va.cpu().numpy()
    for b in range(B):
        live = [s_ for s_ in range(S) if cidx[b, s_] >= 0]
        rk, rv = oracle.gather_kv(ks[b], vs[b], cidx[b, live], tidx[b, live])
        assert np.array_equal(dev_to_bits(kd[b, live]), rk) and np.array_equal(dev_to_bits(vd[b, live]), rv)
        np.testing.assert_array_equal(ka_h[b, live], np.abs(bf16_bits_to_f64(rk)).max(axis=(2, 3)))
        np.testing.assert_array_equal(va_h[b, live], np.abs(bf16_bits_to_f64(rv)).max(axis=(2, 3)))
    assert (ka_h[0, 1] == 123.0).all() and (va_h[0, 1] == 123.0).all() and (kd[0, 1] == 5.0).all()
    # quantise the gathered cache from one read; the skipped segment gets a maximum of its own
    ka[0, 1] = 5.0; va[0, 1] = 5.0
    k8 = fp8_alloc(B, S, Hkv, k, D).fill_(0x55); v8 = fp8_alloc(B, S, Hkv, k, D).fill_(0x55)
    sk = torch.empty((B, S, Hkv), dtype=torch.float32, device="cuda"); sv = torch.empty_like(sk)
    dcnt = torch.from_numpy(cnt).cuda()
    pc.pc_kv_quantize_fp8_amax(kd, vd, ka, va, dcnt, B, S, k, Hkv, D, k8, v8, sk, sv, seg_len_per_head=1)
    k8b = fp8_alloc(B, S, Hkv, k, D).fill_(0x55); v8b = fp8_alloc(B, S, Hkv, k, D).fill_(0x55)
    skb = torch.empty_like(sk); svb = torch.empty_like(sk)
    pc.pc_kv_quantize_fp8(kd, vd, dcnt, B, S, k, Hkv, D, k8b, v8b, skb, svb, seg_len_per_head=1)
    torch.cuda.synchronize()
    assert torch.equal(k8, k8b) and torch.equal(v8, v8b) and torch.equal(sk, skb) and torch.equal(sv, svb)
    for b in range(B):
        rk8, rks, rv8, rvs = oracle.quantize_kv_fp8(dev_bf16_to_f64(kd[b]), dev_bf16_to_f64(vd[b]), cnt[b])
        np.testing.assert_array_equal(fp8_rows_view("k", k8[b], k, D).cpu().numpy(), rk8)
        np.testing.assert_array_equal(fp8_rows_view("v", v8[b], k, D).cpu().numpy(), rv8)
        np.testing.assert_array_equal(sk[b].cpu().numpy(), rks)
        np.testing.assert_array_equal(sv[b].cpu().numpy(), rvs)
