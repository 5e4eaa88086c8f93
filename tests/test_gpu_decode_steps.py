"""GPU parity of the decoding stage (Eq. 9-11 token by token with a growing tail): pc_kv_append
and the decode loop over it, against the fp64 CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2502_14317_amd as pc
from paper_2502_14317_amd.layer import DecodeCache
from workloads import f32_to_bf16_bits, bf16_bits_to_f64
from helpers import (O_ATOL, O_RTOL, LSE_ATOL, bits_to_dev, dev_to_bits, dev_bf16_to_f64,
                     assert_close)

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _mk(r, shape, s=1.0):
    return f32_to_bf16_bits((r.standard_normal(shape) * s).astype(np.float32))


def _to_bf16(x):
    return bf16_bits_to_f64(f32_to_bf16_bits(np.asarray(x, dtype=np.float32)))


def _assert_rotated_keys(gpu_bits, ref, what):
    """Rotated keys are rounded to bf16 once: within one bf16 ulp of the fp64 rotation (2^-8
    relative, 1e-5 absolute where the two products cancel)."""
    assert_close(bf16_bits_to_f64(gpu_bits), ref, 1e-5, 2.0 ** -8, what)


@pytest.mark.parametrize("Bn,S,kt,Hq,Hkv,D,n0,T,base,pos0,ragged",
                         [(2, 3, 160, 8, 2, 128, 37, 9, 5.0e5, 700, True),
                          (1, 2, 1100, 4, 4, 64, 64, 5, 1.0e4, 64, False),
                          (3, 0, 40, 32, 8, 128, 1, 12, 5.0e5, 0, False)],
                         ids=["gqa-ragged", "mha64-two-splits", "tail-only"])
def test_decode_steps_match_oracle(Bn, S, kt, Hq, Hkv, D, n0, T, base, pos0, ragged):
    _say(f"decode steps: B={Bn} S={S} kt={kt} H={Hq}/{Hkv} D={D} n0={n0} T={T} pos0={pos0}")
    r = np.random.default_rng([41, Bn, S, kt])
    kc, vc = _mk(r, (Bn, S, Hkv, kt, D)), _mk(r, (Bn, S, Hkv, kt, D))
    k0, v0 = _mk(r, (Bn, n0, Hkv, D)), _mk(r, (Bn, n0, Hkv, D))
    qn, kn, vn = _mk(r, (Bn, T, Hq, D), 3.0), _mk(r, (Bn, T, Hkv, D)), _mk(r, (Bn, T, Hkv, D))
    sl = r.integers(1, kt + 1, size=(Bn, S)).astype(np.int32) if ragged else None
    cache = DecodeCache(Bn, S, kt, Hq, Hkv, D, base)
    cache.kc.fill_(9.0); cache.vc.fill_(9.0)               # stale rows nothing may read
    cache.load(bits_to_dev(kc), bits_to_dev(vc), torch.from_numpy(sl).cuda() if ragged else None,
               bits_to_dev(k0), bits_to_dev(v0))
    qd, kd, vd = bits_to_dev(qn), bits_to_dev(kn), bits_to_dev(vn)
    outs, lses = [], []
    for t in range(T):
        cache.step(qd[:, t:t + 1].contiguous(), kd[:, t:t + 1].contiguous(),
                   vd[:, t:t + 1].contiguous(), pos0 + t)
        outs.append(cache.out.clone()); lses.append(cache.lse.clone())
    torch.cuda.synchronize()
    assert (cache.seg_len[:, S].cpu().numpy() == n0 + T).all()
    if ragged:
        np.testing.assert_array_equal(cache.seg_len[:, :S].cpu().numpy(), sl)
    tail_k, tail_v = dev_to_bits(cache.kc[:, S]), dev_to_bits(cache.vc[:, S])    # [B, Hkv, kt, D]
    for b in range(Bn):
        # the cache is bf16: the oracle rounds its own rotated key once on entry (store=), and
        # the rows the GPU stored are checked against the oracle's unrounded rotation
        k_rot = oracle.rope(bf16_bits_to_f64(kn[b]), pos0 + np.arange(T), base)
        _assert_rotated_keys(tail_k[b, :, n0:n0 + T].transpose(1, 0, 2), k_rot, f"tail k[b={b}]")
        np.testing.assert_array_equal(tail_k[b, :, :n0].transpose(1, 0, 2), k0[b])
        np.testing.assert_array_equal(tail_v[b, :, :n0].transpose(1, 0, 2), v0[b])
        np.testing.assert_array_equal(tail_v[b, :, n0:n0 + T].transpose(1, 0, 2), vn[b])
        assert (tail_k[b, :, n0 + T:] == 0x4110).all()      # bf16 9.0: rows behind the tail untouched
        ro, rl, _ = oracle.decode_steps(bf16_bits_to_f64(qn[b]), bf16_bits_to_f64(kn[b]),
                                        bf16_bits_to_f64(vn[b]), bf16_bits_to_f64(kc[b]),
                                        bf16_bits_to_f64(vc[b]), bf16_bits_to_f64(k0[b]),
                                        bf16_bits_to_f64(v0[b]), pos0, base,
                                        seg_len=sl[b] if ragged else None, store=_to_bf16)
        go = np.stack([dev_bf16_to_f64(o[b, 0]) for o in outs])
        gl = np.stack([l[b, :, 0].cpu().numpy() for l in lses])
        assert_close(go, ro, O_ATOL, O_RTOL, f"decode out[b={b}]")
        assert_close(gl, rl, LSE_ATOL, 1e-3, f"decode lse[b={b}]")


def test_kv_append_blocks_per_head_lengths_and_saturation():
    """n_new > 1 in one call, per-head lengths, already-rotated rows, and a segment that fills up:
    rows that do not fit are dropped, lengths stop at the capacity, other segments are untouched."""
    _say("kv_append: per-head lengths, saturation")
    r = np.random.default_rng([42])
    Bn, S, Hkv, kt, D, n_new = 2, 3, 4, 10, 64, 4
    kc = _mk(r, (Bn, S, Hkv, kt, D)); vc = _mk(r, (Bn, S, Hkv, kt, D))
    kn = _mk(r, (Bn, n_new, Hkv, D)); vn = _mk(r, (Bn, n_new, Hkv, D))
    sl = r.integers(0, kt + 1, size=(Bn, S, Hkv)).astype(np.int32)
    sl[0, 1] = [0, 7, 9, 10]                               # room for all / 3 / 1 / none
    for pos0 in (-1, 123):
        kcd, vcd, sld = bits_to_dev(kc.copy()), bits_to_dev(vc.copy()), torch.from_numpy(sl.copy()).cuda()
        pc.pc_kv_append(bits_to_dev(kn), bits_to_dev(vn), Bn, n_new, S, 1, kt, Hkv, D, pos0, 1.0e4,
                        kcd, vcd, sld, seg_len_per_head=1)
        torch.cuda.synchronize()
        gk, gv, gl = dev_to_bits(kcd), dev_to_bits(vcd), sld.cpu().numpy()
        want_len = sl.copy(); want_len[:, 1] = np.minimum(sl[:, 1] + n_new, kt)
        np.testing.assert_array_equal(gl, want_len)
        for b in range(Bn):
            k_ref = (bf16_bits_to_f64(kn[b]) if pos0 < 0 else
                     oracle.rope(bf16_bits_to_f64(kn[b]), pos0 + np.arange(n_new), 1.0e4))
            for g in range(Hkv):
                n_fit = int(want_len[b, 1, g] - sl[b, 1, g])
                lo = int(sl[b, 1, g])
                if pos0 < 0:
                    np.testing.assert_array_equal(gk[b, 1, g, lo:lo + n_fit], kn[b, :n_fit, g])
                else:
                    _assert_rotated_keys(gk[b, 1, g, lo:lo + n_fit], k_ref[:n_fit, g], f"k[{b},{g}]")
                np.testing.assert_array_equal(gv[b, 1, g, lo:lo + n_fit], vn[b, :n_fit, g])
                np.testing.assert_array_equal(gk[b, 1, g, :lo], kc[b, 1, g, :lo])
                np.testing.assert_array_equal(gk[b, 1, g, lo + n_fit:], kc[b, 1, g, lo + n_fit:])
                np.testing.assert_array_equal(gv[b, 1, g, lo + n_fit:], vc[b, 1, g, lo + n_fit:])
        np.testing.assert_array_equal(gk[:, [0, 2]], kc[:, [0, 2]])
        np.testing.assert_array_equal(gv[:, [0, 2]], vc[:, [0, 2]])
    # empty calls are no-ops
    pc.pc_kv_append(bits_to_dev(kn), bits_to_dev(vn), Bn, 0, S, 1, kt, Hkv, D, -1, 1.0e4, kcd, vcd, sld,
                    seg_len_per_head=1)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(sld.cpu().numpy(), want_len)
