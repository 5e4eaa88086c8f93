"""The entry point that allocates nothing (pc_parallel_attn_static: the split-KV decode path of
Eq. 9-11 with its scratch in a fixed array inside the library) against pc_parallel_attn, through
the C ABI: two calls in a row, the second with a smaller input, both compared bit for bit with
the workspace entry point (the same kernels run) and with the oracle to the outputs' tolerance."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2502_14317_amd as pc
from helpers import O_ATOL, O_RTOL, LSE_ATOL, dev_bf16_to_f64, assert_close

pytestmark = pytest.mark.gpu


def _case(seed, B, S, kt, Hq, Hkv, D, n_q, ragged, with_self):
    g = torch.Generator(device="cuda").manual_seed(seed)
    bf = torch.bfloat16
    q = (torch.randn((B, n_q, Hq, D), generator=g, device="cuda") * 2.0).to(bf)
    kc = torch.randn((B, S, Hkv, kt, D), generator=g, device="cuda").to(bf)
    vc = torch.randn((B, S, Hkv, kt, D), generator=g, device="cuda").to(bf)
    seg_len = None
    if ragged:
        seg_len = torch.randint(0, kt + 1, (B, S), generator=g, device="cuda", dtype=torch.int32)
        seg_len[:, 0] = kt
    k_self = v_self = None
    if with_self:
        k_self = torch.randn((B, n_q, Hkv, D), generator=g, device="cuda").to(bf)
        v_self = torch.randn((B, n_q, Hkv, D), generator=g, device="cuda").to(bf)
    return q, kc, vc, seg_len, k_self, v_self


def _run_both(case, B, S, kt, Hq, Hkv, D, n_q, q_pos0, base):
    q, kc, vc, seg_len, k_self, v_self = case
    bf = torch.bfloat16
    outs = []
    for static in (False, True):
        # poison the outputs so that a call that writes nothing cannot pass
        out = torch.full((B, n_q, Hq, D), float("nan"), dtype=bf, device="cuda")
        lse = torch.full((B, Hq, n_q), float("nan"), dtype=torch.float32, device="cuda")
        if static:
            pc.pc_parallel_attn_static(q, kc, vc, seg_len, k_self, v_self, B, n_q, S, kt, Hq, Hkv, D,
                                       q_pos0, base, 0.0, out, lse)
        else:
            ws = pc.alloc_workspace(pc.pc_parallel_attn_workspace_bytes(B, n_q, S, kt, Hq, Hkv, D,
                                                                        k_self is not None))
            pc.pc_parallel_attn(q, kc, vc, seg_len, k_self, v_self, B, n_q, S, kt, Hq, Hkv, D, q_pos0,
                                base, 0.0, out, lse, ws)
        torch.cuda.synchronize()
        outs.append((out, lse))
    (o_ws, l_ws), (o_st, l_st) = outs
    assert torch.isfinite(o_st.float()).all() and torch.isfinite(l_st).all()
    assert torch.equal(o_ws.view(torch.int16), o_st.view(torch.int16)), "outputs differ from pc_parallel_attn"
    assert torch.equal(l_ws, l_st), "logsumexps differ from pc_parallel_attn"
    return o_st, l_st


def _check_oracle(case, out, lse, b, B, S, kt, Hq, Hkv, D, n_q, q_pos0, base):
    """Sequence b against one softmax over the concatenation (Eq. 9-11)."""
    q, kc, vc, seg_len, k_self, v_self = case
    qf = dev_bf16_to_f64(q[b])
    if q_pos0 >= 0:
        qf = oracle.rope(qf, q_pos0 + np.arange(n_q), base)
    sl = None if seg_len is None else seg_len[b].cpu().numpy()
    ro, rl = oracle.global_attention_concat(
        qf, dev_bf16_to_f64(kc[b]), dev_bf16_to_f64(vc[b]), seg_len=sl,
        k_self=None if k_self is None else dev_bf16_to_f64(k_self[b]),
        v_self=None if v_self is None else dev_bf16_to_f64(v_self[b]))
    assert_close(dev_bf16_to_f64(out[b]), ro, O_ATOL, O_RTOL, f"static out[b={b}]")
    assert_close(lse[b].cpu().numpy().T, rl, LSE_ATOL, 1e-3, f"static lse[b={b}]")


def test_static_entry_point_two_calls_second_smaller():
    assert pc.pc_parallel_attn_static_max_bytes() == 4 << 20
    # first call: 6 sequences x 7 ragged segments of up to 333 keys, GQA 8/2, one query row
    shape1 = dict(B=6, S=7, kt=333, Hq=8, Hkv=2, D=128, n_q=1)
    case1 = _case(101, ragged=True, with_self=False, **shape1)
    print("static call 1", shape1, flush=True)
    o1, l1 = _run_both(case1, q_pos0=1000, base=5.0e5, **shape1)
    _check_oracle(case1, o1, l1, 3, q_pos0=1000, base=5.0e5, **shape1)
    # second call, smaller in every dimension, 3 query rows with the causal self segment: the
    # scratch still holds the first call's partials beyond what this call writes
    shape2 = dict(B=2, S=3, kt=97, Hq=4, Hkv=1, D=64, n_q=3)
    case2 = _case(102, ragged=False, with_self=True, **shape2)
    print("static call 2", shape2, flush=True)
    o2, l2 = _run_both(case2, q_pos0=-1, base=1.0e4, **shape2)
    _check_oracle(case2, o2, l2, 1, q_pos0=-1, base=1.0e4, **shape2)
    # and the first input again: same result as before (nothing of call 2 leaks into it)
    o1b, l1b = _run_both(case1, q_pos0=1000, base=5.0e5, **shape1)
    assert torch.equal(o1.view(torch.int16), o1b.view(torch.int16)) and torch.equal(l1, l1b)


def test_static_entry_point_rejects_what_does_not_fit():
    one = ctypes.c_void_p(256)
    L = pc.lib()
    args = (4096, 1, 2, 64, 32, 8, 128, -1, 1e4, 0.0)
    assert L.pc_parallel_attn_static(one, one, one, None, 0, None, None, *args, one, None, None) == -3
    args = (1, 64, 2, 64, 8, 2, 128, -1, 1e4, 0.0)
    assert L.pc_parallel_attn_static(one, one, one, None, 0, None, None, *args, one, None, None) == -5
