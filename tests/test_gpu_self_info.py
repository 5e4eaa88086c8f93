"""GPU parity of the chunk self-information reducer (Eq. 3) against the fp64 CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2502_14317_amd as pc
from workloads import lm_logits_inputs, bf16_bits_to_f64
from helpers import bits_to_dev, assert_close

pytestmark = pytest.mark.gpu

# fp32 accumulation of up to 2^17 exponentials per row and of n_t terms per chunk, inputs exact
# (bf16 logits): a row's log-sum-exp is good to ~1e-6 relative, the target logit is exact
NLL_ATOL, NLL_RTOL = 2e-5, 2e-6
INFO_RTOL = 2e-6


def _run(logits_bits, targets, negate=False):
    C, T, V = logits_bits.shape
    nll = torch.full((C, T), -1.0, dtype=torch.float32, device="cuda")
    info = torch.full((C,), -1.0, dtype=torch.float32, device="cuda")
    pc.pc_chunk_self_information(bits_to_dev(logits_bits), torch.from_numpy(targets).cuda(), C, T, V,
                                 negate, nll, info)
    torch.cuda.synchronize()
    return nll.cpu().numpy(), info.cpu().numpy()


@pytest.mark.parametrize("C,T,V,rel", [(3, 17, 1000, (1,)), (2, 5, 128256, (0,)), (1, 1, 8, ()),
                                       (5, 64, 32000, (4, 2)), (2, 300, 264, ())])
def test_self_information_parity(C, T, V, rel):
    print(f"self-information C={C} T={T} V={V}", flush=True)
    lb, targets = lm_logits_inputs(C, T, V, relevant=rel, cfg_id=32 + C)
    ref_I, ref_nll = oracle.chunk_self_information(bf16_bits_to_f64(lb), targets)
    nll, info = _run(lb, targets)
    assert_close(nll, ref_nll, NLL_ATOL, NLL_RTOL, "token_nll")
    assert_close(info, ref_I, 0.0, INFO_RTOL, "info")
    nll2, neg = _run(lb, targets, negate=True)
    assert np.array_equal(nll2, nll) and np.array_equal(neg, -info)      # deterministic, sign only
    if rel and C > len(rel):
        k = len(rel)
        idx = torch.empty((k,), dtype=torch.int32, device="cuda")
        pc.pc_select_chunks_topk(torch.from_numpy(neg).cuda(), C, k, idx, None)
        torch.cuda.synchronize()
        assert sorted(idx.cpu().tolist()) == sorted(rel)                   # Eq. 4: lowest I_c kept
        assert list(idx.cpu().numpy()) == list(oracle.select_chunks(-ref_I, k))


def test_self_information_extreme_logits_and_target_clamp():
    r = np.random.default_rng(61)
    C, T, V = 2, 3, 64
    x = (r.standard_normal((C, T, V)) * 2).astype(np.float32)
    x[0, 0, 5] = 3.0e4; x[0, 1, :] = -2.0e4; x[1, 2, 7] = -3.0e38
    from workloads import f32_to_bf16_bits
    lb = f32_to_bf16_bits(x)
    targets = np.array([5, 63, 0], dtype=np.int32)
    ref_I, ref_nll = oracle.chunk_self_information(bf16_bits_to_f64(lb), targets)
    nll, info = _run(lb, targets)
    assert_close(nll, ref_nll, 1e-3, 1e-6, "token_nll")       # |logit| up to 3e4: one fp32 ulp is 2e-3
    oob = np.array([-4, 1000, 0], dtype=np.int32)             # clamped to [0, V)
    nll_c, _ = _run(lb, oob)
    nll_w, _ = _run(lb, np.array([0, 63, 0], dtype=np.int32))
    assert np.array_equal(nll_c, nll_w)


def test_self_information_masked_vocabulary_entries():
    """-inf logits (masked or padded vocabulary entries) carry probability 0: whole runs of them,
    long enough that some lanes of the reduction see nothing else, must not poison the row."""
    from workloads import f32_to_bf16_bits
    r = np.random.default_rng(62)
    C, T, V = 2, 4, 40000
    x = (r.standard_normal((C, T, V)) * 2).astype(np.float32)
    x[0, 0, :36000] = -np.inf            # only the tail of the row is live
    x[0, 1, 8:] = -np.inf                # only the first vector is live
    x[1, 2, ::2] = -np.inf               # every other entry masked
    x[1, 3, 100:39000] = -np.inf
    lb = f32_to_bf16_bits(x)
    targets = np.array([39999, 3, 1, 50], dtype=np.int32)       # live entries
    ref_I, ref_nll = oracle.chunk_self_information(bf16_bits_to_f64(lb), targets)
    assert np.all(np.isfinite(ref_nll))
    nll, info = _run(lb, targets)
    assert_close(nll, ref_nll, NLL_ATOL, NLL_RTOL, "token_nll")
    assert_close(info, ref_I, 0.0, INFO_RTOL, "info")
