"""Shared pieces of the GPU parity tests: tolerances (written out here), upload helpers and
the selection-set comparison rule."""
import numpy as np
import torch

# attention outputs, bf16 inputs / fp32 accumulation: |gpu - ref| <= 2e-2 + 1e-2 |ref|
O_ATOL, O_RTOL = 2e-2, 1e-2
# scores: 1e-3 relative (tiny absolute floor for exact zeros)
S_RTOL, S_ATOL = 1e-3, 1e-12
# row logsumexp: a probability-weighted mean of logit errors; logits carry the bf16 rounding of
# the rotated q and k (2^-9 relative per element), so the same absolute bound as the outputs
LSE_ATOL = 2e-2
# selection: a differing index is accepted only if its oracle score is within 1e-4 relative
# of the oracle's k-th score
SEL_GAP = 1e-4


def bits_to_dev(bits):
    """uint16 bf16 bit patterns -> bf16 CUDA tensor holding the same bits."""
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def dev_to_bits(t):
    return t.detach().view(torch.int16).cpu().numpy().view(np.uint16)


def dev_bf16_to_f64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def assert_close(gpu, ref, atol, rtol, what):
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert gpu.shape == ref.shape, (what, gpu.shape, ref.shape)
    assert np.all(np.isfinite(gpu)), f"{what}: non-finite values on the GPU side"
    err = np.abs(gpu - ref)
    bound = atol + rtol * np.abs(ref)
    bad = err > bound
    if bad.any():
        i = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError(f"{what}: {bad.sum()} of {bad.size} outside tolerance; worst at {i}: "
                             f"gpu {gpu[i]!r} ref {ref[i]!r} err {err[i]:.3e} bound {bound[i]:.3e}")


def assert_selection_matches(gpu_idx, ref_idx, ref_score, what):
    """gpu_idx, ref_idx: index sets of one problem; ref_score: the oracle's scores [n].
    Sets must be equal except for indices whose oracle score lies within SEL_GAP (relative) of
    the oracle's k-th score."""
    gs, rs = set(int(i) for i in gpu_idx), set(int(i) for i in ref_idx)
    assert len(gs) == len(gpu_idx), f"{what}: duplicate indices"
    assert len(gs) == len(rs), f"{what}: set sizes differ"
    if gs == rs:
        return 0
    kth = min(ref_score[list(rs)])
    for i in gs ^ rs:
        gap = abs(ref_score[i] - kth)
        assert gap <= SEL_GAP * abs(kth), (f"{what}: index {i} differs, oracle score "
                                           f"{ref_score[i]!r} vs k-th {kth!r} (gap {gap:.3e})")
    return len(gs ^ rs)
