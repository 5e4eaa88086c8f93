"""Can the full-size parity checks fail?  CPU-only proof on the peaked 128K input (cfg1p), with the
mistake planted on the oracle's side: the sampled rows of a chunk are recomputed by the oracle
with one 64-key tile of the sequence missing, and with one tile taken from the next chunk, and
the comparison the GPU test makes (helpers.assert_close with the outputs' tolerance) must reject
both; an all-zero output must be rejected too.  The same test checks the closed form that
tests/test_gpu_full_size.py uses to count which key tiles its sampled rows pin
(helpers.pinned_tiles) against the explicit recomputation."""
import numpy as np

import oracle
from workloads import CFG1P, CFG1, prefill_chunk, bf16_bits_to_f64
from helpers import (O_ATOL, O_RTOL, LSE_ATOL, sample_rows, assert_informative, pinned_tiles,
                     rejects)

TILE = 64


def _rotated(cfg, c):
    q, k, v = prefill_chunk(cfg, c)
    pos = np.arange(cfg.seq_len)
    return (oracle.rope(bf16_bits_to_f64(q), pos, cfg.rope_base),
            oracle.rope(bf16_bits_to_f64(k), pos, cfg.rope_base), bf16_bits_to_f64(v))


def test_sampled_rows_reject_a_missing_or_foreign_key_tile():
    cfg = CFG1P
    q0, k0, v0 = _rotated(cfg, 0)
    _, k1, v1 = _rotated(cfg, 1)
    rows = sample_rows(cfg)
    ref_o, ref_lse, P = oracle.local_attention(q0, k0, v0, rows=rows, return_probs=True)
    assert_informative(ref_o, "cfg1p o")
    # zeros, and the flat-softmax answer (the running mean of v), are both far outside
    assert rejects(np.zeros_like(ref_o), ref_o, O_ATOL, O_RTOL)
    pin = pinned_tiles(P, ref_o, ref_lse, v0, TILE)
    assert pin.all(), np.nonzero(~pin)[0]

    # explicit recomputation for a late row: its heaviest tile, a light tile, the first and the last
    ri = int(np.nonzero(rows == cfg.seq_len - 2)[0][0])
    r = int(rows[ri])
    G = cfg.group
    mass = P[ri].reshape(cfg.n_q_heads, -1, TILE).sum(axis=2)              # [H_q, tiles] (L is a multiple of 64)
    h_best, t_best = np.unravel_index(np.argmax(mass * (mass < 0.999)), mass.shape)
    for t in sorted({int(t_best), 0, 17, cfg.seq_len // TILE - 1}):
        keep = np.ones(cfg.seq_len, dtype=bool)
        keep[TILE * t:TILE * (t + 1)] = False
        keep[r] = True                                                      # the row's own key stays (it is its last visible key)
        # (a) tile missing: the same softmax over the remaining keys; the row index moves down
        n_gone = int((~keep[:r + 1]).sum())
        o_a, l_a = oracle.local_attention(np.concatenate([q0[keep][:r - n_gone], q0[r:r + 1]]),
                                          k0[keep][:r - n_gone + 1], v0[keep][:r - n_gone + 1],
                                          rows=[r - n_gone])
        # (b) tile read from the next chunk (same positions, so the same rotation)
        k_b, v_b = k0.copy(), v0.copy()
        sl = slice(TILE * t, min(TILE * (t + 1), r))
        k_b[sl], v_b[sl] = k1[sl], v1[sl]
        o_b, l_b = oracle.local_attention(q0, k_b, v_b, rows=[r])
        # the closed form of pinned_tiles agrees with (a)
        for h in range(cfg.n_q_heads):
            m = mass[h, t]
            if m < 1 - 1e-9 and not (t == r // TILE):
                part = (P[ri, h, TILE * t:TILE * (t + 1), None] * v0[TILE * t:TILE * (t + 1), h // G]).sum(axis=0)
                np.testing.assert_allclose(o_a[0, h], (ref_o[ri, h] - part) / (1 - m), rtol=1e-9, atol=1e-12)
                np.testing.assert_allclose(l_a[0, h], ref_lse[ri, h] + np.log1p(-m), rtol=1e-9, atol=1e-12)
        if t == t_best:
            # the heaviest tile of the row: both corruptions are rejected on that head
            h = int(h_best)
            assert rejects(o_a[0, h], ref_o[ri, h], O_ATOL, O_RTOL) or rejects(l_a[0, h], ref_lse[ri, h], LSE_ATOL, 1e-3)
            assert rejects(o_b[0, h], ref_o[ri, h], O_ATOL, O_RTOL) or rejects(l_b[0, h], ref_lse[ri, h], LSE_ATOL, 1e-3)
        # over all heads of the row, the missing tile is rejected exactly when pinned_tiles' own
        # criterion says so for this row
        rej_a = [rejects(o_a[0, h], ref_o[ri, h], O_ATOL, O_RTOL) or
                 rejects(l_a[0, h], ref_lse[ri, h], LSE_ATOL, 1e-3) for h in range(cfg.n_q_heads)]
        one_row = pinned_tiles(P[ri:ri + 1], ref_o[ri:ri + 1], ref_lse[ri:ri + 1], v0, TILE)
        if t != r // TILE:
            assert any(rej_a) == bool(one_row[t]), (t, rej_a, one_row[t])


def test_flat_inputs_are_not_informative():
    """The configs' own 1/sqrt(D) inputs: the check that guards the peaked tests fires on them."""
    cfg = CFG1
    q0, k0, v0 = _rotated(cfg, 0)
    rows = sample_rows(cfg)
    ref_o, _ = oracle.local_attention(q0, k0, v0, rows=rows)
    assert rejects(np.zeros_like(ref_o[rows >= 255]), ref_o[rows >= 255], O_ATOL, O_RTOL) is False
    try:
        assert_informative(ref_o, "cfg1 o")
    except AssertionError:
        return
    raise AssertionError("flat inputs passed the informativeness check")
