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


# ------------------------------------------------------------------ informative full-size checks
def sample_rows(cfg):
    """Rows of a chunk sequence the full-size tests evaluate the oracle on: tile and chunk
    boundaries plus seeded random rows."""
    L, w = cfg.seq_len, cfg.chunk_len
    fixed = [0, 1, 31, 32, 63, 64, 255, 256, 257, L // 2, w - 1, w, w + 1, L - 33, L - 2, L - 1]
    rng = np.random.default_rng([99, cfg.cfg_id])
    return np.unique(np.concatenate([np.array(fixed), rng.integers(0, L, size=16)]))


def assert_informative(ref_o, what):
    """The reference must carry signal: the median magnitude of the sampled outputs is at least
    five times the absolute tolerance, so a check on it cannot pass on zeros or on a flat mean."""
    med = float(np.median(np.abs(ref_o)))
    assert med >= 5 * O_ATOL, f"{what}: median |ref| {med:.3e} is below 5 x the absolute tolerance"
    return med


def rejects(gpu, ref, atol, rtol):
    """True iff assert_close(gpu, ref, ...) raises."""
    try:
        assert_close(gpu, ref, atol, rtol, "probe")
    except AssertionError:
        return True
    return False


def pinned_tiles(P, o, lse, v, tile=64):
    """Which key tiles do the sampled rows pin?  P [n_rows, H_q, L] the oracle's probabilities,
    o [n_rows, H_q, D] and lse its outputs, v [L, H_kv, D].  For every (row, head) and every
    `tile`-key tile, the output the row would have if that tile's keys were missing is
    (o - m_t o_t) / (1 - m_t) with m_t the tile's mass and o_t its own weighted mean, and the
    logsumexp moves by log(1 - m_t).  Returns a boolean [n_tiles]: True where for at least one
    sampled (row, head) the output without the tile falls outside the outputs' tolerance, or the
    logsumexp outside its own, i.e. where the parity check fails if the kernel drops that tile."""
    n, Hq, L = P.shape
    Hkv = v.shape[1]
    G = Hq // Hkv
    nt = (L + tile - 1) // tile
    pin = np.zeros(nt, dtype=bool)
    pad = nt * tile - L
    for h in range(Hq):
        p = np.pad(P[:, h, :], ((0, 0), (0, pad)))                        # [n, nt * tile]
        vv = np.pad(v[:, h // G, :], ((0, pad), (0, 0)))                   # [nt * tile, D]
        m = p.reshape(n, nt, tile).sum(axis=2)                            # [n, nt]
        part = np.einsum("ntk,tkd->ntd", p.reshape(n, nt, tile), vv.reshape(nt, tile, -1))
        ok = m < 1.0 - 1e-9                                               # a tile holding everything: no output left
        denom = np.where(ok, 1.0 - m, 1.0)
        without = (o[:, h, None, :] - part) / denom[..., None]
        bad_o = (np.abs(without - o[:, h, None, :]) > O_ATOL + O_RTOL * np.abs(o[:, h, None, :])).any(axis=2)
        bad_l = -np.log(denom) > LSE_ATOL + 1e-3 * np.abs(lse[:, h, None])
        pin |= ((bad_o | bad_l) & ok).any(axis=0)
    return pin


# ------------------------------------------------------------------ 8-bit cache: layout views
# Host-side views of the 32-key block layout that pc_kv_quantize_fp8 writes and
# pc_parallel_attn_fp8 reads (include/parallelcomp.h states it), in both directions, so the tests
# can compare codes with the oracle's row-ordered ones.
def fp8_rows(k_t):
    """Key rows the codes of a segment occupy: whole 32-key blocks."""
    return (k_t + 31) // 32 * 32


def _fp8_perm(which, n, to_rows):
    # K block: [blk, tile, i, kk, c, b]  (key = 16 tile + c, d = 64 i + 16 kk + b)
    # V block: [blk, q, g, m, h, j / 4, j % 4]  (key = 16 (j / 4) + 4 g + j % 4, d = 32 q + 16 h + m)
    if which == "k":
        fwd = (n, n + 1, n + 4, n + 2, n + 3, n + 5)               # -> blk, tile, c, i, kk, b
    else:
        fwd = (n, n + 5, n + 2, n + 6, n + 1, n + 4, n + 3)        # -> blk, j / 4, g, j % 4, q, h, m
    if to_rows:
        return fwd
    inv = [0] * len(fwd)
    for pos, src in enumerate(fwd):
        inv[src - n] = n + pos
    return tuple(inv)


def _fp8_block_shape(which, n_blk, head_dim):
    return (n_blk, 2, head_dim // 64, 4, 16, 16) if which == "k" else (n_blk, head_dim // 32, 4, 16, 2, 2, 4)


def _fp8_row_shape(which, n_blk, head_dim):
    return (n_blk, 2, 16, head_dim // 64, 4, 16) if which == "k" else (n_blk, 2, 4, 4, head_dim // 32, 2, 16)


def fp8_rows_view(which, codes, k_t, head_dim, padded=False):
    """The K ("k") or V ("v") codes in row order [..., k_t, D] (a copy; with padded=True all
    ceil(k_t / 32) * 32 rows) from the block layout the kernels use.  K block of 32 keys: two
    16-key tiles of D / 64 pieces of 64 lanes x 16 bytes, lane 16 kk + c holding d = 64 i + 16 kk
    .. + 15 of key c of the tile.  V block: D / 32 pieces of 64 lanes x 16 bytes, lane 16 g + m
    holding [h][j] with d = 32 q + 16 h + m and key 4 g + j (j < 4) or 16 + 4 g + j - 4 (j >= 4)."""
    lead = codes.shape[:-1]
    n_blk, n = fp8_rows(k_t) // 32, len(codes.shape) - 1
    x = codes.reshape(*lead, *_fp8_block_shape(which, n_blk, head_dim))
    x = x.permute(*range(n), *_fp8_perm(which, n, True))
    return x.reshape(*lead, n_blk * 32, head_dim)[..., :(n_blk * 32 if padded else k_t), :].contiguous()


def fp8_from_rows(which, codes):
    """Inverse of fp8_rows_view: codes [..., k_t, D] uint8 in row order -> the block layout
    [..., ceil(k_t / 32) * 32 * D] (keys behind k_t get code 0)."""
    lead, k_t, head_dim = codes.shape[:-2], codes.shape[-2], codes.shape[-1]
    n_blk, n = fp8_rows(k_t) // 32, len(codes.shape) - 2
    x = torch.zeros((*lead, n_blk * 32, head_dim), dtype=torch.uint8, device=codes.device)
    x[..., :k_t, :] = codes
    x = x.reshape(*lead, *_fp8_row_shape(which, n_blk, head_dim))
    x = x.permute(*range(n), *_fp8_perm(which, n, False))
    return x.reshape(*lead, n_blk * 32 * head_dim).contiguous()
