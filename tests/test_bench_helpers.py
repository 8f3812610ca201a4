"""bench.py's counting helpers against brute force on small masks (CPU only)."""
import os
import sys

import numpy as np
import pytest

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import bench  # noqa: E402


def _mask(S, cols, offs, w):
    i = np.arange(S)[:, None]
    j = np.arange(S)[None, :]
    return (j <= i) & (np.isin(j, cols) | np.isin(i - j, offs) | (i - j < w))


@pytest.mark.parametrize("S,seed", [(700, 1), (515, 2), (1024, 3), (130, 4)])
def test_counts_match_brute_force(S, seed):
    rng = np.random.default_rng(seed)
    cols = np.sort(rng.choice(S, 5, replace=False))
    offs = np.sort(rng.choice(S, 4, replace=False))
    w = 3
    M = _mask(S, cols, offs, w)
    assert bench.mask_density(S, cols, offs, w) == pytest.approx(M.sum() / (S * (S + 1) / 2.0), rel=1e-12)
    blk = 128
    nb = (S + blk - 1) // blk
    touched = sum(M[bi * blk:(bi + 1) * blk, bj * blk:(bj + 1) * blk].any()
                  for bi in range(nb) for bj in range(bi + 1))
    assert bench.touched_block_fraction(S, cols, offs, w) == pytest.approx(touched / (nb * (nb + 1) / 2.0), rel=1e-12)


@pytest.mark.parametrize("S,blk,w,seed", [(1024, 128, 128, 1), (1000, 64, 1, 2), (700, 128, 300, 3), (256, 128, 5, 4)])
def test_block_mask_density_matches_brute_force(S, blk, w, seed):
    # block (I, J) is kept when J is selected, or a full block on diagonal I - J
    # (offsets blk*(I-J) - (blk-1) .. blk*(I-J) + (blk-1)) holds a kept offset
    rng = np.random.default_rng(seed)
    nb = (S + blk - 1) // blk
    Ic = np.sort(rng.choice(nb, rng.integers(0, nb // 2 + 1), replace=False))
    Is = np.sort(rng.choice(nb, rng.integers(0, nb // 2 + 1), replace=False))
    keep_off = np.zeros((nb + 2) * blk, dtype=bool)
    for b in Is:
        keep_off[b * blk:(b + 1) * blk] = True
    keep_off[:w] = True
    kept = 0
    for bi in range(nb):
        for bj in range(bi + 1):
            lo, hi = max(blk * (bi - bj) - (blk - 1), 0), blk * (bi - bj) + blk - 1
            kept += bool(bj in Ic or keep_off[lo:hi + 1].any())
    assert bench.block_mask_density(S, Ic, Is, w, blk) == pytest.approx(kept / (nb * (nb + 1) / 2.0), rel=1e-12)


@pytest.mark.parametrize("S,seed", [(700, 1), (1024, 2), (2000, 3)])
def test_schedule_slots_match_brute_force(S, seed):
    rng = np.random.default_rng(seed)
    cols = np.sort(rng.choice(S, 150, replace=False))
    offs = np.sort(rng.choice(S, 6, replace=False))
    w = 5
    keep = np.zeros(S, dtype=bool)
    keep[offs] = True
    keep[:w] = True
    slots = 0
    for a in range((S + 255) // 256):
        last = min(256 * a + 255, S - 1)
        n_col = -(-int((cols <= last).sum()) // 64)
        n_rng = 0
        for d in range(4 * a + 4):                      # key tile 4 a + 3 - d >= 0
            lo, hi = max(64 * d - 255, 0), min(64 * d + 63, S - 1)
            n_rng += bool(lo <= hi and keep[lo:hi + 1].any())
        slots += 8 * (n_col + n_rng)
    assert bench.schedule_slots(S, cols, offs, w) == slots
