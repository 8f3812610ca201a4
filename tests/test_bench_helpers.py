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
