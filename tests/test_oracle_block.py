"""Pins for the oracle's block-granularity functions (Alg. 1 with blk > 1).

Pinned to things other than themselves: the strip functions at blk = 1, sums
over an explicit probability matrix built with scalar loops, a pure-Python
cover of the token-level bands, torch's fp64 scaled_dot_product_attention
with an explicit block mask, and the dense result at alpha = 1.
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import sample_attention as O


def _rand(S, d, seed):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((S, d)), rng.standard_normal((S, d)), rng.standard_normal((S, d))


def _explicit_p(q, k, rows):
    """Causal softmax rows with scalar loops (Eq. 1 + causal mask)."""
    S, d = len(k), len(k[0])
    P = [[0.0] * S for _ in rows]
    for n, i in enumerate(rows):
        s = [sum(q[i][c] * k[j][c] for c in range(d)) / math.sqrt(d) for j in range(i + 1)]
        z = sum(math.exp(x) for x in s)
        for j in range(i + 1):
            P[n][j] = math.exp(s[j]) / z
    return P


@pytest.mark.parametrize("S,blk,n_s", [(24, 4, 8), (23, 4, 5), (30, 8, 30)])
def test_block_scores_from_explicit_matrix(S, blk, n_s):
    # block_reduction of Alg. 1: the sampled probabilities summed over blocks
    # of blk keys, and over blocks of blk offsets i - j
    q, k, _ = _rand(S, 4, 11)
    rows = list(range(S - n_s, S))
    P = _explicit_p(q.tolist(), k.tolist(), rows)
    nb = (S + blk - 1) // blk
    A_c = [0.0] * nb
    A_s = [0.0] * nb
    for n, i in enumerate(rows):
        for j in range(i + 1):
            A_c[j // blk] += P[n][j]
            A_s[(i - j) // blk] += P[n][j]
    col, slash, _ = O.sample_scores(q, k, n_s)
    assert np.abs(O.block_reduce(col, blk) - np.array(A_c)).max() < 1e-12
    assert np.abs(O.block_reduce(slash, blk) - np.array(A_s)).max() < 1e-12
    assert abs(O.block_reduce(col, blk).sum() - n_s) < 1e-9
    assert abs(O.block_reduce(slash, blk).sum() - n_s) < 1e-9


def test_block_reduce_ragged_and_blk1():
    x = np.arange(1.0, 11.0)
    assert O.block_reduce(x, 4).tolist() == [10.0, 26.0, 19.0]
    assert O.block_reduce(x, 1).tolist() == x.tolist()
    assert O.block_reduce(x, 16).tolist() == [55.0]
    with pytest.raises(ValueError):
        O.block_reduce(x, 0)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_blk1_is_the_strip_mask(seed):
    rng = np.random.default_rng(seed)
    S = 41
    Ic = np.sort(rng.choice(S, 6, replace=False))
    Is = np.sort(rng.choice(S, 5, replace=False))
    w = int(rng.integers(1, 5))
    rows = np.arange(S)
    assert np.array_equal(O.block_mask(S, Ic, Is, w, 1, rows), O.strip_mask(S, Ic, Is, w, rows))
    q, k, v = _rand(S, 8, seed)
    a, la = O.block_masked_attn(q, k, v, Ic, Is, w, 1)
    b, lb = O.masked_attn(q, k, v, Ic, Is, w)
    assert np.abs(a - b).max() < 1e-12 and np.abs(la - lb).max() < 1e-12


@pytest.mark.parametrize("S,blk,w,seed", [(48, 4, 1, 0), (48, 4, 4, 1), (64, 8, 3, 2), (45, 4, 6, 3), (40, 8, 20, 4)])
def test_block_mask_is_the_block_cover_of_the_bands(S, blk, w, seed):
    # token-level pattern: selected key blocks as columns, selected offset
    # blocks as bands of blk diagonals, the window.  Every full block of the
    # causal part that holds one of its pairs must be kept entirely, every
    # full block that holds none must be dropped entirely.
    rng = np.random.default_rng(seed)
    nb = (S + blk - 1) // blk
    Ic = np.sort(rng.choice(nb, 2, replace=False))
    Is = np.sort(rng.choice(nb, 2, replace=False))
    M = O.block_mask(S, Ic, Is, w, blk, np.arange(S))
    tok = [[False] * S for _ in range(S)]
    for i in range(S):
        for j in range(i + 1):
            o = i - j
            tok[i][j] = (j // blk in Ic) or (o // blk in Is) or (o < w)
    for i in range(S):
        for j in range(S):
            if j > i:
                assert not M[i, j]
            elif tok[i][j]:
                assert M[i, j]          # the cover loses no pair of the pattern
    for a in range(S // blk):           # full row blocks
        for t in range(a + 1):          # full column blocks (t <= a < S // blk)
            # a block strictly below the diagonal holds every pair; the pattern
            # of such a block depends on (t, a - t) only
            if t == a:
                continue
            pairs = [(i, j) for i in range(a * blk, (a + 1) * blk) for j in range(t * blk, (t + 1) * blk)]
            holds = any(tok[i][j] for i, j in pairs)
            vals = {bool(M[i, j]) for i, j in pairs}
            assert vals == {holds}
    # the diagonal blocks hold offset 0 (window >= 1): kept, causal part only
    for i in range(S):
        for j in range((i // blk) * blk, i + 1):
            assert M[i, j]


def test_block_diagonals_window_and_neighbours():
    # blk = 128, w = 128: offsets 0..127 lie in the diagonal block and in the
    # block left of it; a selected offset block b lies on block diagonals b, b+1
    assert O.block_diagonals(1024, [], 128, 128).nonzero()[0].tolist() == [0, 1]
    assert O.block_diagonals(1024, [], 1, 128).nonzero()[0].tolist() == [0]
    assert O.block_diagonals(1024, [], 129, 128).nonzero()[0].tolist() == [0, 1]
    assert O.block_diagonals(1024, [], 130, 128).nonzero()[0].tolist() == [0, 1, 2]
    assert O.block_diagonals(1024, [3, 4], 1, 128).nonzero()[0].tolist() == [0, 3, 4, 5]
    assert O.block_diagonals(1024, [7], 1, 128).nonzero()[0].tolist() == [0, 7]   # 8 does not exist


def test_block_masked_attn_matches_sdpa_with_explicit_mask():
    S, d, blk = 56, 16, 8
    q, k, v = _rand(S, d, 5)
    Ic, Is, w = [0, 3], [2], 5
    out, lse = O.block_masked_attn(q, k, v, Ic, Is, w, blk)
    # the mask written out independently from block indices
    keep = torch.zeros(S, S, dtype=torch.bool)
    diag = {0, 1, 2, 3}     # window 5 -> diagonals 0, 1; offset block 2 -> 2, 3
    for i in range(S):
        for j in range(i + 1):
            keep[i, j] = (j // blk in Ic) or ((i // blk - j // blk) in diag)
    ref = F.scaled_dot_product_attention(torch.from_numpy(q)[None], torch.from_numpy(k)[None],
                                         torch.from_numpy(v)[None], attn_mask=keep[None])[0].numpy()
    assert np.abs(out - ref).max() < 1e-12
    s = (q @ k.T) / math.sqrt(d)
    s[~keep.numpy()] = -np.inf
    assert np.abs(lse - np.log(np.exp(s).sum(axis=1))).max() < 1e-12


def test_block_alpha_one_is_dense_and_alpha_zero_is_block_window():
    S, d, blk = 40, 8, 8
    q, k, v = _rand(S, d, 6)
    r = O.block_sample_attention(q, k, v, 8, 1.0, 1.0, 1, blk)
    dense, _ = O.dense_attn(q, k, v)
    assert np.abs(r["out"] - dense).max() < 1e-12
    assert r["col_blocks"].tolist() == list(range(5))
    r0 = O.block_sample_attention(q, k, v, 8, 0.0, 0.0, 1, blk)
    assert len(r0["col_blocks"]) == 0 and len(r0["slash_blocks"]) == 0
    # window 1 at alpha 0: only the diagonal blocks -> attention within the own block
    for i in range(S):
        lo = (i // blk) * blk
        o, _ = O.dense_attn(q[lo:], k[lo:], v[lo:], rows=[i - lo])
        assert np.abs(r0["out"][i] - o[0]).max() < 1e-12


def test_block_selection_reaches_alpha_of_sampled_mass():
    S, d, blk, n_s = 64, 8, 8, 16
    q, k, v = _rand(S, d, 7)
    r = O.block_sample_attention(q, k, v, n_s, 0.7, 0.6, 1, blk)
    A_c, A_s = r["col_block_scores"], r["slash_block_scores"]
    assert A_c[r["col_blocks"]].sum() >= 0.7 * n_s - 1e-9
    assert A_s[r["slash_blocks"]].sum() >= 0.6 * n_s - 1e-9
    # dropping the weakest chosen block falls below the threshold
    assert A_c[r["col_blocks"]].sum() - A_c[r["col_blocks"]].min() < 0.7 * n_s
    assert A_s[r["slash_blocks"]].sum() - A_s[r["slash_blocks"]].min() < 0.6 * n_s


def test_block_mask_density_counts_blocks():
    S, blk = 64, 8
    Ic, Is, w = [1], [3], 1
    M = O.block_mask(S, Ic, Is, w, blk, np.arange(S))
    nb = S // blk
    kept = sum(1 for a in range(nb) for t in range(a + 1) if M[a * blk + blk - 1, t * blk])
    assert O.block_mask_density(S, Ic, Is, w, blk) == kept / (nb * (nb + 1) / 2)
