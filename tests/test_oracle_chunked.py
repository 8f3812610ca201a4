"""Pins for the oracle's chunk_n > 1 functions (Alg. 1 stage 1, Q_slice with
itv = S_q / chunk_n; merge_index with itv).

Pinned to things other than themselves: chunk_n = 1 reproduces the functions
pinned elsewhere; the scores of chunk m are those of the (separately pinned)
single-chunk function on the prefix that ends with the chunk's segment; sums
over an explicit probability matrix built with scalar loops; the masked rows
against torch's fp64 scaled_dot_product_attention with a mask written out
row by row.
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


def test_segments():
    assert O.chunk_segments(12, 3) == [(0, 4), (4, 8), (8, 12)]
    assert O.chunk_segments(13, 3) == [(0, 4), (4, 8), (8, 13)]      # the last segment takes the remainder
    assert O.chunk_segments(7, 1) == [(0, 7)]
    with pytest.raises(ValueError):
        O.chunk_segments(4, 0)


def test_one_chunk_is_the_plain_path():
    q, k, v = _rand(48, 8, 0)
    col, slash = O.sample_scores_chunked(q, k, 8, 1)
    c1, s1, _ = O.sample_scores(q, k, 8)
    assert np.array_equal(col[0], c1) and np.array_equal(slash[0], s1)
    a = O.chunked_sample_attention(q, k, v, 8, 1, 0.8, 0.7, 2)
    b = O.sample_attention(q, k, v, 8, 0.8, 0.7, 2)
    assert np.array_equal(a["out"], b["out"]) and np.array_equal(a["col_idx"][0], b["col_idx"])


@pytest.mark.parametrize("S,C,n_s", [(48, 3, 4), (50, 4, 5), (64, 2, 32)])
def test_chunk_scores_are_prefix_scores(S, C, n_s):
    # chunk m samples the bottom rows of segment m; being causal, those rows see
    # nothing after the segment: the scores equal those of the sequence cut there
    q, k, _ = _rand(S, 8, 1)
    col, slash = O.sample_scores_chunked(q, k, n_s, C)
    for m, (lo, hi) in enumerate(O.chunk_segments(S, C)):
        c, s, _ = O.sample_scores(q[:hi], k[:hi], n_s)
        assert np.abs(col[m, :hi] - c).max() < 1e-12 and np.abs(slash[m, :hi] - s).max() < 1e-12
        assert not col[m, hi:].any() and not slash[m, hi:].any()
        assert abs(col[m].sum() - n_s) < 1e-9 and abs(slash[m].sum() - n_s) < 1e-9


def test_chunk_scores_scalar_loops():
    S, d, C, n_s = 18, 3, 3, 2
    q, k, _ = _rand(S, d, 2)
    ql, kl = q.tolist(), k.tolist()
    col, slash = O.sample_scores_chunked(q, k, n_s, C)
    itv = S // C
    for m in range(C):
        cc = [0.0] * S
        ss = [0.0] * S
        for i in range((m + 1) * itv - n_s, (m + 1) * itv):
            sc = [sum(ql[i][c] * kl[j][c] for c in range(d)) / math.sqrt(d) for j in range(i + 1)]
            z = sum(math.exp(x) for x in sc)
            for j in range(i + 1):
                cc[j] += math.exp(sc[j]) / z
                ss[i - j] += math.exp(sc[j]) / z
        assert np.abs(col[m] - np.array(cc)).max() < 1e-12
        assert np.abs(slash[m] - np.array(ss)).max() < 1e-12


@pytest.mark.parametrize("blk", [1, 4])
def test_chunked_mask_applies_per_segment(blk):
    S, d, C, w = 40, 8, 4, 2
    q, k, v = _rand(S, d, 3)
    rng = np.random.default_rng(4)
    n = (S + blk - 1) // blk
    Ic = [np.sort(rng.choice(n, 3, replace=False)) for _ in range(C)]
    Is = [np.sort(rng.choice(n, 2, replace=False)) for _ in range(C)]
    out, lse = O.chunked_masked_attn(q, k, v, Ic, Is, w, C, blk=blk)
    keep = torch.zeros(S, S, dtype=torch.bool)
    itv = S // C
    for i in range(S):
        m = min(i // itv, C - 1)
        if blk == 1:
            for j in range(i + 1):
                keep[i, j] = (j in Ic[m]) or ((i - j) in Is[m]) or (i - j < w)
        else:
            diag = set()
            for b in Is[m]:
                diag |= {int(b), int(b) + 1}
            diag |= {dd for dd in range(n) if blk * dd - (blk - 1) <= w - 1}
            for j in range(i + 1):
                keep[i, j] = (j // blk in Ic[m]) or ((i // blk - j // blk) in diag)
    ref = F.scaled_dot_product_attention(torch.from_numpy(q)[None], torch.from_numpy(k)[None],
                                         torch.from_numpy(v)[None], attn_mask=keep[None])[0].numpy()
    assert np.abs(out - ref).max() < 1e-12
    # a subset of rows gives the same rows
    sub = np.array([0, 9, 10, 25, 39])
    o2, l2 = O.chunked_masked_attn(q, k, v, Ic, Is, w, C, rows=sub, blk=blk)
    assert np.abs(o2 - out[sub]).max() < 1e-12 and np.abs(l2 - lse[sub]).max() < 1e-12


def test_chunked_pipeline_alpha_one_is_dense_and_mass():
    S, d, C, n_s = 48, 8, 3, 4
    q, k, v = _rand(S, d, 5)
    r = O.chunked_sample_attention(q, k, v, n_s, C, 1.0, 1.0, 1)
    dense, _ = O.dense_attn(q, k, v)
    assert np.abs(r["out"] - dense).max() < 1e-12
    r = O.chunked_sample_attention(q, k, v, n_s, C, 0.7, 0.6, 1)
    for m in range(C):
        assert r["col"][m][r["col_idx"][m]].sum() >= 0.7 * n_s - 1e-9
        assert r["slash"][m][r["slash_idx"][m]].sum() >= 0.6 * n_s - 1e-9
        # a chunk never selects a key or an offset its sampled rows cannot see
        hi = O.chunk_segments(S, C)[m][1]
        assert (r["col_idx"][m] < hi).all() and (r["slash_idx"][m] < hi).all()
