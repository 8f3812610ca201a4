"""Pins for the oracle's attention functions (Eq. 1-3 of the paper).

The oracle is pinned to things other than itself: torch's fp64
scaled_dot_product_attention on CPU (a library routine; dense-causal and
banded special cases), pure-Python loops written from the definitions, and
closed forms.
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import sample_attention as O


def _rand(S, d, seed, Hq=1, Hkv=1):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((Hq, S, d)), rng.standard_normal((Hkv, S, d)),
            rng.standard_normal((Hkv, S, d)))


def test_dense_matches_sdpa_fp64_gqa():
    # Eq. 1-2 + causal; GQA mapping h -> h // group is what enable_gqa does.
    Q, K, V = _rand(96, 16, 1, Hq=6, Hkv=2)
    out, _ = O.dense_attn_heads(Q, K, V)
    ref = F.scaled_dot_product_attention(
        torch.from_numpy(Q)[None], torch.from_numpy(K)[None], torch.from_numpy(V)[None],
        is_causal=True, enable_gqa=True)[0].numpy()
    assert np.abs(out - ref).max() < 1e-12


def test_dense_explicit_scale_and_default():
    Q, K, V = _rand(40, 8, 2)
    a, _ = O.dense_attn(Q[0], K[0], V[0])
    b, _ = O.dense_attn(Q[0], K[0], V[0], scale=1.0 / math.sqrt(8))
    c, _ = O.dense_attn(Q[0], K[0], V[0], scale=0.5)
    ref = F.scaled_dot_product_attention(
        torch.from_numpy(Q), torch.from_numpy(K), torch.from_numpy(V), is_causal=True, scale=0.5)[0].numpy()
    assert np.array_equal(a, b)
    assert np.abs(c - ref).max() < 1e-12


def test_dense_pure_python_loops():
    # Eq. 1-2 written out with scalar loops (no numpy in the arithmetic).
    S, d = 9, 3
    Q, K, V = _rand(S, d, 3)
    q, k, v = Q[0].tolist(), K[0].tolist(), V[0].tolist()
    out, lse = O.dense_attn(Q[0], K[0], V[0])
    for i in range(S):
        s = [sum(q[i][c] * k[j][c] for c in range(d)) / math.sqrt(d) for j in range(i + 1)]
        z = sum(math.exp(x) for x in s)
        for c in range(d):
            o = sum(math.exp(s[j]) / z * v[j][c] for j in range(i + 1))
            assert abs(o - out[i, c]) < 1e-12
        assert abs(math.log(z) - lse[i]) < 1e-12


def test_dense_row0_and_constant_values():
    Q, K, V = _rand(33, 8, 4)
    out, lse = O.dense_attn(Q[0], K[0], V[0])
    # row 0 sees only key 0
    assert np.allclose(out[0], V[0][0], atol=1e-14)
    assert abs(lse[0] - (Q[0][0] @ K[0][0]) / math.sqrt(8)) < 1e-13
    # a constant V is reproduced by any softmax (rows sum to one)
    ones = np.ones_like(V[0])
    o1, _ = O.dense_attn(Q[0], K[0], ones)
    assert np.abs(o1 - 1.0).max() < 1e-13


def test_dense_row_subset_equals_full():
    Q, K, V = _rand(70, 8, 5)
    full, lf = O.dense_attn(Q[0], K[0], V[0])
    rows = np.array([0, 3, 17, 69])
    sub, ls = O.dense_attn(Q[0], K[0], V[0], rows=rows)
    assert np.array_equal(full[rows], sub) and np.array_equal(lf[rows], ls)


# ---------------------------------------------------------------- Eq. 3 ----
def test_masked_all_strips_is_dense():
    # alpha = 1 keeps every column and every offset -> full causal mask.
    Q, K, V = _rand(50, 8, 6)
    allidx = np.arange(50)
    a, la = O.masked_attn(Q[0], K[0], V[0], allidx, allidx, 1)
    b, lb = O.dense_attn(Q[0], K[0], V[0])
    assert np.abs(a - b).max() < 1e-12 and np.abs(la - lb).max() < 1e-12
    # either direction alone already covers the triangle
    c, _ = O.masked_attn(Q[0], K[0], V[0], allidx, [], 1)
    e, _ = O.masked_attn(Q[0], K[0], V[0], [], allidx, 1)
    assert np.abs(c - b).max() < 1e-12 and np.abs(e - b).max() < 1e-12


@pytest.mark.parametrize("w", [1, 4, 13])
def test_masked_no_strips_is_sliding_window(w):
    # alpha = 0: only the local window survives -> textbook band attention.
    S, d = 41, 8
    Q, K, V = _rand(S, d, 7)
    got, _ = O.masked_attn(Q[0], K[0], V[0], [], [], w)
    i = torch.arange(S)[:, None]
    j = torch.arange(S)[None, :]
    band = (j <= i) & (i - j < w)
    ref = F.scaled_dot_product_attention(
        torch.from_numpy(Q), torch.from_numpy(K), torch.from_numpy(V), attn_mask=band[None])[0].numpy()
    assert np.abs(got - ref).max() < 1e-12


def test_masked_vs_explicit_mask_sdpa():
    # column strips, slash strips and the window together, against SDPA with
    # the boolean mask built here by scalar loops from the definition.
    S, d, w = 37, 8, 3
    Q, K, V = _rand(S, d, 8)
    Ic, Is = [0, 5, 20], [7, 9, 30]
    M = torch.zeros(S, S, dtype=torch.bool)
    for i in range(S):
        for j in range(S):
            M[i, j] = (j <= i) and ((j in Ic) or ((i - j) in Is) or (i - j < w))
    got, _ = O.masked_attn(Q[0], K[0], V[0], Ic, Is, w)
    ref = F.scaled_dot_product_attention(
        torch.from_numpy(Q), torch.from_numpy(K), torch.from_numpy(V), attn_mask=M[None])[0].numpy()
    assert np.abs(got - ref).max() < 1e-12
    assert np.array_equal(O.strip_mask(S, Ic, Is, w, np.arange(S)), M.numpy())


def test_masked_row_equals_softmax_over_deleted_keys():
    # physically delete the masked keys of one row and run plain softmax.
    S, d, w = 64, 8, 2
    Q, K, V = _rand(S, d, 9)
    Ic, Is = [1, 10, 40], [5, 33]
    i = 50
    keep = [j for j in range(i + 1) if (j in Ic) or ((i - j) in Is) or (i - j < w)]
    s = (K[0][keep] @ Q[0][i]) / math.sqrt(d)
    p = np.exp(s - s.max())
    p /= p.sum()
    ref = p @ V[0][keep]
    got, _ = O.masked_attn(Q[0], K[0], V[0], Ic, Is, w, rows=[i])
    assert np.abs(got[0] - ref).max() < 1e-13


def test_mask_density_and_blocks_bruteforce():
    S, w = 300, 5
    rng = np.random.default_rng(10)
    Ic = np.sort(rng.choice(S, 17, replace=False))
    Is = np.sort(rng.choice(S, 11, replace=False))
    M = O.strip_mask(S, Ic, Is, w, np.arange(S))
    assert abs(O.mask_density(S, Ic, Is, w) - M.sum() / (S * (S + 1) / 2)) < 1e-15
    blk = 32
    nb = (S + blk - 1) // blk
    touched = total = 0
    for a in range(nb):
        for t in range(a + 1):
            total += 1
            touched += bool(M[a * blk:(a + 1) * blk, t * blk:(t + 1) * blk].any())
    assert abs(O.touched_block_fraction(S, Ic, Is, w, blk) - touched / total) < 1e-15


def test_recall_is_kept_mass():
    S, d, w = 48, 8, 2
    Q, K, V = _rand(S, d, 11)
    Ic, Is = [0, 3], [6]
    rows = np.arange(S)
    diag = O.mask_diagnostics(Q[0], K[0], Ic, Is, w, rows)
    P = F.softmax(torch.from_numpy(Q[0] @ K[0].T / math.sqrt(d)).masked_fill(
        ~torch.tril(torch.ones(S, S, dtype=torch.bool)), -math.inf), dim=-1).numpy()
    M = O.strip_mask(S, Ic, Is, w, rows)
    rec = (P * M).sum(1)
    assert abs(diag["cra_min"] - rec.min()) < 1e-13
    assert abs(diag["recall_mean"] - rec.mean()) < 1e-13
    assert rec.max() <= 1 + 1e-13
    full = O.mask_diagnostics(Q[0], K[0], np.arange(S), [], w, rows)
    assert abs(full["cra_min"] - 1.0) < 1e-13 and abs(full["density"] - 1.0) < 1e-15
