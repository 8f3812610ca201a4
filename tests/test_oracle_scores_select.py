"""Pins for the oracle's sampling (Alg. 1 stage 1) and selection (stage 2)."""
import itertools
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import sample_attention as O


def _rand(S, d, seed):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((S, d)), rng.standard_normal((S, d))


# ------------------------------------------------------------- stage 1 -----
@pytest.mark.parametrize("S,n_s", [(24, 8), (50, 50), (31, 1)])
def test_scores_bruteforce_from_definition(S, n_s):
    # explicit P by scalar loops, then the two accumulations as defined:
    # col[j] += P[i][j], slash[i - j] += P[i][j] for sampled rows i, j <= i.
    d = 4
    q, k = _rand(S, d, 100 + S)
    P = [[0.0] * S for _ in range(S)]
    for i in range(S):
        s = [sum(q[i][c] * k[j][c] for c in range(d)) / math.sqrt(d) for j in range(i + 1)]
        z = sum(math.exp(x) for x in s)
        for j in range(i + 1):
            P[i][j] = math.exp(s[j]) / z
    col = [0.0] * S
    slash = [0.0] * S
    for i in range(S - n_s, S):
        for j in range(i + 1):
            col[j] += P[i][j]
            slash[i - j] += P[i][j]
    c, s_, lse = O.sample_scores(q, k, n_s)
    assert np.abs(c - np.array(col)).max() < 1e-12
    assert np.abs(s_ - np.array(slash)).max() < 1e-12
    assert lse.shape == (n_s,)


def test_scores_mass_invariants():
    S, n_s = 300, 64
    q, k = _rand(S, 16, 7)
    col, slash, _ = O.sample_scores(q, k, n_s)
    # every sampled softmax row sums to one
    assert abs(col.sum() - n_s) < 1e-9 * n_s
    assert abs(slash.sum() - n_s) < 1e-9 * n_s
    assert (col >= 0).all() and (slash >= 0).all()
    # offset 0 (the diagonal) and the last key only ever receive n_s / 1 terms
    assert slash[0] <= n_s and col[S - 1] <= 1.0


def test_scores_closed_form_harmonic():
    # Q = 0 -> p_ij = 1/(i+1): col[j] = H(S) - H(max(j, S-n_s)), same for slash.
    S, n_s, d = 200, 37, 8
    k = np.random.default_rng(5).standard_normal((S, d))
    q = np.zeros((S, d))
    H = [Fraction(0)]
    for m in range(1, S + 1):
        H.append(H[-1] + Fraction(1, m))
    want = np.array([float(H[S] - H[max(j, S - n_s)]) for j in range(S)])
    col, slash, lse = O.sample_scores(q, k, n_s)
    assert np.abs(col - want).max() < 1e-13
    assert np.abs(slash - want).max() < 1e-13
    assert np.abs(lse - np.log(np.arange(S - n_s, S) + 1.0)).max() < 1e-13


def test_scores_single_dominant_key_fixes_direction():
    # one key with an overwhelming logit at j*: every sampled row puts ~all its
    # mass there, so col[j*] ~ n_s and slash[o] ~ 1 exactly for the offsets
    # o = i - j* of the sampled rows (a sign or transposition error moves them).
    S, n_s, d, js = 128, 16, 8, 37
    q = np.ones((S, d))
    k = np.zeros((S, d))
    k[js] = 40.0
    col, slash, _ = O.sample_scores(q, k, n_s)
    assert abs(col[js] - n_s) < 1e-6
    lo, hi = S - n_s - js, S - 1 - js
    assert np.abs(slash[lo:hi + 1] - 1.0).max() < 1e-6
    assert slash[:lo].max() < 1e-6 and slash[hi + 1:].max() < 1e-6


def test_scores_scale_argument():
    S, n_s, d = 40, 8, 16
    q, k = _rand(S, d, 9)
    a = O.sample_scores(q, k, n_s)
    b = O.sample_scores(q, k, n_s, scale=1.0 / math.sqrt(d))
    c = O.sample_scores(q * 2.0, k, n_s, scale=0.5 / math.sqrt(d))
    assert np.array_equal(a[0], b[0]) and np.abs(a[1] - c[1]).max() < 1e-13


def test_scores_equal_dense_probabilities():
    # same rows through the dense-attention code path with V = identity columns
    S, n_s, d = 48, 12, 8
    q, k = _rand(S, d, 12)
    rows = np.arange(S - n_s, S)
    P, _ = O.dense_attn(q, k, np.eye(S), rows=rows)
    col, slash, _ = O.sample_scores(q, k, n_s)
    assert np.abs(P.sum(0) - col).max() < 1e-13
    want = np.zeros(S)
    for n, i in enumerate(rows):
        for j in range(i + 1):
            want[i - j] += P[n, j]
    assert np.abs(want - slash).max() < 1e-13


# ------------------------------------------------------------- stage 2 -----
def _brute_select(scores, alpha):
    """Exhaustive search: the smallest subset size whose best achievable mass
    reaches alpha * total, and the canonical set of that size."""
    n = len(scores)
    total = sum(Fraction(float(x)) for x in scores)
    target = Fraction(float(alpha)) * total
    if alpha >= 1:
        return list(range(n))
    if target <= 0:
        return []
    for size in range(1, n + 1):
        best = None
        for sub in itertools.combinations(range(n), size):
            if sum(Fraction(float(scores[i])) for i in sub) >= target:
                # canonical: (score desc, index asc) order, lexicographically first
                key = sorted(((-scores[i], i) for i in sub))
                if best is None or key < best[0]:
                    best = (key, sub)
        if best is not None:
            return sorted(best[1])
    return list(range(n))


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("alpha", [0.0, 0.3, 0.5, 0.8, 0.95, 0.999])
def test_select_bruteforce_minimal_and_canonical(seed, alpha):
    rng = np.random.default_rng(seed)
    n = 10
    scores = rng.random(n) ** 3
    if seed % 2:                       # exact ties, to exercise the index tie-break
        scores[rng.integers(0, n, 4)] = scores[0]
    got = O.select(scores, alpha).tolist()
    assert got == _brute_select(scores, alpha)


def test_select_invariants_large():
    rng = np.random.default_rng(3)
    scores = rng.random(5000) ** 8
    for alpha in (0.5, 0.9, 0.95, 0.98):
        idx = O.select(scores, alpha)
        tot = scores.sum()
        kept = np.sort(scores[idx])[::-1]
        assert kept.sum() >= alpha * tot * (1 - 1e-15)
        assert kept[:-1].sum() < alpha * tot          # dropping the weakest breaks it
        rest = np.delete(scores, idx)
        assert rest.max() <= kept.min()               # it is a top-k set
        assert np.all(np.diff(idx) > 0)               # ascending, unique


def test_select_edges():
    s = np.array([0.5, 0.25, 0.25, 0.0])
    assert O.select(s, 0.0).tolist() == []
    assert O.select(s, 1.0).tolist() == [0, 1, 2, 3]
    assert O.select(s, 1.5).tolist() == [0, 1, 2, 3]
    assert O.select(s, 0.5).tolist() == [0]            # ">=": exactly reaching alpha suffices
    assert O.select(s, 0.75).tolist() == [0, 1]        # tie between 1 and 2 -> lower index
    assert O.select(s, 0.76).tolist() == [0, 1, 2]
    assert O.select(np.zeros(5), 0.9).tolist() == []   # no mass: nothing to keep
    assert O.select(np.zeros(0), 0.9).tolist() == []
    with pytest.raises(ValueError):
        O.select(s, -0.1)


def test_select_ties_harmonic_case():
    # Q = 0 makes all columns j <= S - n_s tie exactly: the kept ones must be
    # the lowest indices among the tied.
    S, n_s = 64, 8
    q = np.zeros((S, 4))
    k = np.ones((S, 4))
    col, _, _ = O.sample_scores(q, k, n_s)
    idx = O.select(col, 0.5)
    assert np.array_equal(idx, np.arange(len(idx)))


# ------------------------------------------------------------ pipeline -----
def test_pipeline_selected_mass_and_alpha_one():
    S, d, n_s, w = 256, 16, 64, 8
    rng = np.random.default_rng(21)
    q = rng.standard_normal((S, d))
    k = rng.standard_normal((S, d))
    v = rng.standard_normal((S, d))
    k[[0, 77, 150]] *= 4.0
    res = O.sample_attention(q, k, v, n_s, 0.9, 0.9, w)
    assert res["col"][res["col_idx"]].sum() >= 0.9 * res["col"].sum() * (1 - 1e-15)
    assert res["slash"][res["slash_idx"]].sum() >= 0.9 * res["slash"].sum() * (1 - 1e-15)
    full = O.sample_attention(q, k, v, n_s, 1.0, 1.0, w)
    dense, _ = O.dense_attn(q, k, v)
    assert np.abs(full["out"] - dense).max() < 1e-12
    # aggregate recall on the sampled rows is at least each direction's alpha
    rows = np.arange(S - n_s, S)
    P, _ = O.dense_attn(q, k, np.eye(S), rows=rows)
    M = O.strip_mask(S, res["col_idx"], res["slash_idx"], w, rows)
    assert (P * M).sum() >= 0.9 * n_s
