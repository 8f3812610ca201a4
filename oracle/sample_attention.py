"""Plain fp64 CPU oracle for the SampleAttention prefill hot path.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this module;
it exists so that tests, the smoke check and the benchmark's CPU-baseline leg
have an independent, slow, obviously-correct statement of what the GPU kernels
must compute.  It shares no code with the HIP path.

Everything is per attention head unless a function says otherwise:
``q`` is [S, d], ``k`` and ``v`` are [S, d]; inputs of any float dtype are
upcast to float64 and all arithmetic is float64.  Rows are processed in chunks
only to bound memory; the chunking does not change any formula.

What follows the paper, and where:

* ``dense_attn``      - Eq. 1-2 (softmax(QK^T/sqrt(d)) V) with the causal mask
                        of Alg. 1 stage 1 / Sec. 5.1 (decoder-only models).
* ``sample_scores``   - Alg. 1 stage 1 and Sec. 4.2: exact causal softmax rows
                        of the sampled queries, accumulated down every key
                        column and along every diagonal ("slash").
* ``select``          - Alg. 1 stage 2 and Sec. 4.3: sort, cumulative sum,
                        smallest k reaching the CRA threshold, top-k indices.
* ``strip_mask``      - Alg. 1 ``merge_index`` / Fig. 6 caption: column and
                        slash indices extended over the whole matrix and OR-ed.
* ``masked_attn``     - Eq. 3 with c -> infinity (masked entries are exactly 0).
* ``sample_attention``- Alg. 1 end to end (chunk_n = 1).
* ``block_reduce``, ``block_mask``, ``block_masked_attn``,
  ``block_sample_attention`` - the same algorithm at block granularity
                        (Alg. 1 ``block_reduction`` with blk = 128, block
                        filtering of Sec. 4.3, block-sparse mask of Fig. 6).
* ``mask_diagnostics``- Sec. 3.3 (CRA = minimum kept probability mass over
                        queries) and Sec. 2.3 (sparsity ratio).

* ``chunk_segments``, ``sample_scores_chunked``, ``chunked_masked_attn``,
  ``chunked_sample_attention`` - chunk_n > 1 (Alg. 1 stage 1 ``Q_slice``,
                        Sec. 4.2 "Query-Guided Chunked Sampling"): the queries are
                        cut into chunk_n equal segments, the rows at the bottom of
                        each segment are sampled, and what is selected from a
                        chunk's scores masks the rows of that chunk's segment
                        (``merge_index(I_c, I_s, itv)``; Fig. 6 caption: one set of
                        strips "for each sampling region").

Readings where the paper is silent (all listed again in the design notes):
sort is descending; alpha is a fraction of the direction's total sampled mass;
the cut uses ">="; alpha = 0 keeps nothing, alpha >= 1 keeps everything; ties
go to the lower index; column j extends to all rows i >= j and offset o to all
rows i >= o; the local window [0, w) is OR-ed in after selection; scores are
kept per key / per offset (granularity 1) and per query head.  At block
granularity the token-level column scores are summed over blocks of blk keys
and the token-level slash scores over blocks of blk offsets; a selected block
of offsets, extended over the matrix, is a band of blk diagonals, and the block
mask keeps every blk x blk block (by block row and block column) that holds at
least one pair (i, j) of a selected key block, of such a band, or of the local
window, decided from the block indices alone (so the mask of a block depends
only on its block column and on block row minus block column).

With chunk_n > 1: itv = S // chunk_n, segment m holds the rows [m itv, (m+1) itv)
(the last one up to S), its sampled rows are the last n_s rows of the segment, and
their softmax is causal as everywhere (keys j <= i).

Pins (tests/test_oracle_*.py): fp64 ``scaled_dot_product_attention`` on CPU for
dense and banded cases, pure-Python brute force from the definitions on small
inputs, the harmonic-number closed form for Q = 0, exhaustive subset
enumeration for the selection, alpha = 1 == dense, alpha = 0 == sliding window;
for the block functions: blk = 1 reproduces the strip functions, block scores
against sums over the explicit probability matrix, the block mask against a
pure-Python cover of the token-level bands (kept blocks touch them, dropped
blocks do not).
"""
from __future__ import annotations

import math
from typing import Dict, Optional, Sequence, Tuple

import numpy as np

ROW_CHUNK_ELEMS = 1 << 25  # score elements held at once (fp64: 256 MiB)


def _f64(x) -> np.ndarray:
    return np.asarray(x, dtype=np.float64)


def _scale(d: int, scale: Optional[float]) -> float:
    return 1.0 / math.sqrt(d) if (scale is None or scale == 0.0) else float(scale)


def _chunks(rows: np.ndarray, S: int):
    step = max(1, ROW_CHUNK_ELEMS // max(S, 1))
    for s in range(0, len(rows), step):
        yield rows[s:s + step]


def _causal_softmax_rows(q, k, rows, scale, allowed=None):
    """Exact softmax of the given query rows over keys j <= i (Eq. 1 + causal).

    ``allowed`` (bool [len(rows), S], optional) further restricts the keys
    (Eq. 3 with c -> infinity).  Returns (p [len(rows), S], lse [len(rows)]).
    """
    S = k.shape[0]
    s = (q[rows] @ k.T) * scale
    keep = np.arange(S)[None, :] <= rows[:, None]
    if allowed is not None:
        keep &= allowed
    s = np.where(keep, s, -np.inf)
    m = s.max(axis=1, keepdims=True)
    e = np.exp(s - m)
    z = e.sum(axis=1, keepdims=True)
    return e / z, (m + np.log(z))[:, 0]


# ----------------------------------------------------------------------------
# Eq. 1-2: dense causal attention
# ----------------------------------------------------------------------------
def dense_attn(q, k, v, scale: Optional[float] = None, rows=None) -> Tuple[np.ndarray, np.ndarray]:
    """O = softmax(Q K^T / sqrt(d)) V with keys j <= i, for the listed rows.

    Returns (O [n_rows, d], lse [n_rows]) where lse_i = log sum_j exp(s_ij).
    """
    q, k, v = _f64(q), _f64(k), _f64(v)
    S, d = k.shape
    sc = _scale(d, scale)
    rows = np.arange(q.shape[0]) if rows is None else np.asarray(rows, dtype=np.int64)
    out = np.empty((len(rows), v.shape[1]))
    lse = np.empty(len(rows))
    at = 0
    for r in _chunks(rows, S):
        p, l = _causal_softmax_rows(q, k, r, sc)
        out[at:at + len(r)] = p @ v
        lse[at:at + len(r)] = l
        at += len(r)
    return out, lse


# ----------------------------------------------------------------------------
# Alg. 1 stage 1: sampled rows -> column and slash scores
# ----------------------------------------------------------------------------
def sampled_rows(S: int, n_sample_rows: int) -> np.ndarray:
    """chunk_n = 1: the last ``n_sample_rows`` query rows (Alg. 1, Q_slice)."""
    if not (1 <= n_sample_rows <= S):
        raise ValueError("n_sample_rows must be in [1, S]")
    return np.arange(S - n_sample_rows, S, dtype=np.int64)


def sample_scores(q, k, n_sample_rows: int, scale: Optional[float] = None):
    """Column and slash scores of the sampled rows R (Alg. 1 stage 1).

    col[j]   = sum_{i in R, i >= j} p_ij
    slash[o] = sum_{i in R, i >= o} p_{i, i-o}          (offset o = i - j)
    with p_i the exact causal softmax row of query i.  Plain sums, no
    normalisation.  Returns (col [S], slash [S], lse [n_sample_rows]).
    """
    q, k = _f64(q), _f64(k)
    S, d = k.shape
    sc = _scale(d, scale)
    R = sampled_rows(S, n_sample_rows)
    col = np.zeros(S)
    slash = np.zeros(S)
    lse = np.empty(len(R))
    at = 0
    for r in _chunks(R, S):
        p, l = _causal_softmax_rows(q, k, r, sc)
        col += p.sum(axis=0)
        for n, i in enumerate(r):
            # keys j = i, i-1, ..., 0 are offsets o = 0, 1, ..., i
            slash[: i + 1] += p[n, i::-1]
        lse[at:at + len(r)] = l
        at += len(r)
    return col, slash, lse


# ----------------------------------------------------------------------------
# Alg. 1 stage 2: CRA cut and top-k
# ----------------------------------------------------------------------------
def select(scores, alpha: float) -> np.ndarray:
    """Fewest strips whose score mass reaches alpha * total (Alg. 1 stage 2).

    Order candidates by (score descending, index ascending); prefix_k is the
    sum of the first k; k = min{k >= 0 : prefix_k >= alpha * total}; alpha >= 1
    keeps all.  Returns the chosen indices in ascending order (int64).
    """
    s = _f64(scores)
    n = s.shape[0]
    alpha = float(alpha)
    if not (0.0 <= alpha):
        raise ValueError("alpha must be >= 0")
    if alpha >= 1.0:
        return np.arange(n, dtype=np.int64)
    order = np.argsort(-s, kind="stable")          # ties keep index order
    prefix = np.cumsum(s[order])                   # sequential fp64 sums
    total = prefix[-1] if n else 0.0
    target = alpha * total
    if target <= 0.0:
        return np.zeros(0, dtype=np.int64)
    kk = int(np.searchsorted(prefix, target, side="left")) + 1
    kk = min(kk, n)
    return np.sort(order[:kk]).astype(np.int64)


# ----------------------------------------------------------------------------
# merge_index + Eq. 3
# ----------------------------------------------------------------------------
def strip_mask(S: int, col_idx, slash_idx, window: int, rows) -> np.ndarray:
    """M[i, j] = (j <= i) and (j in I_c or (i - j) in I_s or i - j < window)."""
    rows = np.asarray(rows, dtype=np.int64)
    col_keep = np.zeros(S, dtype=bool)
    col_keep[np.asarray(col_idx, dtype=np.int64)] = True
    off_keep = np.zeros(S, dtype=bool)
    off_keep[np.asarray(slash_idx, dtype=np.int64)] = True
    off_keep[: max(int(window), 0)] = True
    M = np.zeros((len(rows), S), dtype=bool)
    for n, i in enumerate(rows):
        M[n, : i + 1] = col_keep[: i + 1] | off_keep[i::-1][: i + 1]
    return M


def masked_attn(q, k, v, col_idx, slash_idx, window: int,
                scale: Optional[float] = None, rows=None):
    """Eq. 3 with the strip mask: softmax over {j : M_ij} exactly, then P V.

    Returns (O [n_rows, d], lse [n_rows]).
    """
    q, k, v = _f64(q), _f64(k), _f64(v)
    S, d = k.shape
    sc = _scale(d, scale)
    if window < 1:
        raise ValueError("window must be >= 1 (every row keeps its diagonal)")
    rows = np.arange(q.shape[0]) if rows is None else np.asarray(rows, dtype=np.int64)
    out = np.empty((len(rows), v.shape[1]))
    lse = np.empty(len(rows))
    at = 0
    for r in _chunks(rows, 2 * S):
        M = strip_mask(S, col_idx, slash_idx, window, r)
        p, l = _causal_softmax_rows(q, k, r, sc, allowed=M)
        out[at:at + len(r)] = p @ v
        lse[at:at + len(r)] = l
        at += len(r)
    return out, lse


def sample_attention(q, k, v, n_sample_rows: int, alpha_c: float, alpha_s: float,
                     window: int, scale: Optional[float] = None, rows=None) -> Dict[str, np.ndarray]:
    """Alg. 1 end to end for one head with chunk_n = 1."""
    col, slash, lse_s = sample_scores(q, k, n_sample_rows, scale)
    I_c = select(col, alpha_c)
    I_s = select(slash, alpha_s)
    out, lse = masked_attn(q, k, v, I_c, I_s, window, scale, rows)
    return {"out": out, "lse": lse, "col": col, "slash": slash,
            "col_idx": I_c, "slash_idx": I_s, "sample_lse": lse_s}


# ----------------------------------------------------------------------------
# Block granularity (Alg. 1 block_reduction, blk = 128 in the paper)
# ----------------------------------------------------------------------------
def block_reduce(scores, blk: int) -> np.ndarray:
    """A[b] = sum of scores[b*blk : (b+1)*blk] (the last block may be short)."""
    s = _f64(scores)
    if blk < 1:
        raise ValueError("blk must be >= 1")
    nb = (len(s) + blk - 1) // blk
    return np.array([s[b * blk:(b + 1) * blk].sum() for b in range(nb)])


def block_diagonals(S: int, slash_blocks, window: int, blk: int) -> np.ndarray:
    """bool [n_blocks]: block diagonal delta (= block row - block column) is
    kept when a full blk x blk block on it, which spans the offsets
    blk*delta - (blk-1) .. blk*delta + (blk-1), holds a kept offset: one of a
    selected offset block [blk*b, blk*b + blk) or of the window [0, w)."""
    nb = (S + blk - 1) // blk
    off_keep = np.zeros((nb + 2) * blk, dtype=bool)
    for b in np.asarray(slash_blocks, dtype=np.int64):
        off_keep[b * blk:(b + 1) * blk] = True
    off_keep[: max(int(window), 0)] = True
    keep = np.zeros(nb, dtype=bool)
    for delta in range(nb):
        lo, hi = max(blk * delta - (blk - 1), 0), blk * delta + (blk - 1)
        keep[delta] = off_keep[lo:hi + 1].any()
    return keep


def block_mask(S: int, col_blocks, slash_blocks, window: int, blk: int, rows) -> np.ndarray:
    """M[i, j] = (j <= i) and (block(j) in I_c or block(i) - block(j) on a kept
    block diagonal), block(x) = x // blk."""
    rows = np.asarray(rows, dtype=np.int64)
    nb = (S + blk - 1) // blk
    col_keep = np.zeros(nb, dtype=bool)
    col_keep[np.asarray(col_blocks, dtype=np.int64)] = True
    diag_keep = block_diagonals(S, slash_blocks, window, blk)
    jb = np.arange(S) // blk
    M = np.zeros((len(rows), S), dtype=bool)
    for n, i in enumerate(rows):
        ok = col_keep[jb[: i + 1]] | diag_keep[i // blk - jb[: i + 1]]
        M[n, : i + 1] = ok
    return M


def block_masked_attn(q, k, v, col_blocks, slash_blocks, window: int, blk: int,
                      scale: Optional[float] = None, rows=None):
    """Eq. 3 with the block mask.  Returns (O [n_rows, d], lse [n_rows])."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    S, d = k.shape
    sc = _scale(d, scale)
    if window < 1:
        raise ValueError("window must be >= 1 (every row keeps its diagonal)")
    rows = np.arange(q.shape[0]) if rows is None else np.asarray(rows, dtype=np.int64)
    out = np.empty((len(rows), v.shape[1]))
    lse = np.empty(len(rows))
    at = 0
    for r in _chunks(rows, 2 * S):
        M = block_mask(S, col_blocks, slash_blocks, window, blk, r)
        p, l = _causal_softmax_rows(q, k, r, sc, allowed=M)
        out[at:at + len(r)] = p @ v
        lse[at:at + len(r)] = l
        at += len(r)
    return out, lse


def block_sample_attention(q, k, v, n_sample_rows: int, alpha_c: float, alpha_s: float,
                           window: int, blk: int, scale: Optional[float] = None,
                           rows=None) -> Dict[str, np.ndarray]:
    """Alg. 1 end to end for one head with chunk_n = 1 at block granularity."""
    col, slash, lse_s = sample_scores(q, k, n_sample_rows, scale)
    A_c, A_s = block_reduce(col, blk), block_reduce(slash, blk)
    I_c = select(A_c, alpha_c)
    I_s = select(A_s, alpha_s)
    out, lse = block_masked_attn(q, k, v, I_c, I_s, window, blk, scale, rows)
    return {"out": out, "lse": lse, "col_block_scores": A_c, "slash_block_scores": A_s,
            "col_blocks": I_c, "slash_blocks": I_s, "sample_lse": lse_s}


def block_mask_density(S: int, col_blocks, slash_blocks, window: int, blk: int) -> float:
    """Kept fraction of the blk x blk blocks of the causal triangle."""
    nb = (S + blk - 1) // blk
    col_keep = np.zeros(nb, dtype=bool)
    col_keep[np.asarray(col_blocks, dtype=np.int64)] = True
    diag_keep = block_diagonals(S, slash_blocks, window, blk)
    kept = 0
    for a in range(nb):
        t = np.arange(a + 1)
        kept += int(np.sum(col_keep[t] | diag_keep[a - t]))
    return kept / (nb * (nb + 1) / 2.0)


# ----------------------------------------------------------------------------
# chunk_n > 1 (Alg. 1 stage 1: itv = S_q / chunk_n, Q_slice)
# ----------------------------------------------------------------------------
def chunk_segments(S: int, n_chunks: int):
    """[(first row, one past the last row)] of the chunk_n query segments."""
    if not (1 <= n_chunks <= S):
        raise ValueError("n_chunks must be in [1, S]")
    itv = S // n_chunks
    return [(m * itv, (m + 1) * itv if m + 1 < n_chunks else S) for m in range(n_chunks)]


def sample_scores_chunked(q, k, n_sample_rows: int, n_chunks: int, scale: Optional[float] = None):
    """Per chunk: column and slash scores of the last ``n_sample_rows`` rows of
    the chunk's segment.  Returns (col [chunk_n, S], slash [chunk_n, S])."""
    q, k = _f64(q), _f64(k)
    S, d = k.shape
    sc = _scale(d, scale)
    cols, slashes = [], []
    for lo, hi in chunk_segments(S, n_chunks):
        if not (1 <= n_sample_rows <= hi - lo):
            raise ValueError("n_sample_rows must fit in a segment")
        col = np.zeros(S)
        slash = np.zeros(S)
        for r in _chunks(np.arange(hi - n_sample_rows, hi, dtype=np.int64), S):
            p, _ = _causal_softmax_rows(q, k, r, sc)
            col += p.sum(axis=0)
            for n, i in enumerate(r):
                slash[: i + 1] += p[n, i::-1]
        cols.append(col)
        slashes.append(slash)
    return np.stack(cols), np.stack(slashes)


def chunked_masked_attn(q, k, v, col_idx, slash_idx, window: int, n_chunks: int,
                        scale: Optional[float] = None, rows=None, blk: int = 1):
    """Eq. 3 where the rows of segment m are masked by the strips (or, with
    blk > 1, the blocks) selected from chunk m: ``col_idx[m]``, ``slash_idx[m]``.
    Returns (O [n_rows, d], lse [n_rows])."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    S = k.shape[0]
    rows = np.arange(q.shape[0]) if rows is None else np.asarray(rows, dtype=np.int64)
    out = np.empty((len(rows), v.shape[1]))
    lse = np.empty(len(rows))
    for m, (lo, hi) in enumerate(chunk_segments(S, n_chunks)):
        sel = np.flatnonzero((rows >= lo) & (rows < hi))
        if len(sel) == 0:
            continue
        if blk == 1:
            o, l = masked_attn(q, k, v, col_idx[m], slash_idx[m], window, scale, rows[sel])
        else:
            o, l = block_masked_attn(q, k, v, col_idx[m], slash_idx[m], window, blk, scale, rows[sel])
        out[sel] = o
        lse[sel] = l
    return out, lse


def chunked_sample_attention(q, k, v, n_sample_rows: int, n_chunks: int, alpha_c: float, alpha_s: float,
                             window: int, scale: Optional[float] = None, rows=None,
                             blk: int = 1) -> Dict[str, object]:
    """Alg. 1 end to end for one head with chunk_n >= 1 (and blk >= 1)."""
    col, slash = sample_scores_chunked(q, k, n_sample_rows, n_chunks, scale)
    if blk > 1:
        col = np.stack([block_reduce(c, blk) for c in col])
        slash = np.stack([block_reduce(s_, blk) for s_ in slash])
    I_c = [select(c, alpha_c) for c in col]
    I_s = [select(s_, alpha_s) for s_ in slash]
    out, lse = chunked_masked_attn(q, k, v, I_c, I_s, window, n_chunks, scale, rows, blk)
    return {"out": out, "lse": lse, "col": col, "slash": slash, "col_idx": I_c, "slash_idx": I_s}


# ----------------------------------------------------------------------------
# GQA wrappers: query head h reads KV head h // (Hq / Hkv)
# ----------------------------------------------------------------------------
def kv_head_of(h: int, n_q_heads: int, n_kv_heads: int) -> int:
    if n_q_heads % n_kv_heads:
        raise ValueError("n_q_heads must be a multiple of n_kv_heads")
    return h // (n_q_heads // n_kv_heads)


def dense_attn_heads(Q, K, V, scale: Optional[float] = None, rows=None):
    """Eq. 1-2 for [Hq, S, d] queries against [Hkv, S, d] keys/values."""
    Hq, Hkv = Q.shape[0], K.shape[0]
    outs, lses = [], []
    for h in range(Hq):
        kv = kv_head_of(h, Hq, Hkv)
        o, l = dense_attn(Q[h], K[kv], V[kv], scale, rows)
        outs.append(o)
        lses.append(l)
    return np.stack(outs), np.stack(lses)


# ----------------------------------------------------------------------------
# diagnostics
# ----------------------------------------------------------------------------
def mask_density(S: int, col_idx, slash_idx, window: int) -> float:
    """|M| / (S (S + 1) / 2): kept fraction of the causal triangle
    (1 - sparsity ratio of Sec. 2.3), counted exactly without forming M."""
    col_keep = np.zeros(S, dtype=bool)
    col_keep[np.asarray(col_idx, dtype=np.int64)] = True
    off_keep = np.zeros(S, dtype=bool)
    off_keep[np.asarray(slash_idx, dtype=np.int64)] = True
    off_keep[: max(int(window), 0)] = True
    # column j holds rows i = j..S-1; offset o holds rows i = o..S-1
    n_col = int(np.sum(S - np.nonzero(col_keep)[0]))
    n_off = int(np.sum(S - np.nonzero(off_keep)[0]))
    # overlap: pairs (i, j) with j kept and (i - j) kept  <=>  j + o <= S - 1
    cj = np.nonzero(col_keep)[0]
    oo = np.nonzero(off_keep)[0]
    # for each kept column j count kept offsets o <= S - 1 - j
    both = int(np.sum(np.searchsorted(oo, S - 1 - cj, side="right")))
    return (n_col + n_off - both) / (S * (S + 1) / 2.0)


def mask_diagnostics(q, k, col_idx, slash_idx, window: int, rows,
                     scale: Optional[float] = None) -> Dict[str, float]:
    """Per-row recall sum_j M_ij p_ij of the dense softmax on the given rows;
    its minimum is the CRA of the mask (Sec. 3.3)."""
    q, k = _f64(q), _f64(k)
    S, d = k.shape
    sc = _scale(d, scale)
    rows = np.asarray(rows, dtype=np.int64)
    rec = np.empty(len(rows))
    at = 0
    for r in _chunks(rows, 2 * S):
        p, _ = _causal_softmax_rows(q, k, r, sc)
        M = strip_mask(S, col_idx, slash_idx, window, r)
        rec[at:at + len(r)] = (p * M).sum(axis=1)
        at += len(r)
    return {"cra_min": float(rec.min()), "recall_mean": float(rec.mean()),
            "density": mask_density(S, col_idx, slash_idx, window)}


def touched_block_fraction(S: int, col_idx, slash_idx, window: int, blk: int = 128) -> float:
    """Fraction of blk x blk blocks of the causal triangle that contain at
    least one kept (i, j) - the "ratio of calculated blocks" on the paper's
    128-block grid (Alg. 1, blk = 128)."""
    nb = (S + blk - 1) // blk
    col_blk = np.zeros(nb, dtype=bool)
    col_blk[np.asarray(col_idx, dtype=np.int64) // blk] = True
    off_keep = np.zeros(S + 2 * blk, dtype=bool)
    off_keep[np.asarray(slash_idx, dtype=np.int64)] = True
    off_keep[: max(int(window), 0)] = True
    csum = np.concatenate([[0], np.cumsum(off_keep)])
    touched = 0
    total = 0
    for a in range(nb):          # query block
        i_lo, i_hi = a * blk, min((a + 1) * blk, S) - 1
        for t in range(a + 1):   # key block
            j_lo, j_hi = t * blk, min((t + 1) * blk, S) - 1
            total += 1
            if col_blk[t]:
                # a kept column in this key block has some row >= it in the
                # query block unless it lies entirely above the diagonal
                js = np.asarray(col_idx, dtype=np.int64)
                js = js[(js >= j_lo) & (js <= j_hi)]
                if np.any(js <= i_hi):
                    touched += 1
                    continue
            o_lo, o_hi = max(i_lo - j_hi, 0), i_hi - j_lo
            if o_hi >= o_lo and csum[o_hi + 1] - csum[o_lo] > 0:
                touched += 1
    return touched / total
