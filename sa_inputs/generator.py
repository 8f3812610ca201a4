"""Synthetic ChatGLM3-6B-shaped attention inputs with planted structure.

Recipe (per KV head, every step in float32 unless noted, then one rounding to
bf16):

1. Q[g] for each of the ``group`` query heads sharing the KV head, K and V are
   i.i.d. N(0, 1), shape [S, d].
2. Rotary position embedding, base 10000, on Q and K: the head dimension is
   split into pairs (p, p + d/2), pair p rotates by ``pos * base**(-2p/d)``.
   Angles are formed in float64.
3. Slash offsets (optional): ``n_slash`` distinct offsets drawn uniformly from
   [2*window, S/2).  For each offset o one vector w_o ~ N(0, I_d) is planted
   *rotary-consistently*: key j gets ``+rope(w_o, j)`` and query row i >= o of
   every head in the group gets ``+rope(w_o, i - o)``.  The extra logit
   between row i and key j is then sum_p |w_o,p|^2 cos((i - j - o) theta_p),
   which peaks on the diagonal i - j = o.
4. Sinks: one unit vector u per KV head; sink positions are {0} plus
   ``n_sinks - 1`` distinct uniform positions in [1, S).  A sink key row is
   *replaced* by ``sink_gain*u + noise*N(0, I)``; every query row of the group
   gets ``+ q_bias*u``.  Done after steps 2-3 so u is position independent.
5. Round to nearest-even bf16.  V is left as drawn.

Random streams: ``default_rng([seed, config_id, kv_head, 0])`` feeds K, V and
the planted structure; ``default_rng([seed, config_id, kv_head, 1 + g])`` feeds
query head g of the group, so a single query head can be produced without the
others.
"""
from __future__ import annotations

import math
import os
import threading
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace
from typing import Callable, Dict, Iterable, Optional, Sequence, Tuple

import numpy as np

DEFAULT_SEED = 20240615
ROPE_BASE = 10000.0


@dataclass(frozen=True)
class Workload:
    """One synthetic workload: shape, planted structure, method parameters."""

    name: str
    config_id: int
    seq_len: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int = 128
    n_sinks: int = 0          # per KV head, position 0 included
    n_slash: int = 0          # planted slash offsets per KV head
    sample_ratio: float = 0.05
    window: int = 128
    alphas: Tuple[float, ...] = (0.95,)
    # generator constants (the literal values of the workload description)
    sink_gain: float = 4.0
    q_bias: float = 1.5
    noise: float = 0.1
    slash_scale: float = 1.0

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def n_sample_rows(self) -> int:
        return rows_from_ratio(self.seq_len, self.sample_ratio)

    def scaled(self, seq_len: int, **kw) -> "Workload":
        """Same recipe at another sequence length (used by small parity cases)."""
        return replace(self, seq_len=seq_len, **kw)

    def with_structure_gain(self, gain: float) -> "Workload":
        """Variant with ``sink_gain`` and ``q_bias`` multiplied by ``gain``.

        With the literal constants a sink's logit is no larger than a random
        key's; the variant makes the planted columns dominate, which is the
        regime of high sparsity.  Always reported under its own name.
        """
        return replace(
            self,
            name=f"{self.name}+gain{gain:g}",
            sink_gain=self.sink_gain * gain,
            q_bias=self.q_bias * gain,
        )


CONFIGS: Dict[str, Workload] = {
    "tiny": Workload("tiny", 1, 1024, 1, 1, n_sinks=8, n_slash=0, window=64),
    "glm8k": Workload("glm8k", 2, 8192, 32, 2, n_sinks=16, n_slash=0, window=128),
    "glm32k": Workload("glm32k", 3, 32768, 32, 2, n_sinks=32, n_slash=4, window=128),
    "glm128k": Workload(
        "glm128k", 4, 131072, 32, 2, n_sinks=32, n_slash=4, window=128,
        alphas=(0.80, 0.90, 0.95, 0.98),
    ),
    "glm1m": Workload(
        "glm1m", 5, 1048576, 32, 2, n_sinks=64, n_slash=8, window=128,
        sample_ratio=0.02,
    ),
}

# Heads of one pattern each (the three kinds of heads the paper's attention maps
# show): strong planted columns and no diagonal structure, planted diagonals and no
# sinks, and both.  Same shape and recipe as the 128K workload; ``.scaled(S)`` gives
# the same heads at another length.  The sinks are given five times the literal gain,
# so that they carry most of the mass and the head really is a column head.
HEAD_PATTERNS: Dict[str, Workload] = {
    "column": Workload("head-column", 11, 131072, 32, 2, n_sinks=32, n_slash=0, window=128,
                       sink_gain=20.0, q_bias=7.5),
    "slash": Workload("head-slash", 12, 131072, 32, 2, n_sinks=0, n_slash=2, window=128),
    "composed": Workload("head-composed", 13, 131072, 32, 2, n_sinks=32, n_slash=2, window=128,
                         sink_gain=20.0, q_bias=7.5),
}


def rows_from_ratio(seq_len: int, ratio: float) -> int:
    """Sampled-row count: 64 * ceil(ratio * S / 64), clamped to [min(64,S), S]."""
    blocks = math.ceil(float(ratio) * seq_len / 64.0 - 1e-9)
    n = 64 * max(blocks, 1)
    return int(min(n, seq_len))


# ----------------------------------------------------------------------------
# bf16 <-> f32 bit helpers (numpy has no bf16 dtype)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (nearest even); returns the uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.reshape(-1).view(np.uint32)
    out = np.empty(u.shape[0], dtype=np.uint16)
    step = 1 << 18                      # cache-sized pieces: the temporaries stay small
    t = np.empty(step, dtype=np.uint32)
    for a in range(0, u.shape[0], step):
        e = min(a + step, u.shape[0])
        r = t[: e - a]
        np.right_shift(u[a:e], np.uint32(16), out=r)
        np.bitwise_and(r, np.uint32(1), out=r)
        r += np.uint32(0x7FFF)
        r += u[a:e]
        np.right_shift(r, np.uint32(16), out=r)
        out[a:e] = r
    return out.reshape(x.shape)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact upcast of bf16 bit patterns (uint16) to float32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------------
# rotary embedding
# ----------------------------------------------------------------------------
class _RopeTable:
    """cos / sin of ``pos * base**(-p/half)`` for pos = 0 .. n-1, formed in float64 and
    rounded once to float32; rows are computed on first use and kept, so that the
    many rotations of one workload (every head, every planted vector) share them."""

    def __init__(self, half: int):
        self.half = half
        self.inv_freq = ROPE_BASE ** (-np.arange(half, dtype=np.float64) / half)
        self.cos = np.zeros((0, half), dtype=np.float32)
        self.sin = np.zeros((0, half), dtype=np.float32)
        self.lock = threading.Lock()

    def upto(self, n: int, chunk: int = 1 << 15):
        with self.lock:
            have = self.cos.shape[0]
            if n > have:
                c = np.empty((n, self.half), dtype=np.float32)
                s = np.empty((n, self.half), dtype=np.float32)
                c[:have], s[:have] = self.cos, self.sin
                for a in range(have, n, chunk):
                    e = min(a + chunk, n)
                    ang = np.arange(a, e, dtype=np.int64)[:, None].astype(np.float64) * self.inv_freq[None, :]
                    c[a:e] = np.cos(ang).astype(np.float32)
                    s[a:e] = np.sin(ang).astype(np.float32)
                self.cos, self.sin = c, s
            return self.cos, self.sin


_ROPE_TABLES: Dict[int, _RopeTable] = {}
_ROPE_TABLES_LOCK = threading.Lock()


def _rope_table(half: int) -> _RopeTable:
    with _ROPE_TABLES_LOCK:
        if half not in _ROPE_TABLES:
            _ROPE_TABLES[half] = _RopeTable(half)
        return _ROPE_TABLES[half]


def release_tables() -> None:
    """Drop the cached rotary tables (0.5 GB at one million positions)."""
    with _ROPE_TABLES_LOCK:
        _ROPE_TABLES.clear()


def _rope_inplace(x: np.ndarray, n_pos: int, chunk: int = 1 << 15) -> None:
    """Rotate row r of x ([n, d] float32) by position r, r = 0 .. n-1, in place."""
    n, d = x.shape
    assert n == n_pos
    half = d // 2
    cos, sin = _rope_table(half).upto(n)
    for s in range(0, n, chunk):
        e = min(s + chunk, n)
        c, sn = cos[s:e], sin[s:e]
        a = x[s:e, :half].copy()
        b = x[s:e, half:]
        x[s:e, :half] = a * c - b * sn
        x[s:e, half:] = b * c + a * sn


def _rope_of_vector(w: np.ndarray, n_pos: int) -> np.ndarray:
    """rope(w, pos) for one vector w [d] at positions 0 .. n_pos-1 -> [n_pos, d] float32."""
    out = np.broadcast_to(w.astype(np.float32), (n_pos, w.shape[0])).copy()
    _rope_inplace(out, n_pos)
    return out


# ----------------------------------------------------------------------------
# generator
# ----------------------------------------------------------------------------
def _structure(wl: Workload, kv_head: int, seed: int):
    """Draw K, V and the planted structure of one KV head (float32, pre-bf16)."""
    S, d = wl.seq_len, wl.head_dim
    rng = np.random.default_rng([seed, wl.config_id, kv_head, 0])
    k = rng.standard_normal((S, d), dtype=np.float32)
    v = rng.standard_normal((S, d), dtype=np.float32)
    _rope_inplace(k, S)

    slash_offsets = np.zeros(0, dtype=np.int64)
    slash_vecs = np.zeros((0, d), dtype=np.float32)
    if wl.n_slash > 0:
        lo, hi = 2 * wl.window, S // 2
        if hi - lo < wl.n_slash:
            raise ValueError("sequence too short for the requested slash offsets")
        slash_offsets = np.sort(rng.choice(np.arange(lo, hi), size=wl.n_slash, replace=False))
        slash_vecs = (wl.slash_scale * rng.standard_normal((wl.n_slash, d))).astype(np.float32)
        for w_o in slash_vecs:
            k += _rope_of_vector(w_o, S)

    u = np.zeros(d, dtype=np.float32)
    sink_pos = np.zeros(0, dtype=np.int64)
    if wl.n_sinks > 0:
        u64 = rng.standard_normal(d)
        u = (u64 / np.linalg.norm(u64)).astype(np.float32)
        rest = rng.choice(np.arange(1, S), size=wl.n_sinks - 1, replace=False)
        sink_pos = np.sort(np.concatenate([[0], rest]).astype(np.int64))
        noise = rng.standard_normal((wl.n_sinks, d), dtype=np.float32)
        k[sink_pos] = wl.sink_gain * u[None, :] + wl.noise * noise
    return k, v, u, sink_pos, slash_offsets, slash_vecs


def make_group(
    wl: Workload,
    kv_head: int,
    seed: int = DEFAULT_SEED,
    q_heads: Optional[Sequence[int]] = None,
    q_out: Optional[np.ndarray] = None,
    workers: int = 1,
    progress: Optional[Callable[[str], None]] = None,
):
    """Inputs of one KV head and (some of) the query heads that share it.

    Returns a dict with bf16 bit patterns (uint16): ``q`` [len(q_heads), S, d],
    ``k`` [S, d], ``v`` [S, d]; plus ``sink_pos``, ``slash_offsets`` and the
    list ``q_heads`` (indices *within the group*, default all).  ``q_out``, if
    given, receives the query heads (same shape).  ``workers`` threads draw the
    query heads side by side (every head has a random stream of its own, so the
    result does not depend on it); ``progress`` is called with a short message
    after each finished part.
    """
    S, d = wl.seq_len, wl.head_dim
    say = progress or (lambda msg: None)
    k, v, u, sink_pos, slash_offsets, slash_vecs = _structure(wl, kv_head, seed)
    say(f"{wl.name}: kv head {kv_head}: K, V and planted structure drawn")
    heads = list(range(wl.group)) if q_heads is None else list(q_heads)

    # the planted query-side addend is shared by every head of the group
    q_add = np.zeros((S, d), dtype=np.float32)
    for o, w_o in zip(slash_offsets, slash_vecs):
        q_add[o:] += _rope_of_vector(w_o, S - int(o))
    if wl.n_sinks > 0:
        q_add += wl.q_bias * u[None, :]

    q_bits = np.empty((len(heads), S, d), dtype=np.uint16) if q_out is None else q_out
    assert q_bits.shape == (len(heads), S, d) and q_bits.dtype == np.uint16

    def one_head(n: int) -> int:
        rng = np.random.default_rng([seed, wl.config_id, kv_head, 1 + heads[n]])
        q = rng.standard_normal((S, d), dtype=np.float32)
        _rope_inplace(q, S)
        q += q_add
        q_bits[n] = f32_to_bf16_bits(q)
        return n

    if workers > 1 and len(heads) > 1:
        with ThreadPoolExecutor(max_workers=min(workers, len(heads))) as pool:
            for n in pool.map(one_head, range(len(heads))):
                say(f"{wl.name}: kv head {kv_head}: query head {heads[n]} of the group done")
    else:
        for n in range(len(heads)):
            one_head(n)
            say(f"{wl.name}: kv head {kv_head}: query head {heads[n]} of the group done")
    return {
        "q": q_bits,
        "k": f32_to_bf16_bits(k),
        "v": f32_to_bf16_bits(v),
        "sink_pos": sink_pos,
        "slash_offsets": slash_offsets,
        "q_heads": heads,
    }


def default_workers(wl: Workload) -> int:
    """Threads for make_inputs: a few at large sizes (each holds about 12 bytes per
    query element while it works), one for small workloads."""
    if wl.seq_len < 16384:
        return 1
    return max(1, min(8, (os.cpu_count() or 2) // 2))


def make_inputs(wl: Workload, seed: int = DEFAULT_SEED, kv_heads: Optional[Iterable[int]] = None,
                workers: Optional[int] = None, progress: Optional[Callable[[str], None]] = None):
    """All heads of a workload: ``q`` [Hq, S, d], ``k``/``v`` [Hkv, S, d] as
    bf16 bit patterns (uint16), query head h using KV head h // group.  The result
    is the same for any ``workers``; ``progress`` as in make_group."""
    kvs = list(range(wl.n_kv_heads)) if kv_heads is None else list(kv_heads)
    S, d, G = wl.seq_len, wl.head_dim, wl.group
    nw = default_workers(wl) if workers is None else workers
    q = np.empty((len(kvs) * G, S, d), dtype=np.uint16)
    k = np.empty((len(kvs), S, d), dtype=np.uint16)
    v = np.empty((len(kvs), S, d), dtype=np.uint16)
    meta = []
    for n, kv in enumerate(kvs):
        g = make_group(wl, kv, seed, q_out=q[n * G:(n + 1) * G], workers=nw, progress=progress)
        k[n] = g["k"]
        v[n] = g["v"]
        meta.append({"sink_pos": g["sink_pos"], "slash_offsets": g["slash_offsets"]})
    if S >= (1 << 19):
        release_tables()
    return {"q": q, "k": k, "v": v, "meta": meta}
