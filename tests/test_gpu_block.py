"""GPU parity of the block-granularity entry points (Algorithm 1 with blk > 1)
against the fp64 oracle, on the same seeded inputs.

Tolerances as for the strip path: block scores |gpu - oracle| <= 1e-4 * oracle
+ 1e-6; block index sets bit-exact against the oracle run on the same fp32
block scores; attention outputs max-abs <= 2e-2, mean-abs <= 2e-3.
"""
import sys

import numpy as np
import pytest
import torch

from oracle import sample_attention as O
from sa_inputs import CONFIGS, bf16_bits_to_f32, make_inputs

pytestmark = pytest.mark.gpu

MAX_ABS, MEAN_ABS = 2e-2, 2e-3


from gpu_progress import record as _record, say as _say  # noqa: E402


def _dev(bits):
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16)
    return t[None].contiguous().cuda()


def _f64(bits):
    return bf16_bits_to_f32(bits).astype(np.float64)


def _inputs(name, S, Hq, Hkv, seed=7, gain=None, **kw):
    from dataclasses import replace
    wl = replace(CONFIGS[name], seq_len=S, n_q_heads=Hq, n_kv_heads=Hkv, **kw)
    if gain:
        wl = wl.with_structure_gain(gain)
    return wl, make_inputs(wl, seed=seed)


def _check_out(got, want, what):
    err = np.abs(got.astype(np.float64) - want)
    _say(f"{what}: max-abs {err.max():.3e} mean-abs {err.mean():.3e}")
    assert np.isfinite(got).all(), what
    assert err.max() <= MAX_ABS, (what, err.max())
    assert err.mean() <= MEAN_ABS, (what, err.mean())


def _score_tol(got, want, what):
    err = np.abs(got.astype(np.float64) - want)
    bound = 1e-4 * np.abs(want) + 1e-6
    worst = (err / bound).max()
    _say(f"{what}: worst err/bound {worst:.3f}")
    assert worst <= 1.0, (what, worst)


# ------------------------------------------------------------ block scores ----
@pytest.mark.parametrize("S,Hq,Hkv,n_s,blk", [(1024, 1, 1, 128, 128), (2500, 4, 2, 192, 128), (1100, 2, 1, 64, 64),
                                              (900, 2, 2, 900, 256), (100, 1, 1, 100, 128)])
def test_block_scores_match_oracle(S, Hq, Hkv, n_s, blk):
    import paper_2406_15486_amd as sa
    _say(f"block scores S={S} Hq={Hq} n_s={n_s} blk={blk}")
    wl, x = _inputs("glm8k", S, Hq, Hkv, n_sinks=min(8, S))
    q, k = _dev(x["q"]), _dev(x["k"])
    cb, sb = sa.sa_sample_scores(q, k, n_s, granularity=blk)
    cb2, sb2 = sa.sa_sample_scores(q, k, n_s, granularity=blk)
    col, slash = sa.sa_sample_scores(q, k, n_s)
    cb3, sb3 = sa.sa_block_scores(col, slash, blk, sa.Shape(1, Hq, Hkv, S))
    torch.cuda.synchronize()
    nb = (S + blk - 1) // blk
    assert cb.shape == (Hq, nb) and sb.shape == (Hq, nb)
    assert torch.equal(cb, cb2) and torch.equal(sb, sb2), "run-to-run bits differ"
    assert torch.equal(cb, cb3) and torch.equal(sb, sb3), "the two routes to block scores differ"
    qf, kf = _f64(x["q"]), _f64(x["k"])
    G = Hq // Hkv
    for h in range(Hq):
        wc, ws, _ = O.sample_scores(qf[h], kf[h // G], n_s)
        _score_tol(cb[h].cpu().numpy(), O.block_reduce(wc, blk), f"col blocks h{h}")
        _score_tol(sb[h].cpu().numpy(), O.block_reduce(ws, blk), f"slash blocks h{h}")
        # the reduction itself, on the GPU's own per-token scores
        assert np.abs(cb[h].cpu().numpy() - O.block_reduce(col[h].cpu().numpy(), blk)).max() <= 1e-6 * n_s
        assert abs(float(cb[h].double().sum()) - n_s) < 1e-3 * n_s
        assert abs(float(sb[h].double().sum()) - n_s) < 1e-3 * n_s


# --------------------------------------------------------- block selection ----
@pytest.mark.parametrize("S,blk", [(1024, 128), (100, 128), (70000, 64), (5000, 256)])
@pytest.mark.parametrize("alpha", [0.0, 0.6, 0.95, 1.0])
def test_select_blocks_bit_exact(S, blk, alpha):
    import paper_2406_15486_amd as sa
    _say(f"select blocks S={S} blk={blk} alpha={alpha}")
    nb = (S + blk - 1) // blk
    rng = np.random.default_rng(S + blk)
    a = (rng.random((3, nb)) ** 6).astype(np.float32)
    b = np.exp(rng.standard_normal((3, nb)) * 3).astype(np.float32)
    b[1, : nb // 2] = b[1, 0]                          # ties
    sh = sa.Shape(1, 3, 3, S)
    ci, cc, si, sc = sa.sa_select_blocks(torch.from_numpy(a).cuda(), torch.from_numpy(b).cuda(), alpha, alpha, blk, sh)
    torch.cuda.synchronize()
    for h in range(3):
        for idx, cnt, scores in ((ci, cc, a), (si, sc, b)):
            want = O.select(scores[h], float(np.float32(alpha)))
            assert int(cnt[h]) == len(want)
            assert np.array_equal(idx[h, :int(cnt[h])].cpu().numpy(), want)


# ------------------------------------------------------------------ attend ----
def _block_case(x, Ic, Is, w, blk, what, f32_out=False):
    import paper_2406_15486_amd as sa
    Hq, S = x["q"].shape[0], x["q"].shape[1]
    G = Hq // x["k"].shape[0]
    nb = (S + blk - 1) // blk
    ci = torch.zeros(Hq, nb, dtype=torch.int32)
    si = torch.zeros(Hq, nb, dtype=torch.int32)
    cc = torch.zeros(Hq, dtype=torch.int32)
    sc = torch.zeros(Hq, dtype=torch.int32)
    for h in range(Hq):
        ci[h, :len(Ic[h])] = torch.from_numpy(np.asarray(Ic[h], dtype=np.int32))
        si[h, :len(Is[h])] = torch.from_numpy(np.asarray(Is[h], dtype=np.int32))
        cc[h], sc[h] = len(Ic[h]), len(Is[h])
    out, lse, tiles = sa.sa_block_sparse_attn(_dev(x["q"]), _dev(x["k"]), _dev(x["v"]), ci.cuda(), cc.cuda(),
                                              si.cuda(), sc.cuda(), w, blk,
                                              out_dtype=sa.SA_OUT_F32 if f32_out else sa.SA_OUT_BF16,
                                              want_lse=True, want_tiles=True)
    torch.cuda.synchronize()
    qf, kf, vf = _f64(x["q"]), _f64(x["k"]), _f64(x["v"])
    for h in range(Hq):
        want, wlse = O.block_masked_attn(qf[h], kf[h // G], vf[h // G], Ic[h], Is[h], w, blk)
        _check_out(out[0, h].float().cpu().numpy(), want, f"{what} h{h}")
        assert np.abs(lse[h].cpu().numpy() - wlse).max() < 2e-3
    return tiles.cpu().numpy()


@pytest.mark.parametrize("S,Hq,Hkv,w,blk", [(1024, 1, 1, 64, 128), (1500, 4, 2, 128, 128), (1300, 2, 2, 1, 64),
                                            (2000, 2, 1, 300, 256), (300, 2, 2, 1, 128), (100, 1, 1, 5, 128),
                                            (1, 1, 1, 1, 128), (64, 2, 1, 500, 64), (257, 1, 1, 2, 256)])
def test_block_sparse_attn_random_blocks(S, Hq, Hkv, w, blk):
    _say(f"block sparse random S={S} Hq={Hq} w={w} blk={blk}")
    wl, x = _inputs("glm8k", S, Hq, Hkv, n_sinks=min(8, S))
    nb = (S + blk - 1) // blk
    rng = np.random.default_rng(S + w + blk)
    Ic = [np.sort(rng.choice(nb, rng.integers(0, nb // 3 + 1), replace=False)) for _ in range(Hq)]
    Is = [np.sort(rng.choice(nb, rng.integers(0, nb // 4 + 1), replace=False)) for _ in range(Hq)]
    _block_case(x, Ic, Is, w, blk, "block sparse random")


def test_block_sparse_attn_degenerate_sets():
    _say("block sparse degenerate sets")
    S, Hq, blk = 1100, 4, 128
    wl, x = _inputs("glm8k", S, Hq, 2, n_sinks=8)
    nb = (S + blk - 1) // blk
    allb, none = np.arange(nb), np.zeros(0, dtype=np.int64)
    Ic = [none, allb, none, np.array([nb - 1])]      # window only / all columns / all diagonals / the short last block
    Is = [none, none, allb, np.array([nb - 1])]
    tiles = _block_case(x, Ic, Is, 1, blk, "block degenerate", f32_out=True)
    # window 1 and nothing selected: only the diagonal blocks are computed
    S_pad = (S + 255) // 256 * 256
    assert 0 < tiles[0] <= (S_pad // 32) * (blk // 64) * 2


def test_block_all_blocks_equals_dense_kernel():
    import paper_2406_15486_amd as sa
    _say("block alpha=1 vs dense kernel")
    S, Hq, blk = 900, 2, 128
    wl, x = _inputs("glm8k", S, Hq, 1, n_sinks=8)
    q, k, v = _dev(x["q"]), _dev(x["k"]), _dev(x["v"])
    sh = sa.Shape(1, Hq, 1, S)
    cb, sb = sa.sa_sample_scores(q, k, 128, granularity=blk)
    ci, cc, si, sc = sa.sa_select_blocks(cb, sb, 1.0, 1.0, blk, sh)
    out, _, _ = sa.sa_block_sparse_attn(q, k, v, ci, cc, si, sc, 1, blk, out_dtype=sa.SA_OUT_F32)
    dense, _ = sa.sa_dense_attn(q, k, v, out_dtype=sa.SA_OUT_F32)
    torch.cuda.synchronize()
    assert int(cc.min()) == (S + blk - 1) // blk
    assert (out - dense).abs().max().item() < 2e-2


# ---------------------------------------------------------------- pipeline ----
@pytest.mark.parametrize("name,S,Hq,Hkv,gain,n_s", [("tiny", 1024, 1, 1, None, 128), ("glm32k", 3000, 4, 2, 5.0, 128),
                                                    ("glm32k", 4096, 2, 1, None, 256)])
def test_block_pipeline_end_to_end(name, S, Hq, Hkv, gain, n_s):
    """The paper's configuration: blk = 128 and the last 128 (or more) rows
    sampled.  Block sets may differ from the oracle's only where fp32 and fp64
    scores order candidates differently near the cut; the output is compared
    on the GPU's own block lists."""
    import paper_2406_15486_amd as sa
    _say(f"block pipeline {name} S={S} gain={gain} n_s={n_s}")
    blk, alpha = 128, 0.95
    wl, x = _inputs(name, S, Hq, Hkv, gain=gain)
    w = wl.window
    q, k, v = _dev(x["q"]), _dev(x["k"]), _dev(x["v"])
    sh = sa.Shape(1, Hq, Hkv, S)
    cb, sb = sa.sa_sample_scores(q, k, n_s, granularity=blk)
    ci, cc, si, sc = sa.sa_select_blocks(cb, sb, alpha, alpha, blk, sh)
    out, _, _ = sa.sa_block_sparse_attn(q, k, v, ci, cc, si, sc, w, blk)
    out2 = sa.block_sample_attention(q, k, v, n_s, alpha, alpha, w, blk)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)
    qf, kf, vf = _f64(x["q"]), _f64(x["k"]), _f64(x["v"])
    G = Hq // Hkv
    a32 = float(np.float32(alpha))
    for h in range(Hq):
        res = O.block_sample_attention(qf[h], kf[h // G], vf[h // G], n_s, a32, a32, w, blk)
        gc = ci[h, :int(cc[h])].cpu().numpy()
        gs = si[h, :int(sc[h])].cpu().numpy()
        for got, want, scores, nm in ((gc, res["col_blocks"], res["col_block_scores"], "col"),
                                      (gs, res["slash_blocks"], res["slash_block_scores"], "slash")):
            diff = np.setxor1d(got, want)
            gap = float(np.abs(scores[diff] - scores[want].min()).max() / scores[want].min()) if len(diff) else 0.0
            _say(f"h{h} {nm}: gpu {len(got)} oracle {len(want)} differing {len(diff)}, gap {gap:.2e}")
            _record(f"block pipeline {name} S={S}/h{h}/{nm}/strip_sets",
                    {"gpu": int(len(got)), "oracle": int(len(want)), "differing": int(len(diff)),
                     "largest_rel_gap_to_cut": gap})
            assert gap <= 2.5e-4, (nm, h, gap)       # twice the 1e-4 score tolerance, plus a little
        want_out, _ = O.block_masked_attn(qf[h], kf[h // G], vf[h // G], gc, gs, w, blk)
        _check_out(out[0, h].float().cpu().numpy(), want_out, f"block pipeline out h{h}")
