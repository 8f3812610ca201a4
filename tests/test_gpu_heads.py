"""Separate thresholds for columns and slashes (alpha_c != alpha_s) on heads of
one pattern each: strong columns only, diagonals only, both (the three kinds of
heads in the paper's attention maps; Sec. 3 and the threshold study of
Sec. 5.3).  Every entry point of the path against the oracle: stage-1 scores
element by element, selection bit-exact on the same fp32 scores, strip sets of
the two pipelines, attention output on the GPU's lists."""
import numpy as np
import pytest
import torch

from oracle import sample_attention as O
from sa_inputs import HEAD_PATTERNS, bf16_bits_to_f32, make_inputs

from gpu_progress import record as _record, say as _say

pytestmark = pytest.mark.gpu


def _dev(bits):
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16)
    return t[None].contiguous().cuda()


def _f64(bits):
    return bf16_bits_to_f32(bits).astype(np.float64)


@pytest.mark.parametrize("pattern,alpha_c,alpha_s", [
    ("column", 0.95, 0.30),      # a column head wants its columns and hardly any diagonal
    ("column", 0.90, 0.0),       # ... none at all: the mask is columns plus the local window
    ("slash", 0.30, 0.95),       # a slash head the other way round
    ("composed", 0.95, 0.80),
])
def test_head_patterns_with_separate_thresholds(pattern, alpha_c, alpha_s):
    import paper_2406_15486_amd as sa
    from dataclasses import replace
    S, Hq, Hkv = 5000, 4, 2
    wl = replace(HEAD_PATTERNS[pattern], seq_len=S, n_q_heads=Hq, n_kv_heads=Hkv)
    n_s, w = wl.n_sample_rows, wl.window
    _say(f"head pattern {pattern}: S={S} n_s={n_s} alpha_c={alpha_c} alpha_s={alpha_s}")
    x = make_inputs(wl)
    q, k, v = _dev(x["q"]), _dev(x["k"]), _dev(x["v"])
    sh = sa.Shape(1, Hq, Hkv, S)
    col, slash = sa.sa_sample_scores(q, k, n_s)
    ci, cc, si, sc = sa.sa_select_strips(col, slash, alpha_c, alpha_s, sh)
    out, lse, _ = sa.sa_sparse_attn(q, k, v, ci, cc, si, sc, w, out_dtype=sa.SA_OUT_F32, want_lse=True)
    torch.cuda.synchronize()
    col, slash = col.cpu().numpy(), slash.cpu().numpy()
    ci, cc, si, sc = ci.cpu().numpy(), cc.cpu().numpy(), si.cpu().numpy(), sc.cpu().numpy()
    ac32, as32 = float(np.float32(alpha_c)), float(np.float32(alpha_s))
    G = Hq // Hkv
    for h in range(Hq):
        qf, kf, vf = _f64(x["q"][h]), _f64(x["k"][h // G]), _f64(x["v"][h // G])
        wc, ws, _ = O.sample_scores(qf, kf, n_s)
        for got, want, nm in ((col[h], wc, "col"), (slash[h], ws, "slash")):
            worst = (np.abs(got - want) / (1e-4 * np.abs(want) + 1e-6)).max()
            assert worst <= 1.0, (nm, h, worst)
        gc, gs = ci[h, :cc[h]], si[h, :sc[h]]
        assert np.array_equal(gc, O.select(col[h], ac32)), ("col", h)
        assert np.array_equal(gs, O.select(slash[h], as32)), ("slash", h)
        # the oracle's own pipeline: strips may differ only next to the cut
        for got, scores, a, nm in ((gc, wc, ac32, "col"), (gs, ws, as32, "slash")):
            want = O.select(scores, a)
            diff = np.setxor1d(got, want)
            gap = float(np.abs(scores[diff] - scores[want].min()).max() / scores[want].min()) if len(diff) else 0.0
            _record(f"head {pattern} ({alpha_c},{alpha_s})/h{h}/{nm}/strip_sets",
                    {"gpu": int(len(got)), "oracle": int(len(want)), "differing": int(len(diff)),
                     "largest_rel_gap_to_cut": gap})
            assert gap <= 2.5e-4, (nm, h, gap)
        want, wlse = O.masked_attn(qf, kf, vf, gc, gs, w)
        err = np.abs(out[0, h].cpu().numpy() - want)
        _say(f"   h{h}: k_c {len(gc)} k_s {len(gs)} density {O.mask_density(S, gc, gs, w):.3f} "
             f"max-abs {err.max():.2e} mean-abs {err.mean():.2e}")
        assert err.max() <= 2e-2 and err.mean() <= 2e-3
        assert np.abs(lse[h].cpu().numpy() - wlse).max() < 2e-3
    if alpha_s == 0.0:
        assert (sc == 0).all()          # no slash strip at all: diagonals come from the window only
