"""GPU parity: every C-ABI entry point against the fp64 oracle, element by
element, on the same seeded inputs.  Sizes span several tiles and ragged tails
and stay small enough for the oracle to finish in seconds.

Tolerances
- attention outputs (bf16 inputs, fp32 accumulation): max-abs <= 2e-2 and
  mean-abs <= 2e-3 against the fp64 oracle;
- sampled scores: |gpu - oracle| <= 1e-4 * oracle + 1e-6 per entry;
- strip index sets: bit-exact against the oracle run on the same fp32 scores.
"""
import sys

import numpy as np
import pytest
import torch

from oracle import sample_attention as O
from sa_inputs import CONFIGS, bf16_bits_to_f32, make_inputs

pytestmark = pytest.mark.gpu

MAX_ABS, MEAN_ABS = 2e-2, 2e-3
# End to end (oracle scores -> oracle selection against GPU scores -> GPU selection) the
# strip sets may differ only in strips whose oracle score is this close, relatively, to
# the oracle's cut score: twice the 1e-4 score tolerance (the strip's own score and the
# score that defines the cut can both be off by it) plus a little for the few ranks by
# which the same error moves alpha * total.
STRIP_GAP_BOUND = 2.5e-4


def _strip_set_gap(got, want, scores):
    """(size of the symmetric difference, largest |score - cut| / cut over it), with the
    oracle's scores and the oracle's cut (its smallest selected score)."""
    diff = np.setxor1d(got, want)
    if len(diff) == 0 or len(want) == 0:
        return int(len(diff)), 0.0
    cut = scores[want].min()
    return int(len(diff)), float(np.abs(scores[diff] - cut).max() / cut)


from gpu_progress import record as _record, say as _say  # noqa: E402


def _dev(bits):
    """[H, S, d] uint16 bf16 patterns -> [1, H, S, d] bf16 CUDA tensor."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16)
    return t[None].contiguous().cuda()


def _f64(bits):
    return bf16_bits_to_f32(bits).astype(np.float64)


def _inputs(name, S=None, Hq=None, Hkv=None, seed=7, gain=None, **kw):
    wl = CONFIGS[name]
    over = dict(kw)
    if S is not None:
        over["seq_len"] = S
    if Hq is not None:
        over["n_q_heads"] = Hq
    if Hkv is not None:
        over["n_kv_heads"] = Hkv
    if over:
        from dataclasses import replace
        wl = replace(wl, **over)
    if gain:
        wl = wl.with_structure_gain(gain)
    return wl, make_inputs(wl, seed=seed)


def _check_out(got, want, what):
    err = np.abs(got.astype(np.float64) - want)
    _say(f"{what}: max-abs {err.max():.3e} mean-abs {err.mean():.3e}")
    assert np.isfinite(got).all(), what
    assert err.max() <= MAX_ABS, (what, err.max())
    assert err.mean() <= MEAN_ABS, (what, err.mean())


# ------------------------------------------------------------------ dense ----
@pytest.mark.parametrize("S,Hq,Hkv", [(1024, 1, 1), (1100, 4, 2), (333, 2, 1), (64, 1, 1), (1, 1, 1)])
@pytest.mark.parametrize("f32_out", [False, True])
def test_dense_attn_matches_oracle(S, Hq, Hkv, f32_out):
    import paper_2406_15486_amd as sa
    _say(f"dense S={S} Hq={Hq} Hkv={Hkv} f32_out={f32_out}")
    wl, x = _inputs("tiny", S=S, Hq=Hq, Hkv=Hkv, n_sinks=min(8, S))
    out, lse = sa.sa_dense_attn(_dev(x["q"]), _dev(x["k"]), _dev(x["v"]),
                                out_dtype=sa.SA_OUT_F32 if f32_out else sa.SA_OUT_BF16, want_lse=True)
    torch.cuda.synchronize()
    want, want_lse = O.dense_attn_heads(_f64(x["q"]), _f64(x["k"]), _f64(x["v"]))
    _check_out(out[0].float().cpu().numpy(), want, "dense out")
    assert np.abs(lse.cpu().numpy() - want_lse).max() < 2e-3


def test_dense_attn_explicit_scale():
    import paper_2406_15486_amd as sa
    _say("dense explicit scale")
    wl, x = _inputs("tiny", S=256)
    out, _ = sa.sa_dense_attn(_dev(x["q"]), _dev(x["k"]), _dev(x["v"]), scale=0.05)
    torch.cuda.synchronize()
    want, _ = O.dense_attn(_f64(x["q"])[0], _f64(x["k"])[0], _f64(x["v"])[0], scale=float(np.float32(0.05)))
    _check_out(out[0, 0].float().cpu().numpy(), want, "dense scale=0.05")


# ----------------------------------------------------------------- stage 1 ----
def _score_tol(got, want, what):
    err = np.abs(got.astype(np.float64) - want)
    bound = 1e-4 * np.abs(want) + 1e-6
    worst = (err / bound).max()
    _say(f"{what}: worst err/bound {worst:.3f}, max-abs {err.max():.3e}")
    assert worst <= 1.0, (what, worst)


@pytest.mark.parametrize("name,S,Hq,Hkv,n_s,gain", [
    ("tiny", 1024, 1, 1, 64, None),
    ("glm8k", 2500, 4, 2, 192, None),        # ragged: S not a multiple of 128
    ("glm32k", 4096, 2, 1, 2304, 5.0),       # more than one chunk of sampled rows
    ("tiny", 200, 1, 1, 200, None),          # every row sampled
    ("glm8k", 777, 2, 1, 50, None),          # a sampled-row count that is no multiple of 32
    ("glm8k", 1500, 2, 2, 1, None),          # a single sampled row
    ("glm32k", 3000, 2, 1, 1100, None),      # ragged count, more than one row chunk
])
def test_sample_scores_matches_oracle(name, S, Hq, Hkv, n_s, gain):
    import paper_2406_15486_amd as sa
    _say(f"sample_scores {name} S={S} Hq={Hq} n_s={n_s} gain={gain}")
    wl, x = _inputs(name, S=S, Hq=Hq, Hkv=Hkv, gain=gain)
    q, k = _dev(x["q"]), _dev(x["k"])
    col, slash, lse = sa.sa_sample_scores(q, k, n_s, want_lse=True)
    col2, slash2 = sa.sa_sample_scores(q, k, n_s)
    torch.cuda.synchronize()
    assert torch.equal(col, col2) and torch.equal(slash, slash2), "run-to-run bits differ"
    qf, kf = _f64(x["q"]), _f64(x["k"])
    G = Hq // Hkv
    for h in range(Hq):
        wc, ws, wl_ = O.sample_scores(qf[h], kf[h // G], n_s)
        _score_tol(col[h].cpu().numpy(), wc, f"col h{h}")
        _score_tol(slash[h].cpu().numpy(), ws, f"slash h{h}")
        assert np.abs(lse[h].cpu().numpy() - wl_).max() < 2e-3
        assert abs(float(col[h].double().sum()) - n_s) < 1e-3 * n_s
        assert abs(float(slash[h].double().sum()) - n_s) < 1e-3 * n_s


def test_sample_scores_with_a_small_workspace_takes_the_heads_in_passes():
    """Any workspace from SA_OP_SAMPLE_SCORES_MIN up is accepted: the heads are then
    processed as many at a time as fit.  The split of the keys of the log-sum-exp sweep
    depends on the number of heads in a launch, so the scores agree to rounding, not bit
    for bit; both are checked against the oracle's tolerance."""
    import paper_2406_15486_amd as sa
    import paper_2406_15486_amd.binding as B
    _say("sample_scores in head passes")
    S, Hq, Hkv, n_s = 2300, 8, 2, 160
    wl, x = _inputs("glm32k", S=S, Hq=Hq, Hkv=Hkv)
    q, k = _dev(x["q"]), _dev(x["k"])
    sh = sa.Shape(1, Hq, Hkv, S)
    full = sa.sa_workspace_bytes(B.SA_OP_SAMPLE_SCORES, sh, n_s)
    least = sa.sa_workspace_bytes(B.SA_OP_SAMPLE_SCORES_MIN, sh, n_s)
    assert 0 < least < full / 4
    col, slash, lse = sa.sa_sample_scores(q, k, n_s, want_lse=True)
    qf, kf = _f64(x["q"]), _f64(x["k"])
    for nbytes in (least, least * 2 + 4096, full // 2 + 4096, full - 256):   # 1, 2, 4 heads per pass; 4 again
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        c2, s2, l2 = sa.sa_sample_scores(q, k, n_s, workspace=ws, want_lse=True)
        torch.cuda.synchronize()
        assert torch.allclose(c2, col, rtol=2e-5, atol=1e-8) and torch.allclose(s2, slash, rtol=2e-5, atol=1e-8)
        assert torch.allclose(l2, lse, rtol=0, atol=1e-4)
        for h in (0, 5, 7):
            wc, wsl, _ = O.sample_scores(qf[h], kf[h // (Hq // Hkv)], n_s)
            _score_tol(c2[h].cpu().numpy(), wc, f"col h{h} ws={nbytes}")
            _score_tol(s2[h].cpu().numpy(), wsl, f"slash h{h} ws={nbytes}")
    with pytest.raises(sa.SaError):
        sa.sa_sample_scores(q, k, n_s, workspace=torch.empty(least - 256, dtype=torch.uint8, device="cuda"))
    # block granularity and chunks go through the same passes
    cb, sb = sa.sa_sample_scores(q, k, 128, granularity=128, n_chunks=2)
    ws = torch.empty(sa.sa_workspace_bytes(B.SA_OP_SAMPLE_SCORES_MIN, sh, 128, granularity=128, n_chunks=2),
                     dtype=torch.uint8, device="cuda")
    cb2, sb2 = sa.sa_sample_scores(q, k, 128, granularity=128, n_chunks=2, workspace=ws)
    torch.cuda.synchronize()
    assert torch.allclose(cb2, cb, rtol=2e-5, atol=1e-8) and torch.allclose(sb2, sb, rtol=2e-5, atol=1e-8)


# ----------------------------------------------------------------- stage 2 ----
def _select_case(scores_c, scores_s, alpha_c, alpha_s):
    import paper_2406_15486_amd as sa
    n, S = scores_c.shape
    sh = sa.Shape(1, n, n, S)
    ci, cc, si, sc = sa.sa_select_strips(torch.from_numpy(scores_c).cuda(), torch.from_numpy(scores_s).cuda(),
                                         alpha_c, alpha_s, sh)
    torch.cuda.synchronize()
    ci, cc, si, sc = ci.cpu().numpy(), cc.cpu().numpy(), si.cpu().numpy(), sc.cpu().numpy()
    for h in range(n):
        for idx, cnt, scores, alpha, nm in ((ci, cc, scores_c, alpha_c, "col"), (si, sc, scores_s, alpha_s, "slash")):
            want = O.select(scores[h], float(np.float32(alpha)))
            got = idx[h, :cnt[h]]
            assert cnt[h] == len(want), (nm, h, cnt[h], len(want))
            assert np.array_equal(got, want), (nm, h)


@pytest.mark.parametrize("S", [1, 7, 1000, 5000, 70000])
@pytest.mark.parametrize("alpha", [0.0, 0.5, 0.95, 0.999, 1.0])
def test_select_strips_random_scores(S, alpha):
    _say(f"select random S={S} alpha={alpha}")
    rng = np.random.default_rng(S)
    a = (rng.random((3, S)) ** 6).astype(np.float32)
    b = np.exp(rng.standard_normal((3, S)) * 3).astype(np.float32)
    _select_case(a, b, alpha, alpha)


def test_select_strips_ties_and_zeros():
    _say("select ties/zeros")
    S = 3000
    rng = np.random.default_rng(0)
    a = np.zeros((4, S), dtype=np.float32)
    a[0] = 1.0                                   # all tied
    a[1, rng.choice(S, 50, replace=False)] = 2.5  # few equal spikes, rest exactly zero
    a[2] = rng.integers(0, 4, S).astype(np.float32)   # heavy ties over 4 values
    a[3] = 0.0                                   # no mass at all
    b = np.roll(a, 1, axis=0).copy()
    for alpha in (0.3, 0.5, 0.95):
        _select_case(a, b, alpha, alpha)


def test_select_strips_denormals_and_wide_range():
    """Scores spread over the whole fp32 range, denormals included: the bin masses are
    formed from integer mantissa sums per exponent, which must hold there too."""
    _say("select denormals / wide range")
    S = 20000
    rng = np.random.default_rng(3)
    a = np.exp2(rng.uniform(-149, 20, (2, S))).astype(np.float32)
    b = (rng.integers(1, 1 << 22, (2, S)).astype(np.uint32)).view(np.float32)    # denormals only
    for alpha in (0.5, 0.99, 0.999999):
        _select_case(a, b, alpha, alpha)


def test_select_strips_bad_scores_count_as_zero():
    """A negative, infinite or NaN score carries no mass and ranks with the zeros (it is
    kept last, and only if everything with mass does not reach the threshold)."""
    import paper_2406_15486_amd as sa
    _say("select with non-finite / negative scores")
    S = 5000
    rng = np.random.default_rng(4)
    a = np.exp(rng.standard_normal((2, S)) * 2).astype(np.float32)
    bad = rng.choice(S, 40, replace=False)
    a[0, bad[:10]] = np.nan
    a[0, bad[10:20]] = np.inf
    a[0, bad[20:30]] = -np.inf
    a[0, bad[30:]] = -3.0
    a[1, bad] = -0.0
    clean = np.where(np.isfinite(a) & (a > 0), a, np.float32(0)).astype(np.float32)
    sh = sa.Shape(1, 2, 2, S)
    for alpha in (0.5, 0.95):
        got = sa.sa_select_strips(torch.from_numpy(a).cuda(), torch.from_numpy(a).cuda(), alpha, alpha, sh)
        want = sa.sa_select_strips(torch.from_numpy(clean).cuda(), torch.from_numpy(clean).cuda(), alpha, alpha, sh)
        torch.cuda.synchronize()
        for h in range(2):
            n = int(want[1][h])
            assert int(got[1][h]) == n
            assert torch.equal(got[0][h, :n], want[0][h, :n])
            assert np.array_equal(want[0][h, :n].cpu().numpy(), O.select(clean[h], float(np.float32(alpha))))
            assert not np.isin(bad, got[0][h, :n].cpu().numpy()).any()


def test_select_strips_repeatable():
    """Selection sums integers and walks the bins in a fixed order: two runs on the same
    scores give the same bits, also where many candidates tie at the cut."""
    import paper_2406_15486_amd as sa
    _say("select repeatability")
    S = 100000
    rng = np.random.default_rng(5)
    a = np.round(np.exp(rng.standard_normal((4, S))) * 8).astype(np.float32) / 8     # many exact ties
    sh = sa.Shape(1, 4, 4, S)
    t = torch.from_numpy(a).cuda()
    r1 = sa.sa_select_strips(t, t, 0.9, 0.97, sh)
    r2 = sa.sa_select_strips(t, t, 0.9, 0.97, sh)
    torch.cuda.synchronize()
    for x, y in zip(r1[1::2], r2[1::2]):
        assert torch.equal(x, y)
    for h in range(4):
        for idx, cnt, idx2 in ((r1[0], r1[1], r2[0]), (r1[2], r1[3], r2[2])):
            assert torch.equal(idx[h, :int(cnt[h])], idx2[h, :int(cnt[h])])
    _select_case(a, a, 0.9, 0.97)


def test_select_on_gpu_scores_matches_oracle_on_same_scores():
    import paper_2406_15486_amd as sa
    _say("select on GPU-produced scores")
    wl, x = _inputs("glm32k", S=4096, Hq=4, Hkv=2)
    col, slash = sa.sa_sample_scores(_dev(x["q"]), _dev(x["k"]), 256)
    torch.cuda.synchronize()
    _select_case(col.cpu().numpy(), slash.cpu().numpy(), 0.95, 0.9)


# ------------------------------------------------------------------ attend ----
def _sparse_case(wl, x, Ic, Is, w, what, f32_out=False):
    import paper_2406_15486_amd as sa
    Hq, S = x["q"].shape[0], x["q"].shape[1]
    G = Hq // x["k"].shape[0]
    ci = torch.zeros(Hq, S, dtype=torch.int32)
    si = torch.zeros(Hq, S, dtype=torch.int32)
    cc = torch.zeros(Hq, dtype=torch.int32)
    sc = torch.zeros(Hq, dtype=torch.int32)
    for h in range(Hq):
        ci[h, :len(Ic[h])] = torch.from_numpy(np.asarray(Ic[h], dtype=np.int32))
        si[h, :len(Is[h])] = torch.from_numpy(np.asarray(Is[h], dtype=np.int32))
        cc[h], sc[h] = len(Ic[h]), len(Is[h])
    out, lse, tiles = sa.sa_sparse_attn(_dev(x["q"]), _dev(x["k"]), _dev(x["v"]), ci.cuda(), cc.cuda(),
                                        si.cuda(), sc.cuda(), w,
                                        out_dtype=sa.SA_OUT_F32 if f32_out else sa.SA_OUT_BF16,
                                        want_lse=True, want_tiles=True)
    torch.cuda.synchronize()
    qf, kf, vf = _f64(x["q"]), _f64(x["k"]), _f64(x["v"])
    for h in range(Hq):
        want, wlse = O.masked_attn(qf[h], kf[h // G], vf[h // G], Ic[h], Is[h], w)
        _check_out(out[0, h].float().cpu().numpy(), want, f"{what} h{h}")
        assert np.abs(lse[h].cpu().numpy() - wlse).max() < 2e-3
    return tiles.cpu().numpy()


@pytest.mark.parametrize("S,Hq,Hkv,w", [(1024, 1, 1, 64), (1500, 4, 2, 128), (300, 2, 2, 1)])
def test_sparse_attn_random_strips(S, Hq, Hkv, w):
    _say(f"sparse random strips S={S} Hq={Hq} w={w}")
    wl, x = _inputs("glm8k", S=S, Hq=Hq, Hkv=Hkv, n_sinks=8)
    rng = np.random.default_rng(S + w)
    Ic = [np.sort(rng.choice(S, rng.integers(0, S // 3), replace=False)) for _ in range(Hq)]
    Is = [np.sort(rng.choice(S, rng.integers(0, S // 5), replace=False)) for _ in range(Hq)]
    _sparse_case(wl, x, Ic, Is, w, "sparse random")


@pytest.mark.parametrize("n_off", [0, 2, 40])
def test_sparse_attn_column_counts_around_the_loop_stretches(n_off):
    """The kernel's tile loop changes form where gathered tiles end and where the schedule
    ends: column counts of 0 .. 10 tiles of 64 and few / many range tiles put every one of
    those boundaries at the first, a middle and the last iteration."""
    S, counts = 1280, [0, 1, 64, 65, 255, 256, 257, 320, 321, 384, 449, 640]
    _say(f"sparse column counts around the stretches, {n_off} offsets")
    wl, x = _inputs("glm8k", S=S, Hq=len(counts), Hkv=2, n_sinks=8)
    rng = np.random.default_rng(n_off)
    Ic = [np.sort(rng.choice(S, c, replace=False)) for c in counts]
    Ic[3] = np.arange(65)                                     # the first keys: every query tile sees all of them
    Ic[7] = np.arange(S - 320, S)                             # the last keys: only the last tiles do
    Is = [np.sort(rng.choice(S, n_off, replace=False)) for _ in counts]
    _sparse_case(wl, x, Ic, Is, 1 if n_off else 70, "stretches")


@pytest.mark.parametrize("S,fc,fs", [(1500, 0.7, 0.6), (1024, 0.95, 0.9), (2304, 0.5, 0.8)])
def test_sparse_attn_nearly_full_lists(S, fc, fs):
    """Lists so full that most keys are selected columns AND most offsets are kept: every
    pair is still counted once (a key taken by the column pass is masked out of its range
    tile), whatever the two passes cost."""
    _say(f"sparse nearly full lists S={S} columns {fc} offsets {fs}")
    Hq = 3
    wl, x = _inputs("glm8k", S=S, Hq=Hq, Hkv=1, n_sinks=8)
    rng = np.random.default_rng(S)
    Ic = [np.sort(rng.choice(S, int(fc * S), replace=False)) for _ in range(Hq)]
    Is = [np.sort(rng.choice(S, int(fs * S), replace=False)) for _ in range(Hq)]
    Ic[2] = Ic[2][:S // 50]
    Is[2] = Is[2][:S // 100]
    _sparse_case(wl, x, Ic, Is, 16, "nearly full")


def test_sparse_attn_degenerate_strip_sets():
    _say("sparse degenerate sets")
    S, Hq = 700, 4
    wl, x = _inputs("glm8k", S=S, Hq=Hq, Hkv=2, n_sinks=8)
    allidx = np.arange(S)
    none = np.zeros(0, dtype=np.int64)
    Ic = [none, allidx, none, allidx]        # window only / all columns / all slashes / both
    Is = [none, none, allidx, allidx]
    tiles = _sparse_case(wl, x, Ic, Is, 3, "sparse degenerate", f32_out=True)
    assert tiles[0] > 0


def test_sparse_attn_all_strips_equals_dense_kernel():
    import paper_2406_15486_amd as sa
    _say("sparse alpha=1 vs dense kernel")
    S, Hq = 900, 2
    wl, x = _inputs("glm8k", S=S, Hq=Hq, Hkv=1, n_sinks=8)
    q, k, v = _dev(x["q"]), _dev(x["k"]), _dev(x["v"])
    sh = sa.Shape(1, Hq, 1, S)
    col, slash = sa.sa_sample_scores(q, k, 64)
    ci, cc, si, sc = sa.sa_select_strips(col, slash, 1.0, 1.0, sh)
    out, _, _ = sa.sa_sparse_attn(q, k, v, ci, cc, si, sc, 1, out_dtype=sa.SA_OUT_F32)
    dense, _ = sa.sa_dense_attn(q, k, v, out_dtype=sa.SA_OUT_F32)
    torch.cuda.synchronize()
    assert int(cc.min()) == S and int(sc.min()) == S
    assert (out - dense).abs().max().item() < 2e-2


# ---------------------------------------------------------------- pipeline ----
@pytest.mark.parametrize("name,S,Hq,Hkv,gain", [("tiny", 1024, 1, 1, None), ("glm32k", 3000, 4, 2, 5.0)])
def test_pipeline_end_to_end(name, S, Hq, Hkv, gain):
    """Oracle pipeline vs GPU pipeline.  Strip sets may differ only where the
    fp32 scores of the GPU and the fp64 scores of the oracle order candidates
    differently near the cut; the attention output is compared on the GPU's own
    strips (oracle masked attention on the same lists)."""
    import paper_2406_15486_amd as sa
    _say(f"pipeline {name} S={S} gain={gain}")
    wl, x = _inputs(name, S=S, Hq=Hq, Hkv=Hkv, gain=gain)
    n_s, w, alpha = wl.n_sample_rows, wl.window, 0.95
    q, k, v = _dev(x["q"]), _dev(x["k"]), _dev(x["v"])
    sh = sa.Shape(1, Hq, Hkv, S)
    col, slash = sa.sa_sample_scores(q, k, n_s)
    ci, cc, si, sc = sa.sa_select_strips(col, slash, alpha, alpha, sh)
    out, _, _ = sa.sa_sparse_attn(q, k, v, ci, cc, si, sc, w)
    torch.cuda.synchronize()
    qf, kf, vf = _f64(x["q"]), _f64(x["k"]), _f64(x["v"])
    G = Hq // Hkv
    a32 = float(np.float32(alpha))
    for h in range(Hq):
        res = O.sample_attention(qf[h], kf[h // G], vf[h // G], n_s, a32, a32, w)
        gc = ci[h, :int(cc[h])].cpu().numpy()
        gs = si[h, :int(sc[h])].cpu().numpy()
        for got, want, scores, nm in ((gc, res["col_idx"], res["col"], "col"),
                                      (gs, res["slash_idx"], res["slash"], "slash")):
            n_diff, gap = _strip_set_gap(got, want, scores)
            _say(f"h{h} {nm}: gpu {len(got)} oracle {len(want)} differing {n_diff}, "
                 f"largest relative score gap to the cut among them {gap:.3e}")
            _record(f"pipeline {name} S={S}/h{h}/{nm}/strip_sets",
                    {"gpu": int(len(got)), "oracle": int(len(want)), "differing": n_diff,
                     "largest_rel_gap_to_cut": gap})
            assert gap <= STRIP_GAP_BOUND, (nm, h, gap)
        want_out, _ = O.masked_attn(qf[h], kf[h // G], vf[h // G], gc, gs, w)
        _check_out(out[0, h].float().cpu().numpy(), want_out, f"pipeline out h{h}")


# ------------------------------------------------------------------- batch ----
@pytest.mark.parametrize("blk", [1, 128])
def test_batch_of_two_sequences(blk):
    """[batch, heads, seq, d] with batch = 2: every (batch, head) pair is an
    independent problem and query head h of batch b reads KV head h // group of
    the same batch.  Compared with the same calls on each sequence alone."""
    import paper_2406_15486_amd as sa
    _say(f"batch 2, blk={blk}")
    S, Hq, Hkv, n_s, w, alpha = 1300, 4, 2, 64, 32, 0.9
    xs = [_inputs("glm8k", S=S, Hq=Hq, Hkv=Hkv, seed=s, n_sinks=8)[1] for s in (11, 12)]
    q = torch.cat([_dev(x["q"]) for x in xs]).contiguous()
    k = torch.cat([_dev(x["k"]) for x in xs]).contiguous()
    v = torch.cat([_dev(x["v"]) for x in xs]).contiguous()
    if blk == 1:
        out = sa.sample_attention(q, k, v, n_s, alpha, alpha, w)
        ones = [sa.sample_attention(q[b:b + 1].contiguous(), k[b:b + 1].contiguous(), v[b:b + 1].contiguous(),
                                    n_s, alpha, alpha, w) for b in range(2)]
    else:
        out = sa.block_sample_attention(q, k, v, n_s, alpha, alpha, w, blk)
        ones = [sa.block_sample_attention(q[b:b + 1].contiguous(), k[b:b + 1].contiguous(),
                                          v[b:b + 1].contiguous(), n_s, alpha, alpha, w, blk) for b in range(2)]
    dense, _ = sa.sa_dense_attn(q, k, v)
    torch.cuda.synchronize()
    for b in range(2):
        assert torch.equal(out[b], ones[b][0]), f"batch element {b} differs from the single-sequence call"
    # and against the oracle: the dense kernel on the second sequence, one head of its second KV group
    x = xs[1]
    want, _ = O.dense_attn(_f64(x["q"])[3], _f64(x["k"])[1], _f64(x["v"])[1])
    _check_out(dense[1, 3].float().cpu().numpy(), want, "batch dense b1 h3")


def test_partitioned_sparse_attn_across_batches():
    """Head partition with a pass that straddles two batch elements (3 heads per pass, 4
    query heads per sequence, 2 sequences) and query segments on a ragged length."""
    import paper_2406_15486_amd as sa
    _say("partitioned sparse attention, batch 2")
    S, Hq, Hkv, w = 1300, 4, 2, 32
    xs = [_inputs("glm8k", S=S, Hq=Hq, Hkv=Hkv, seed=s, n_sinks=8)[1] for s in (21, 22)]
    q = torch.cat([_dev(x["q"]) for x in xs]).contiguous()
    k = torch.cat([_dev(x["k"]) for x in xs]).contiguous()
    v = torch.cat([_dev(x["v"]) for x in xs]).contiguous()
    sh = sa.Shape(2, Hq, Hkv, S)
    col, slash = sa.sa_sample_scores(q, k, 64)
    ci, cc, si, sc = sa.sa_select_strips(col, slash, 0.9, 0.8, sh)
    want, want_lse, want_tiles = sa.sa_sparse_attn(q, k, v, ci, cc, si, sc, w, want_lse=True, want_tiles=True)
    for hpp, segs in ((3, 2), (1, 1), (8, 100)):
        got, lse, tiles = sa.sa_sparse_attn_partitioned(q, k, v, ci, cc, si, sc, w, hpp, segs, want_lse=True,
                                                        want_tiles=True)
        torch.cuda.synchronize()
        assert torch.equal(got, want) and torch.equal(lse, want_lse) and torch.equal(tiles, want_tiles), (hpp, segs)
    # against the oracle: second sequence, a head of its second KV group
    x = xs[1]
    gc, gs = ci[7, :int(cc[7])].cpu().numpy(), si[7, :int(sc[7])].cpu().numpy()
    ref, _ = O.masked_attn(_f64(x["q"])[3], _f64(x["k"])[1], _f64(x["v"])[1], gc, gs, w)
    _check_out(got[1, 3].float().cpu().numpy(), ref, "partitioned b1 h3")


# ---------------------------------------------------------------- numerics ----
def _bf16_bits(a):
    """float array -> bf16 bit patterns (round to nearest even), as the generator does."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


@pytest.mark.parametrize("kind", ["rising", "falling", "spiky"])
def test_large_logits_exercise_the_reference_maximum(kind):
    """Scores far from N(0,1): a maximum that rises with every key tile (the
    accumulators are rescaled again and again), one that is met in the first tile
    and never again, and isolated keys 40 logits above the rest.  Dense and
    strip-masked kernels against the oracle."""
    import paper_2406_15486_amd as sa
    _say(f"large logits: {kind}")
    S, d = 1500, 128
    rng = np.random.default_rng(5)
    u = rng.standard_normal(d)
    u /= np.linalg.norm(u)
    q = rng.standard_normal((1, S, d)) + 6.0 * u
    k = rng.standard_normal((1, S, d))
    v = rng.standard_normal((1, S, d))
    ramp = np.arange(S)[:, None] / S
    if kind == "rising":
        k += 60.0 * ramp * u            # logit grows by ~32 over the sequence
    elif kind == "falling":
        k += 60.0 * (1.0 - ramp) * u
    else:
        k[0, rng.choice(S, 12, replace=False)] += 75.0 * u
    x = {"q": _bf16_bits(q), "k": _bf16_bits(k), "v": _bf16_bits(v)}
    qd, kd, vd = _dev(x["q"]), _dev(x["k"]), _dev(x["v"])
    dense, dlse = sa.sa_dense_attn(qd, kd, vd, out_dtype=sa.SA_OUT_F32, want_lse=True)
    torch.cuda.synchronize()
    qf, kf, vf = _f64(x["q"])[0], _f64(x["k"])[0], _f64(x["v"])[0]
    want, wlse = O.dense_attn(qf, kf, vf)
    _check_out(dense[0, 0].cpu().numpy(), want, f"dense {kind}")
    assert np.abs(dlse[0].cpu().numpy() - wlse).max() < 2e-3 * max(1.0, np.abs(wlse).max() / 10)
    Ic = [np.sort(rng.choice(S, 300, replace=False))]
    Is = [np.sort(rng.choice(S, 200, replace=False))]
    _sparse_case(None, x, Ic, Is, 16, f"sparse {kind}", f32_out=True)
    # stage 1 on the same inputs: the probabilities are recomputed from the row log-sum-exps
    col, slash = sa.sa_sample_scores(qd, kd, 192)
    torch.cuda.synchronize()
    wc, ws, _ = O.sample_scores(qf, kf, 192)
    _score_tol(col[0].cpu().numpy(), wc, f"col {kind}")
    _score_tol(slash[0].cpu().numpy(), ws, f"slash {kind}")


# ----------------------------------------------------------------- boundary ----
def test_side_stream_and_repeatability():
    """The library enqueues on the stream it is given and nothing else: the whole
    path on a side stream gives the bits of the default-stream run, and so does a
    second run (no atomics on floating point anywhere in the path)."""
    import paper_2406_15486_amd as sa
    _say("side stream / repeatability")
    wl, x = _inputs("glm32k", S=3000, Hq=4, Hkv=2)
    q, k, v = _dev(x["q"]), _dev(x["k"]), _dev(x["v"])
    args = (wl.n_sample_rows // 64 * 64 or 64, 0.95, 0.9, wl.window)
    a = sa.sample_attention(q, k, v, *args)
    b = sa.sample_attention(q, k, v, *args)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        c = sa.sample_attention(q, k, v, *args)
        d = sa.block_sample_attention(q, k, v, 128, 0.95, 0.9, wl.window, 128)
    side.synchronize()
    e = sa.block_sample_attention(q, k, v, 128, 0.95, 0.9, wl.window, 128)
    torch.cuda.synchronize()
    assert torch.equal(a, b), "two runs differ"
    assert torch.equal(a, c), "side-stream run differs"
    assert torch.equal(d, e), "block path: side-stream run differs"


def test_sparse_attn_explicit_scale_and_shared_workspace():
    """softmax_scale other than 1/sqrt(d), and one caller-owned workspace reused by
    consecutive calls of different entry points."""
    import paper_2406_15486_amd as sa
    _say("explicit scale, shared workspace")
    S, Hq = 1100, 2
    wl, x = _inputs("glm8k", S=S, Hq=Hq, Hkv=1, n_sinks=8)
    q, k, v = _dev(x["q"]), _dev(x["k"]), _dev(x["v"])
    sh = sa.Shape(1, Hq, 1, S, softmax_scale=0.05)
    need = max(sa.sa_workspace_bytes(op, sh, 64) for op in (0, 2, 3))
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    col, slash = sa.sa_sample_scores(q, k, 64, scale=0.05, workspace=ws)
    ci, cc, si, sc = sa.sa_select_strips(col, slash, 0.9, 0.9, sh)
    out, lse, _ = sa.sa_sparse_attn(q, k, v, ci, cc, si, sc, 8, scale=0.05, workspace=ws, want_lse=True,
                                    out_dtype=sa.SA_OUT_F32)
    dense, _ = sa.sa_dense_attn(q, k, v, scale=0.05, workspace=ws, out_dtype=sa.SA_OUT_F32)
    torch.cuda.synchronize()
    s32 = float(np.float32(0.05))
    qf, kf, vf = _f64(x["q"]), _f64(x["k"])[0], _f64(x["v"])[0]
    for h in range(Hq):
        wc, wsl, _ = O.sample_scores(qf[h], kf, 64, scale=s32)
        _score_tol(col[h].cpu().numpy(), wc, f"col scale h{h}")
        gc, gs = ci[h, :int(cc[h])].cpu().numpy(), si[h, :int(sc[h])].cpu().numpy()
        want, wlse = O.masked_attn(qf[h], kf, vf, gc, gs, 8, scale=s32)
        _check_out(out[0, h].cpu().numpy(), want, f"sparse scale h{h}")
        assert np.abs(lse[h].cpu().numpy() - wlse).max() < 2e-3
        wd, _ = O.dense_attn(qf[h], kf, vf, scale=s32)
        _check_out(dense[0, h].cpu().numpy(), wd, f"dense scale h{h}")
