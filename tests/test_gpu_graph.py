"""The whole path recorded into a HIP graph and replayed.

The library allocates nothing, never synchronises and clears its counters and bitmaps with
fill kernels (no memset nodes), so the three calls of a layer can be captured once and
replayed.  Every replay is checked against an eager run on the same inputs, bit for bit
(the kernels are deterministic), with eager work and synchronisations between replays; the
first replay is also checked against the fp64 oracle.
"""
import numpy as np
import pytest
import torch

from oracle import sample_attention as O
from sa_inputs import CONFIGS, bf16_bits_to_f32, make_inputs

from gpu_progress import say as _say

pytestmark = pytest.mark.gpu


def _dev(bits):
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16)
    return t[None].contiguous().cuda()


@pytest.mark.parametrize("granularity,n_chunks", [(1, 1), (128, 2)])
def test_graph_replays_match_eager_runs(granularity, n_chunks):
    import paper_2406_15486_amd as sa
    from dataclasses import replace
    S, Hq, Hkv, n_s, w, alpha = 2048, 4, 2, 128, 64, 0.9
    _say(f"graph capture of the path: S={S} granularity={granularity} chunk_n={n_chunks}")
    wl = replace(CONFIGS["glm32k"], seq_len=S, n_q_heads=Hq, n_kv_heads=Hkv).with_structure_gain(5.0)
    xs = [make_inputs(wl, seed=s) for s in (3, 4, 5)]
    shape = sa.Shape(1, Hq, Hkv, S)
    kw = dict(with_lse=True, granularity=granularity, n_chunks=n_chunks)
    eager = sa.SampleAttentionPlan(shape, n_s, **kw)
    graphed = sa.SampleAttentionPlan(shape, n_s, **kw)
    q, k, v = (torch.empty_like(_dev(xs[0][n])) for n in ("q", "k", "v"))       # the graph's fixed input buffers

    def load(x):
        q.copy_(_dev(x["q"])); k.copy_(_dev(x["k"])); v.copy_(_dev(x["v"]))

    load(xs[0])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        graphed.run(q, k, v, alpha, alpha, w)                                   # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        graphed.run(q, k, v, alpha, alpha, w)
    torch.cuda.synchronize()

    for rep, x in enumerate(xs + [xs[0]]):
        load(x)
        g.replay()
        torch.cuda.synchronize()
        got_out, got_lse = graphed.out.clone(), graphed.lse.clone()
        got_cnt = (graphed.col_cnt.clone(), graphed.slash_cnt.clone())
        eager.run(q, k, v, alpha, alpha, w)                                     # eager work between the replays
        torch.cuda.synchronize()
        assert torch.equal(got_cnt[0], eager.col_cnt) and torch.equal(got_cnt[1], eager.slash_cnt), rep
        assert torch.equal(got_out, eager.out), rep
        assert torch.equal(got_lse, eager.lse), rep
        _say(f"   replay {rep}: identical to the eager run")
        if rep == 0 and granularity == 1:
            qf, kf, vf = (bf16_bits_to_f32(x[n]).astype(np.float64) for n in ("q", "k", "v"))
            cc, sc = got_cnt[0].cpu().numpy(), got_cnt[1].cpu().numpy()
            ci, si = graphed.col_idx.cpu().numpy(), graphed.slash_idx.cpu().numpy()
            for h in (0, Hq - 1):
                want, _ = O.masked_attn(qf[h], kf[h // (Hq // Hkv)], vf[h // (Hq // Hkv)], ci[h, :cc[h]], si[h, :sc[h]], w)
                err = np.abs(got_out[0, h].float().cpu().numpy() - want)
                assert err.max() <= 2e-2 and err.mean() <= 2e-3, (h, err.max(), err.mean())
