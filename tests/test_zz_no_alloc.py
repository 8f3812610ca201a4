"""The entry point that allocates nothing (sa_dense_attn_static) against the
entry point it is a variant of (sa_dense_attn): same kernels, so the outputs
must agree bit for bit; two calls in a row, the second on a smaller input
(the static scratch then still holds the first call's transposed V), then a
third on yet another shape; the last one also against the oracle.  (The size
limit is a host-side check: tests/test_abi.py.)"""
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


def _case(S, Hq, Hkv, seed):
    from dataclasses import replace
    wl = replace(CONFIGS["glm8k"], seq_len=S, n_q_heads=Hq, n_kv_heads=Hkv, n_sinks=8)
    x = make_inputs(wl, seed=seed)
    return x, _dev(x["q"]), _dev(x["k"]), _dev(x["v"])


def test_static_scratch_entry_point_matches_dense_attn():
    import paper_2406_15486_amd as sa
    lib = sa.load_library()
    results = []
    # first call: a large input that fills most of the scratch; second: a smaller one;
    # third: a ragged length with fp32 output and the log-sum-exp
    for n, (S, Hq, Hkv, f32) in enumerate([(20000, 4, 2, False), (1100, 4, 2, False), (333, 2, 1, True)]):
        _say(f"static-scratch dense call {n}: S={S} Hq={Hq} Hkv={Hkv} f32_out={f32}")
        x, q, k, v = _case(S, Hq, Hkv, seed=20 + n)
        odt = torch.float32 if f32 else torch.bfloat16
        out = torch.empty(q.shape, dtype=odt, device="cuda")
        lse = torch.empty(Hq, S, dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        sa.sa_dense_attn_static(q, k, v, out, lse=lse)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        results.append((x, q, k, v, out, lse, f32))
    # the reference calls come afterwards, so that nothing between the static calls rewrites the scratch
    for n, (x, q, k, v, out, lse, f32) in enumerate(results):
        want, want_lse = sa.sa_dense_attn(q, k, v, out_dtype=sa.SA_OUT_F32 if f32 else sa.SA_OUT_BF16, want_lse=True)
        torch.cuda.synchronize()
        assert torch.equal(out, want), f"call {n}: output differs from sa_dense_attn"
        assert torch.equal(lse, want_lse), f"call {n}: log-sum-exp differs from sa_dense_attn"
    # the last (small) case against the oracle as well
    x, q, k, v, out, lse, _ = results[-1]
    qf = bf16_bits_to_f32(x["q"]).astype(np.float64)
    kf = bf16_bits_to_f32(x["k"]).astype(np.float64)
    vf = bf16_bits_to_f32(x["v"]).astype(np.float64)
    ref, ref_lse = O.dense_attn_heads(qf, kf, vf)
    err = np.abs(out[0].float().cpu().numpy() - ref)
    assert err.max() <= 2e-2 and err.mean() <= 2e-3
    assert np.abs(lse.cpu().numpy() - ref_lse).max() < 2e-3
