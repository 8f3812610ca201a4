"""Host-side checks of the seeded input generator (no method arithmetic here)."""
import numpy as np
import torch

from sa_inputs import (CONFIGS, bf16_bits_to_f32, f32_to_bf16_bits, make_group,
                       make_inputs, rows_from_ratio)


def test_rows_from_ratio_matches_workload_table():
    assert rows_from_ratio(1024, 0.05) == 64
    assert rows_from_ratio(8192, 0.05) == 448
    assert rows_from_ratio(32768, 0.05) == 1664
    assert rows_from_ratio(131072, 0.05) == 6592
    assert rows_from_ratio(1048576, 0.02) == 20992
    assert rows_from_ratio(32, 0.05) == 32
    assert rows_from_ratio(4096, 1.0) == 4096


def test_bf16_round_trip_matches_torch():
    x = np.random.default_rng(0).standard_normal(4096).astype(np.float32) * 3
    bits = f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16)
    assert np.array_equal(bits.view(np.int16), ref.view(torch.int16).numpy())
    assert np.array_equal(bf16_bits_to_f32(bits), ref.float().numpy())


def test_generator_is_seeded_and_shaped():
    wl = CONFIGS["tiny"]
    a = make_inputs(wl)
    b = make_inputs(wl)
    assert a["q"].shape == (1, 1024, 128) and a["k"].shape == (1, 1024, 128)
    assert a["q"].dtype == np.uint16
    assert np.array_equal(a["q"], b["q"]) and np.array_equal(a["v"], b["v"])
    c = make_inputs(wl, seed=1)
    assert not np.array_equal(a["q"], c["q"])
    assert a["meta"][0]["sink_pos"][0] == 0 and len(a["meta"][0]["sink_pos"]) == 8


def test_single_query_head_matches_full_group():
    wl = CONFIGS["glm8k"].scaled(512)
    full = make_group(wl, 1)
    one = make_group(wl, 1, q_heads=[5])
    assert np.array_equal(full["q"][5], one["q"][0])
    assert np.array_equal(full["k"], one["k"])


def test_planted_slash_peaks_on_its_diagonal():
    wl = CONFIGS["glm32k"].scaled(2048, n_sinks=0, n_slash=1)
    g = make_group(wl, 0, q_heads=[0])
    q = bf16_bits_to_f32(g["q"][0]).astype(np.float64)
    k = bf16_bits_to_f32(g["k"]).astype(np.float64)
    for o in g["slash_offsets"]:
        i = np.arange(o + 300, o + 400)
        on = np.einsum("nd,nd->n", q[i], k[i - o]).mean()
        off = np.einsum("nd,nd->n", q[i], k[i - o - 37]).mean()
        assert on > off + 20.0          # the high-frequency rotary pairs only align at i - j = o


def test_sink_rows_and_query_bias():
    wl = CONFIGS["glm8k"].scaled(1024)
    g = make_group(wl, 0, q_heads=[0])
    k = bf16_bits_to_f32(g["k"]).astype(np.float64)
    sinks = g["sink_pos"]
    u = k[sinks].mean(0)
    u /= np.linalg.norm(u)
    assert np.all(np.abs(np.linalg.norm(k[sinks], axis=1) - 4.0) < 0.6)
    q = bf16_bits_to_f32(g["q"][0]).astype(np.float64)
    assert abs((q @ u).mean() - 1.5) < 0.2
