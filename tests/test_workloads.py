"""The seeded input generators: shapes, determinism, storage-dtype exactness, structure."""
import numpy as np
import torch

import workloads as W


def test_config_shapes_match_the_stated_workloads():
    want = {0: (1, 2, 4, 2, 64, 512, 32), 1: (1, 32, 32, 8, 128, 2944, 32),
            2: (4, 32, 32, 8, 128, 10368, 64), 3: (4, 60, 56, 8, 128, 10368, 64),
            4: (1, 32, 32, 8, 128, 32768, 64)}
    for c in W.CONFIGS:
        assert (c.B, c.L, c.Hq, c.Hkv, c.d, c.m, c.tau) == want[c.cid]
        lo, hi = c.visual_span
        assert hi <= c.m - c.tau and c.Hq % c.Hkv == 0
    assert [W.budget_total(W.CONFIGS[i], (1, 10)) for i in range(4)] == [102, 9420, 33177, 62208]
    assert [W.budget_total(W.CONFIGS[4], a) for a in W.CONFIGS[4].alphas] == [10485, 52428, 104857, 209715]


def test_draws_are_deterministic_and_keyed():
    c = W.CONFIGS[0]
    a, b = W.layer_inputs(c, 0, 1), W.layer_inputs(c, 0, 1)
    for k in a:
        assert np.array_equal(a[k], b[k])
    other = W.layer_inputs(c, 0, 0)
    assert not np.array_equal(a["k"], other["k"])
    assert a["q_win"].shape == (4, 32, 64) and a["k"].shape == (2, 512, 64) == a["v"].shape
    d0, d1 = W.decode_inputs(c, 0, 0), W.decode_inputs(c, 1, 0)
    assert d0["q"].shape == (1, 4, 64) and not np.array_equal(d0["q"], d1["q"])


def test_bf16_values_are_exact_in_bf16():
    c = W.custom_config(dtype="bf16", m=64, tau=8, lead_text=8, n_visual=40, d=32)
    t = W.layer_inputs(c, 0, 0)
    for k in ("q_win", "k", "v"):
        x = torch.from_numpy(t[k])
        assert torch.equal(x.to(torch.bfloat16).float(), x)
    raw = np.array([1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -9], dtype=np.float32)  # ties-to-even cases
    got = W.round_to_dtype(raw.copy(), "bf16")
    assert np.array_equal(got, torch.from_numpy(raw).to(torch.bfloat16).float().numpy())


def test_sinks_are_scaled_visual_keys_and_temperatures_in_range():
    c = W.CONFIGS[0]
    pos = W.sink_positions(c, 0, 0)
    lo, hi = c.visual_span
    assert pos.shape == (2, 8) and pos.min() >= lo and pos.max() < hi
    k = W.layer_inputs(c, 0, 0)["k"]
    norms = np.linalg.norm(k[0], axis=1)
    assert norms[pos[0]].min() > 2.5 * np.median(norms)
    T = W.temperatures(c)
    assert T.shape == (2,) and np.all((T >= 0.5) & (T <= 2.0))
    np.testing.assert_allclose(W.sm_scale(c), 1 / (T * 8.0), rtol=1e-6)


def test_frame_structure_shares_a_mean_inside_a_frame():
    c = W.custom_config(cid=98, m=8 + 4 * 50 + 8, tau=8, lead_text=8, n_visual=200, frame_len=50, d=32, sinks=2)
    k = W.layer_inputs(c, 0, 0, want_v=False)["k"][0]
    f0, f1 = k[8:58].mean(0), k[58:108].mean(0)
    assert np.linalg.norm(f0) > 3 and np.linalg.norm(f0 - f1) > 3     # frame means ~ N(0,1)^32
