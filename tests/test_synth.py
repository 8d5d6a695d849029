"""Host-side checks of the seeded input generators (CPU only)."""
import numpy as np
import torch

from paper_2505_24544_amd import synth


def test_bf16_rounding_matches_torch_rne():
    r = np.random.default_rng(0)
    a = np.concatenate([r.standard_normal(200000).astype(np.float32) * 10.0 ** r.integers(-20, 20, 200000),
                        np.array([0.0, -0.0, np.inf, -np.inf, np.nan, 1.00390625, 1.01171875, 3.3895314e38],
                                 np.float32)]).astype(np.float32)
    want = torch.from_numpy(a).to(torch.bfloat16)
    got = synth.round_to_bf16(a)
    assert np.array_equal(got, want.float().numpy(), equal_nan=True)
    bits = synth.f32_to_bf16_bits(a)
    assert np.array_equal(bits[~np.isnan(a)], want.view(torch.int16).numpy().view(np.uint16)[~np.isnan(a)])
    assert np.array_equal(synth.bf16_bits_to_f32(bits), got, equal_nan=True)


def test_generators_are_seeded_and_shaped():
    cfg = synth.CONFIGS["c3"].with_(batch=1, seq_q=40, seq_kv=40, hidden=256, n_q_heads=4, n_kv_heads=2)
    a, b = synth.make_inputs(cfg), synth.make_inputs(cfg)
    assert set(a) == {"xq", "xkv", "wq", "wk", "wv", "wo", "dy"}
    for n in a:
        assert a[n].dtype == np.float32 and np.array_equal(a[n], b[n])
        assert np.array_equal(a[n], synth.round_to_bf16(a[n]))     # bf16-representable
    assert a["wk"].shape == (256, 2 * 128) and a["wq"].shape == (256, 4 * 128)
    ms = (a["xkv"].astype(np.float64) ** 2).mean(-1)
    assert np.allclose(ms, 1.0, atol=2e-2)
    c = synth.make_inputs(cfg.with_(seed_base=cfg.seed_base + 1))
    assert not np.array_equal(a["xq"], c["xq"])


def test_outlier_recipe_has_heavy_channels():
    cfg = synth.CONFIGS["c5"].with_(seq_q=2000, seq_kv=2000, hidden=512, n_q_heads=4, n_kv_heads=4)
    x = synth.make_inputs(cfg, with_dy=False)["xkv"][0]
    big = (np.abs(x) > 6).sum(axis=1)
    assert 5 <= (big >= 4).sum() <= 60          # ~1% of 2000 positions carry outlier channels
    c1 = synth.make_inputs(synth.CONFIGS["c1"])
    assert c1["xq"].shape == (1, 128, 256) and c1["wq"].shape == (256, 256)
