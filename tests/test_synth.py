"""The seeded input generators: determinism, bf16 storage rounding, workload shapes (CPU only)."""
import numpy as np
import torch

from paper_2206_03382_amd import synth


def test_bf16_rounding_matches_torch():
    a = np.random.default_rng(0).standard_normal(100000).astype(np.float32) * 37.0
    a[:4] = [1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -0.0, 1e-30]          # exact ties (to even both ways), signed zero, tiny
    r = synth.round_to_bf16(a)
    ref = torch.from_numpy(a).to(torch.bfloat16)
    assert np.array_equal(r, ref.float().numpy())
    bits = synth.bf16_bits(r)
    assert np.array_equal(bits.view(np.int16), ref.view(torch.int16).numpy())
    assert np.array_equal(synth.bf16_bits_to_f32(bits), r)


def test_inputs_are_seeded_and_shaped():
    cfg = synth.CONFIGS[1].scaled(T=64, M=32, H=48, E=4)
    a, b = synth.make_inputs(cfg, seed=0, bias_std=0.1), synth.make_inputs(cfg, seed=0, bias_std=0.1)
    c = synth.make_inputs(cfg, seed=1, bias_std=0.1)
    for key in ("x", "Wg", "W1", "W2", "b1", "b2"):
        assert np.array_equal(a[key], b[key]) and not np.array_equal(a[key], c[key])
        assert np.array_equal(a[key], synth.round_to_bf16(a[key]))       # bf16-representable values
    assert a["x"].shape == (64, 32) and a["Wg"].shape == (32, 4) and a["W1"].shape == (4, 32, 48) and a["W2"].shape == (4, 48, 32)
    assert abs(float(a["W1"].std()) - 32 ** -0.5) < 0.02 and abs(float(a["W2"].std()) - 48 ** -0.5) < 0.02


def test_workload_recipes():
    v = synth.make_inputs(synth.CONFIGS[2].scaled(T=128, M=64, H=32, E=4))["x"]
    assert np.abs(v.mean(axis=1)).max() < 0.02 and np.abs(v.std(axis=1) - 1).max() < 0.05   # LayerNorm'd then bf16
    b = synth.zipf_gate_bias(64)
    w = np.exp(b.astype(np.float64) / 2.0)
    assert abs(w.sum() - 1) < 1e-5 and np.all(np.diff(b) < 0)
    np.testing.assert_allclose(w[0] / w[9], 10 ** 1.2, rtol=1e-5)
    shapes = [(c.T, c.M, c.H, c.E, c.k, c.f) for c in synth.CONFIGS]
    assert shapes == [(1024, 256, 512, 4, 1, 1.0), (16384, 2048, 2048, 8, 2, 1.25), (25088, 768, 3072, 32, 1, 1.25),
                      (65536, 1024, 4096, 64, 2, 1.0), (131072, 4096, 1024, 128, 8, 2.0)]
