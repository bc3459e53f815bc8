"""The seeded input generators: determinism, distributions, and bf16 rounding against a library."""
import numpy as np
import pytest

from paper_2511_09741_amd import inputs as I


def test_bf16_rounding_matches_library_rne():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(0)
    a = np.concatenate([rng.standard_normal(100000).astype(np.float32) * 10.0 ** rng.integers(-6, 6, 100000),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38], dtype=np.float32)]).astype(np.float32)
    bits = I.f32_to_bf16_bits(a)
    ref = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, ref)
    back = I.bf16_bits_to_f32(bits)
    assert np.array_equal(back, torch.from_numpy(a).to(torch.bfloat16).float().numpy())
    # ties to even: 1 + 2^-8 is exactly between 1 and 1 + 2^-7
    assert I.bf16_bits_to_f32(I.f32_to_bf16_bits(np.array([1.00390625], np.float32)))[0] == 1.0
    assert I.bf16_bits_to_f32(I.f32_to_bf16_bits(np.array([1.01171875], np.float32)))[0] == 1.015625


def test_generators_are_seeded_and_shaped():
    cfg = I.CONFIGS["C1"]
    x, dy = I.make_activations(cfg, seed=0)
    x2, _ = I.make_activations(cfg, seed=0)
    x3, _ = I.make_activations(cfg, seed=1)
    assert x.shape == (1, 128, 64) and x.dtype == np.float32
    assert np.array_equal(x, x2) and not np.array_equal(x, x3) and not np.array_equal(x, dy)
    w = I.make_weights(cfg, seed=0)
    assert w["w_qkv"].shape == (192, 64) and w["w_down"].shape == (64, 176) and w["w_gate_up"].shape == (352, 64)
    assert np.all(w["gamma_attn"] == 1) and np.all(w["gamma_mlp"] == 1)
    assert abs(float(np.std(w["w_qkv"])) - 0.02) < 0.002 and abs(float(np.std(x)) - 1.0) < 0.05
    w1 = I.make_weights(cfg, seed=0, layer=1)
    assert not np.array_equal(w["w_o"], w1["w_o"])


def test_storage_roundtrip_is_exact():
    cfg = I.CONFIGS["C1"].with_(dtype=I.BF16)
    x, _ = I.make_activations(cfg, seed=3)
    assert x.dtype == np.uint16
    x64 = I.to_f64(x, I.BF16)
    assert np.array_equal(I.f32_to_bf16_bits(x64.astype(np.float32)), x)   # already representable


def test_config_presets_follow_the_named_workloads():
    c = I.CONFIGS
    assert (c["C2"].S, c["C2"].H, c["C2"].n_heads, c["C2"].head_dim, c["C2"].I) == (8192, 4096, 32, 128, 11008)
    assert (c["C3"].S, c["C3"].H) == (32768, 4096)
    assert (c["C4"].B, c["C4"].S, c["C4"].H, c["C4"].I, c["C4"].n_layers) == (2, 16384, 5120, 13824, 4)
    assert (c["C5"].S, c["C5"].H, c["C5"].n_heads, c["C5"].I, c["C5"].n_microbatches) == (16384, 8192, 64, 22016, 4)
    for k in c.values():
        assert k.H == k.n_heads * k.head_dim
