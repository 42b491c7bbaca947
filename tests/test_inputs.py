"""The seeded input generator: determinism, distribution, exact bf16 rounding."""
import numpy as np

import dfk_inputs as di


def test_counter_based_and_deterministic():
    a = di.standard_normal(7, 1000)
    b = di.standard_normal(7, 1000, chunk=64)
    np.testing.assert_array_equal(a, b)                       # chunking does not matter
    np.testing.assert_array_equal(di.standard_normal(7, 10), a[:10])  # draw i depends on (seed, i) only
    assert not np.array_equal(a, di.standard_normal(8, 1000))


def test_moments():
    z = di.standard_normal(123, 400000)
    assert abs(z.mean()) < 0.01 and abs(z.std() - 1.0) < 0.01
    assert abs(np.mean(z ** 3)) < 0.03 and abs(np.mean(z ** 4) - 3.0) < 0.08


def test_bf16_round_to_nearest_even():
    f = np.array([1.0, 1.00390625, 1.01171875, -1.00390625, 0.0, 3.140625], np.float32)
    # 1 + 2^-8 is a tie between 0x3F80 and 0x3F81 -> even (0x3F80);
    # 1 + 3*2^-8 is a tie between 0x3F81 and 0x3F82 -> even (0x3F82)
    bits = di.f32_to_bf16_bits(f)
    assert list(bits) == [0x3F80, 0x3F80, 0x3F82, 0xBF80, 0x0000, 0x4049]
    back = di.bf16_bits_to_f32(bits)
    assert back[0] == 1.0 and back[5] == 3.140625
    assert np.isnan(di.bf16_bits_to_f32(di.f32_to_bf16_bits(np.array([np.nan], np.float32))))[0]


def test_recipe_scales_and_torch_roundtrip():
    t = di.mlp_inputs(4, 256, 512, seed=3)
    assert t["X"].dtype == np.uint16 and t["Wg"].shape == (512, 256) and t["Wd"].shape == (512, 256)
    assert abs(di.as_f64(t["Wg"]).std() * 16.0 - 1.0) < 0.02      # std 1/sqrt(d_model)
    assert abs(di.as_f64(t["Wd"]).std() * np.sqrt(512.0) - 1.0) < 0.02
    import torch
    tt = di.to_torch(t["Wg"])
    assert tt.dtype == torch.bfloat16
    np.testing.assert_array_equal(di.to_numpy(tt), t["Wg"])
    f = di.mlp_inputs(1, 8, 16, seed=3, dtype="fp32")
    np.testing.assert_array_equal(di.to_numpy(di.to_torch(f["X"])), f["X"])
