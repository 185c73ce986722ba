"""The seeded input generators: reproducible, and bf16 rounding agrees with torch's (CPU only)."""
import numpy as np
import torch

from paper_2504_06095_amd import inputs as I


def test_normal_is_reproducible_and_keyed():
    a = I.normal_f32(0, "X", (64, 33))
    b = I.normal_f32(0, "X", (64, 33))
    c = I.normal_f32(0, "dZ", (64, 33))
    d = I.normal_f32(1, "X", (64, 33))
    assert np.array_equal(a, b) and not np.array_equal(a, c) and not np.array_equal(a, d)
    big = I.normal_f32(0, "X", (400_000,), std=0.02)
    assert abs(float(big.mean())) < 2e-4 and abs(float(big.std()) - 0.02) < 2e-4


def test_bf16_rounding_matches_torch():
    x = I.normal_f32(3, "r", (100_000,))
    x[:6] = [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38]  # ties to even both ways, near-max
    bits = I.round_to_bf16_bits(x)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, want)
    back = I.bf16_bits_to_f32(bits)
    assert np.array_equal(back, torch.from_numpy(x).to(torch.bfloat16).float().numpy())
