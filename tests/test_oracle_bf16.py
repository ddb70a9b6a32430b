"""Pins for the oracle's bfloat16 rounding: exhaustive round trip, explicit tie cases, and
agreement with an independent implementation (torch's fp32 -> bf16 conversion)."""
import numpy as np
import torch

from oracle.bf16 import round_to_bf16, bf16_bits_to_f64, f64_to_bf16_bits


def test_roundtrip_all_bit_patterns():
    bits = np.arange(1 << 16, dtype=np.uint16)
    vals = bf16_bits_to_f64(bits)
    fin = np.isfinite(vals)
    assert np.array_equal(f64_to_bf16_bits(vals[fin]), bits[fin])
    assert np.array_equal(round_to_bf16(vals[fin]), vals[fin])


def test_ties_to_even_and_no_double_rounding():
    ulp = 2.0 ** -7                      # spacing of bf16 in [1, 2)
    assert round_to_bf16(1 + ulp / 2) == 1.0             # tie -> even significand
    assert round_to_bf16(1 + 3 * ulp / 2) == 1 + 2 * ulp  # tie -> even significand
    assert round_to_bf16(1 + ulp / 2 + 2.0 ** -40) == 1 + ulp   # just above the tie
    assert round_to_bf16(-(1 + ulp / 2 - 2.0 ** -40)) == -1.0
    assert round_to_bf16(0.0) == 0.0 and round_to_bf16(2.0 ** -133) == 2.0 ** -133
    assert np.isinf(round_to_bf16(3.4e38)) and round_to_bf16(3.38e38) < np.inf


def test_matches_torch_on_fp32_values():
    rng = np.random.default_rng(7)
    x = (rng.standard_normal(200000) * np.exp(rng.uniform(-60, 60, 200000))).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(round_to_bf16(x.astype(np.float64)), want)
