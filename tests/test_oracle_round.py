"""Pins for the oracle's 16-bit weight rounding: torch's CPU conversions (another library than
the one the oracle uses), hand-made ties, range ends."""
import numpy as np
import pytest
import torch

import oracle


def _samples():
    rng = np.random.default_rng(0)
    a = np.concatenate([
        rng.normal(0, 0.05, 20000), rng.normal(0, 50.0, 2000), rng.uniform(-1e-7, 1e-7, 2000),   # incl. f16 subnormals / underflow
        np.array([0.0, -0.0, 1.0, -1.0, 65504.0, 65519.9, 65520.0, 1e5, -1e5, 6e-8, 2.98e-8, 2.99e-8, 1e-45, 3.3e38, 3.4e38,
                  np.inf, -np.inf])]).astype(np.float32)
    # every float32 whose low 16 bits are exactly the tie pattern or next to it
    hi = rng.integers(0, 0x7F7F, 4000).astype(np.uint32) << np.uint32(16)
    ties = np.concatenate([hi | np.uint32(0x8000), hi | np.uint32(0x7FFF), hi | np.uint32(0x8001)]).view(np.float32)
    return np.concatenate([a, ties, -ties])


def test_bf16_is_torch_bfloat16_bit_for_bit():
    a = _samples()
    got = oracle.round_weights(a, "bf16")
    want = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    assert np.all((got.view(np.uint32) & 0xFFFF) == 0)


def test_f16_is_torch_float16_bit_for_bit():
    a = _samples()
    got = oracle.round_weights(a, "f16")
    want = torch.from_numpy(a).to(torch.float16).to(torch.float32).numpy()
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_hand_made_cases():
    f = lambda v, fmt: float(oracle.round_weights(np.array([v], np.float32), fmt)[0])
    # binary16 keeps 10 fraction bits: 1 + 2^-11 is a tie -> even (1.0); 1 + 3 * 2^-11 -> 1 + 2^-9
    assert f(1.0 + 2.0 ** -11, "f16") == 1.0
    assert f(1.0 + 3 * 2.0 ** -11, "f16") == 1.0 + 2.0 ** -9
    assert f(1.0 + 2.0 ** -11 + 2.0 ** -20, "f16") == 1.0 + 2.0 ** -10
    assert f(65520.0, "f16") == np.inf and f(65519.0, "f16") == 65504.0
    assert f(2.0 ** -25, "f16") == 0.0 and f(2.0 ** -24, "f16") == 2.0 ** -24      # half the smallest subnormal ties to 0
    # bfloat16 keeps 7 fraction bits
    assert f(1.0 + 2.0 ** -8, "bf16") == 1.0
    assert f(1.0 + 3 * 2.0 ** -8, "bf16") == 1.0 + 2.0 ** -6
    assert f(1.0 + 2.0 ** -8 + 2.0 ** -20, "bf16") == 1.0 + 2.0 ** -7
    assert f(3.4e38, "bf16") == np.inf
    assert np.isnan(f(np.nan, "bf16")) and np.isnan(f(np.nan, "f16"))
    # idempotent; sign-symmetric
    a = _samples()
    for fmt in ("f16", "bf16"):
        r = oracle.round_weights(a, fmt)
        assert np.array_equal(oracle.round_weights(r, fmt).view(np.uint32), r.view(np.uint32))
        assert np.array_equal(oracle.round_weights(-a, fmt).view(np.uint32), (-r).view(np.uint32))
