"""Pins for the oracle's bfloat16 rounding (storage format of the largest workload)."""
import numpy as np
import torch

import oracle
from oracle.buffer import bf16_bits_to_f32


def _f(bits):
    return np.array([bits], dtype=np.uint32).view(np.float32)[0]


def test_known_bit_patterns():
    L = oracle.lib()
    assert L.oracle_bf16_bits(1.0) == 0x3F80
    assert L.oracle_bf16_bits(-2.0) == 0xC000
    assert L.oracle_bf16_bits(0.0) == 0x0000
    assert L.oracle_bf16_bits(_f(0x3F808000)) == 0x3F80     # tie, even stays
    assert L.oracle_bf16_bits(_f(0x3F818000)) == 0x3F82     # tie, odd rounds up to even
    assert L.oracle_bf16_bits(_f(0x3F808001)) == 0x3F81     # just above the tie
    assert L.oracle_bf16_bits(_f(0x3F807FFF)) == 0x3F80     # just below
    assert L.oracle_bf16_bits(_f(0x7F7FFFFF)) == 0x7F80     # largest fp32 rounds to +inf
    assert L.oracle_bf16_bits(float("inf")) == 0x7F80
    nan_bits = L.oracle_bf16_bits(float("nan"))
    assert (nan_bits & 0x7F80) == 0x7F80 and (nan_bits & 0x007F) != 0


def test_matches_an_independent_library_and_is_idempotent():
    rng = np.random.default_rng(30)
    x = np.concatenate([rng.normal(size=20000).astype(np.float32) * 3,
                        rng.uniform(-2, 0.5, 20000).astype(np.float32),
                        np.array([1e-40, -1e-40, 3.3e38, 65504.0, 1e-30], np.float32)])
    bits, vals = oracle.quantize_bf16(x)
    want = torch.from_numpy(x).to(torch.bfloat16)
    np.testing.assert_array_equal(bits.view(np.int16), want.view(torch.int16).numpy())
    np.testing.assert_array_equal(vals, want.to(torch.float32).numpy())
    bits2, vals2 = oracle.quantize_bf16(vals)
    np.testing.assert_array_equal(bits, bits2)
    np.testing.assert_array_equal(vals, vals2)
    np.testing.assert_array_equal(bf16_bits_to_f32(bits), vals)
    # relative error bound of round-to-nearest with 8 significand bits
    nz = np.abs(x) > 1e-30
    assert np.all(np.abs(vals[nz] - x[nz]) <= np.abs(x[nz]) * 2.0 ** -8)
