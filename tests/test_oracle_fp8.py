"""Pins of the oracle's 8-bit weight decoding (oracle/fp8_weights.py) against what the OCP
8-bit floating point specification fixes for E4M3 and against torch's float8_e4m3fn type."""
import numpy as np
import torch

from oracle import fp8_weights as f8


def test_named_values_of_the_format():
    v = f8.e4m3_values()
    assert v[0x00] == 0.0 and v[0x80] == 0.0 and np.signbit(v[0x80])
    assert v[0x38] == 1.0 and v[0xB8] == -1.0          # exponent field = bias, mantissa 0
    assert v[0x7E] == 448.0 and v[0xFE] == -448.0      # largest finite: 2^8 * 1.75
    assert v[0x08] == 2.0 ** -6                        # smallest normal
    assert v[0x01] == 2.0 ** -9                        # smallest subnormal
    assert v[0x07] == 7 * 2.0 ** -9                    # largest subnormal
    assert v[0x40] == 2.0 and v[0x3C] == 1.5 and v[0x39] == 1.125
    assert np.isnan(v[0x7F]) and np.isnan(v[0xFF])     # the only two NaN codes, no infinities
    assert np.isfinite(np.delete(v, [0x7F, 0xFF])).all()


def test_positive_codes_are_ordered_and_mirror_the_negative_ones():
    v = f8.e4m3_values()
    assert (np.diff(v[:0x7F]) > 0).all()
    assert np.array_equal(v[0x80:0xFF], -v[0x00:0x7F])


def test_all_codes_against_torch():
    codes = torch.arange(256, dtype=torch.uint8)
    ref = codes.view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(f8.e4m3_values(), ref, equal_nan=True)


def test_dequantise_applies_one_scale_per_output_row():
    rng = np.random.Generator(np.random.PCG64(5))
    codes = rng.integers(0, 0x7F, size=(6, 10)).astype(np.uint8)
    scale = rng.uniform(0.01, 2.0, size=6).astype(np.float32)
    w = f8.dequantise(codes, scale)
    v = f8.e4m3_values()
    for n in range(6):
        for k in range(10):
            assert w[n, k] == v[codes[n, k]] * float(scale[n])
