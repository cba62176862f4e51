"""Pins of the oracle's 4-bit integer weight decoding (oracle/int4_weights.py): a worked example
written out by hand, the order of the codes and of the two codes in a byte, the row scale."""
import os

import numpy as np

from oracle import int4_weights as i4

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "int4_example.txt")


def _worked_example():
    rows = []
    for line in open(GOLDEN):
        if not line.startswith("bytes"):
            continue
        tok = line.split()
        i_scale, i_val = tok.index("scale"), tok.index("values")
        rows.append(([int(t, 16) for t in tok[1:i_scale]], float(tok[i_scale + 1]),
                     [float(t) for t in tok[i_val + 1:]]))
    return rows


def test_worked_example():
    rows = _worked_example()
    assert len(rows) == 2
    packed = np.array([r[0] for r in rows], dtype=np.uint8)
    scale = np.array([r[1] for r in rows], dtype=np.float32)
    want = np.array([r[2] for r in rows], dtype=np.float64)
    assert np.array_equal(i4.dequantise(packed, scale), want)


def test_codes_are_the_integers_minus_8_to_7_in_order():
    packed = np.array([[lo | (hi << 4) for lo, hi in zip(range(0, 16, 2), range(1, 16, 2))]], dtype=np.uint8)
    w = i4.dequantise(packed, np.ones(1, dtype=np.float32))
    assert w.tolist() == [[float(v) for v in range(-8, 8)]]


def test_low_four_bits_hold_the_even_k():
    packed = np.array([[0x0F, 0xF0]], dtype=np.uint8)
    assert i4.unpack_codes(packed).tolist() == [[15, 0, 0, 15]]
    assert i4.dequantise(packed, np.array([2.0])).tolist() == [[14.0, -16.0, -16.0, 14.0]]


def test_one_scale_per_output_row_and_zero_code():
    rng = np.random.Generator(np.random.PCG64(11))
    packed = rng.integers(0, 256, size=(5, 6)).astype(np.uint8)
    scale = rng.uniform(0.01, 2.0, size=5).astype(np.float32)
    w = i4.dequantise(packed, scale)
    assert w.shape == (5, 12)
    for n in range(5):
        for j in range(6):
            b = int(packed[n, j])
            assert w[n, 2 * j] == ((b & 15) - 8) * float(scale[n])
            assert w[n, 2 * j + 1] == ((b >> 4) - 8) * float(scale[n])
    # the code 8 is exactly zero whatever the scale
    assert np.array_equal(i4.dequantise(np.full((2, 3), 0x88, dtype=np.uint8), np.array([3.0, 7.0])),
                          np.zeros((2, 6)))
