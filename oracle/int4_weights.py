"""4-bit integer weight storage for the CPU oracle: dequantise, then compute in float64.
TEST INFRASTRUCTURE ONLY (same rules as verify_oracle.py: nothing of the product imports this
file, and this file imports nothing of the product).

The paper's App. C (Tables 5 and 6) runs the verifier with int8 and int4 weights; it says
nothing about the format.  The reading taken here: every linear layer's matrix W [out, in] is
stored as 4-bit codes with one float32 scale per output row,

    W[n][k] = (code[n][k] - 8) * scale[n],      code in 0 .. 15, i.e. integers -8 .. 7,

two codes per byte, the code of the even k in the low four bits of byte k / 2.  As with the
8-bit floating point storage (fp8_weights.py) the oracle's definition of such a model is the
ordinary float64 forward pass (verify_oracle.py) on the dequantised matrices.

Pins (tests/test_oracle_int4.py): a worked example written out by hand
(tests/golden/int4_example.txt), the sixteen codes in order, the nibble order, and the scale
acting per output row.
"""
from __future__ import annotations

import numpy as np


def unpack_codes(packed: np.ndarray) -> np.ndarray:
    """uint8 [out, in / 2] -> codes uint8 [out, in] (0 .. 15): byte j of a row holds k = 2j in its
    low four bits and k = 2j + 1 in its high four bits."""
    packed = np.asarray(packed)
    assert packed.dtype == np.uint8 and packed.ndim == 2
    out = np.empty((packed.shape[0], 2 * packed.shape[1]), dtype=np.uint8)
    out[:, 0::2] = packed & 0x0F
    out[:, 1::2] = packed >> 4
    return out


def dequantise(packed: np.ndarray, row_scale: np.ndarray) -> np.ndarray:
    """packed uint8 [out, in / 2], row_scale [out] -> float64 [out, in]."""
    codes = unpack_codes(packed)
    row_scale = np.asarray(row_scale, dtype=np.float64)
    assert row_scale.shape == (codes.shape[0],)
    return (codes.astype(np.float64) - 8.0) * row_scale[:, None]
