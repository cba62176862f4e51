"""Low-precision weight storage for the CPU oracle: dequantise, then compute in float64.
TEST INFRASTRUCTURE ONLY (same rules as verify_oracle.py: nothing of the product imports this
file, and this file imports nothing of the product).

The paper's App. C runs the verifier with weights stored in fewer bits and dequantised on the
fly.  The MI355X form of that idea used here: every linear layer's matrix W [out, in] is stored
as 8-bit floating point codes (E4M3 of the OCP 8-bit floating point specification: 1 sign bit,
4 exponent bits with bias 7, 3 mantissa bits, no infinities, S.1111.111 = NaN, largest finite
value 448) together with one float32 scale per output row:

    W[n][k] = value(code[n][k]) * scale[n]

The oracle's definition of such a model is the ordinary float64 forward pass (verify_oracle.py)
on the dequantised matrices - what is computed does not depend on how the weights are stored.

Pins (tests/test_oracle_fp8.py): the values the specification names (1.0, the largest and the
smallest normal and subnormal numbers, signs, the NaN codes), monotonic order of the positive
codes, and the decoding of all 256 codes by torch's float8_e4m3fn type.
"""
from __future__ import annotations

import numpy as np


def e4m3_values() -> np.ndarray:
    """float64 value of each of the 256 E4M3 codes (OCP 8-bit floating point, E4M3):
    normal numbers (-1)^s 2^(e-7) (1 + m/8) for e = 1..15, subnormals (-1)^s 2^-6 (m/8) for
    e = 0, except that e = 15, m = 7 is NaN."""
    out = np.empty(256, dtype=np.float64)
    for code in range(256):
        s, e, m = code >> 7, (code >> 3) & 15, code & 7
        if e == 15 and m == 7:
            v = np.nan
        elif e == 0:
            v = 2.0 ** -6 * (m / 8.0)
        else:
            v = 2.0 ** (e - 7) * (1.0 + m / 8.0)
        out[code] = -v if s else v
    return out


def dequantise(codes: np.ndarray, row_scale: np.ndarray) -> np.ndarray:
    """codes uint8 [out, in], row_scale [out] -> float64 [out, in]."""
    codes = np.asarray(codes)
    assert codes.dtype == np.uint8 and codes.ndim == 2 and row_scale.shape == (codes.shape[0],)
    return e4m3_values()[codes] * np.asarray(row_scale, dtype=np.float64)[:, None]
