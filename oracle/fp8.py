"""Decoding of the 8-bit KV cache format for the CPU oracle: TEST INFRASTRUCTURE ONLY.

App. F of the paper stores K and V as fp8 and keeps queries and the arithmetic in 16/32 bits.
The format here is OCP E4M3: bit 7 sign, bits 6..3 exponent E (bias 7), bits 2..0 mantissa M;
E = 0: value = M / 8 * 2**-6 (zero and subnormals); otherwise (1 + M / 8) * 2**(E - 7); the
single non-finite code is E = 15, M = 7 (NaN); there are no infinities and the largest
magnitude is 1.75 * 2**8 = 448.  Written from the format definition; shares nothing with the
encoder of the input generators or with the GPU path (which uses the hardware conversion).
"""
from __future__ import annotations

import numpy as np


def e4m3_to_f64(codes: np.ndarray) -> np.ndarray:
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    sign = np.where(c & 0x80, -1.0, 1.0)
    E = (c >> 3) & 0xF
    M = (c & 0x7).astype(np.float64)
    sub = M / 8.0 * 2.0 ** -6
    nor = (1.0 + M / 8.0) * np.exp2((E - 7).astype(np.float64))
    val = np.where(E == 0, sub, nor)
    val = np.where((E == 15) & ((c & 0x7) == 7), np.nan, val)
    return sign * val
