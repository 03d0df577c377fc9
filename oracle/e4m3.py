"""OCP e4m3 (8-bit floating point, 4 exponent bits, bias 7, 3 mantissa bits) in NumPy.

TEST INFRASTRUCTURE ONLY, like kd_oracle.py: the reference the library's quantiser kernel
(kd_quantize_e4m3) is checked against bit for bit, and the means by which the tests build fp8 teacher
operands and the exact values they stand for.  Shares no code with the HIP kernels and imports nothing
from the package.  Context: the paper runs the teacher's inference in FP8 (Table 3); quantising the
teacher head for the logit recomputation is this build's extension.

Format (OCP 8-bit floating point specification, E4M3): no infinities, 0x7f / 0xff are NaN, largest
magnitude 448, subnormals in steps of 2^-9.  The quantiser is written as a nearest-value search over the
table of representable values (ties to the even code), not as bit manipulation; it is pinned to
torch's float8_e4m3fn cast and to hand-picked ties in tests/test_e4m3_oracle.py.
"""
from __future__ import annotations

import numpy as np


def e4m3_values() -> np.ndarray:
    """The 256 values of the OCP e4m3 byte codes (sign, 4 exponent bits with bias 7, 3 mantissa
    bits; no infinities; 0x7f and 0xff are NaN), as float64."""
    c = np.arange(256)
    e, m = (c >> 3) & 15, c & 7
    v = np.where(e == 0, m * 2.0 ** -9, (1.0 + m / 8.0) * 2.0 ** (e.astype(np.float64) - 7))
    v[(e == 15) & (m == 7)] = np.nan
    return np.where(c & 128, -v, v)


def quantize_e4m3(x: np.ndarray, scale: float) -> np.ndarray:
    """uint8 e4m3 codes of x * (1 / scale), the reciprocal and the product in fp32: nearest
    representable value, ties to the even code, magnitudes beyond 448 saturate, NaN -> 0x7f | sign.
    Written as a search over the value table, not as bit manipulation."""
    x = np.asarray(x, dtype=np.float32)
    inv = np.float32(1.0) / np.float32(scale)
    pos = e4m3_values()[:127]                       # codes 0x00..0x7e: 0 .. 448, increasing
    out = np.empty(x.shape, dtype=np.uint8)
    xf, of = x.reshape(-1), out.reshape(-1)
    for i0 in range(0, xf.size, 1 << 24):           # blocks only bound the temporaries
        y = (xf[i0:i0 + (1 << 24)] * inv).astype(np.float32)
        a = np.abs(y).astype(np.float64)
        hi = np.clip(np.searchsorted(pos, a, side="left"), 1, 126)
        lo = hi - 1
        d_lo, d_hi = a - pos[lo], pos[hi] - a
        code = np.where(d_lo < d_hi, lo, np.where(d_hi < d_lo, hi, np.where(lo % 2 == 0, lo, hi)))
        code = np.where(a >= 448.0, 126, code)
        code = np.where(np.isnan(a), 127, code)
        of[i0:i0 + (1 << 24)] = (code | np.where(np.signbit(y), 128, 0)).astype(np.uint8)
    return out
