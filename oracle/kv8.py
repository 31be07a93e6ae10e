"""CPU oracle, part 3: 8-bit KV cache (test infrastructure only; nothing in the product path imports this).

The paper names KV-cache compression as the way past the long-sequence memory wall (Section 4.2, last paragraph, and
Section 5) but fixes no format.  The reading taken here, stated in full because the paper is silent:

* a cache row (one slot of one key/value head, head_dim numbers) is stored as head_dim 8-bit codes plus one fp32 scale;
  K rows and V rows are quantised the same way, independently;
* the code format is OCP FP8 E4M3: 1 sign, 4 exponent (bias 7), 3 mantissa bits; no infinities; codes 0x7F / 0xFF are
  NaN and never produced; largest finite value 448 = 2^8 x 1.75; subnormals m/8 x 2^-6;
* scale = max|row| / 448 (1 for an all-zero row), code = the E4M3 value nearest to x / scale, ties to the even code,
  values clamped to +-448 first; the quantised decision is taken in fp32 (amax, the two divisions), the precision the
  kernels take it in, on the fp32 value of the row (K after RoPE);
* the row the attention reads is value(code) x scale, the product taken in fp32.

Pins (tests/test_oracle_kv8.py): the decode table against the format's closed form and its known landmarks; rounding
against brute-force nearest-value search, against hand-picked ties and against torch's float8_e4m3fn cast; error
bound 2^-4 relative per element above the subnormal range; idempotence; scale landmarks; zero rows.
"""
from __future__ import annotations

import numpy as np

F32 = np.float32
E4M3_MAX = 448.0


def e4m3_value(code: int) -> float:
    """Value of one E4M3 code, written out from the format definition (NaN for 0x7F and 0xFF)."""
    s = -1.0 if code & 0x80 else 1.0
    e = (code >> 3) & 0xF
    m = code & 0x7
    if e == 0xF and m == 0x7:
        return float("nan")
    if e == 0:
        return s * (m / 8.0) * 2.0 ** -6
    return s * (1.0 + m / 8.0) * 2.0 ** (e - 7)


def e4m3_table() -> np.ndarray:
    """All 256 code values as float64."""
    return np.array([e4m3_value(c) for c in range(256)], dtype=np.float64)


def e4m3_round(y) -> np.ndarray:
    """Codes (uint8) of the E4M3 values nearest to y (any float array, |y| <= 448 after clamping), ties to even."""
    y = np.clip(np.asarray(y, dtype=np.float64), -E4M3_MAX, E4M3_MAX)
    grid = e4m3_table()[:0x7F]                       # the 127 non-negative finite values, ascending with the code
    a = np.abs(y)
    hi = np.searchsorted(grid, a, side="left")       # first grid value >= a
    hi = np.minimum(hi, len(grid) - 1)
    lo = np.maximum(hi - 1, 0)
    d_lo, d_hi = a - grid[lo], grid[hi] - a
    pick_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (hi % 2 == 0))   # ties: the even code (mantissa LSB 0)
    code = np.where(pick_hi, hi, lo).astype(np.uint8)
    neg = np.signbit(y) & (code != 0)                # -0 is stored as +0
    return np.where(neg, code | 0x80, code).astype(np.uint8)


def quantize_rows(x):
    """x [..., hd] -> (codes uint8 [..., hd], scale fp32 [...]).  Decisions in fp32, see the module header."""
    x = np.asarray(x, dtype=F32)
    amax = np.max(np.abs(x), axis=-1)
    scale = np.where(amax > 0, amax / F32(E4M3_MAX), F32(1.0)).astype(F32)
    y = (x / scale[..., None]).astype(F32)
    return e4m3_round(y), scale


def dequantize_rows(codes, scale) -> np.ndarray:
    """value(code) x scale with the product in fp32, returned as float64."""
    v = e4m3_table()[np.asarray(codes, dtype=np.uint8)].astype(F32)
    return (v * np.asarray(scale, dtype=F32)[..., None]).astype(F32).astype(np.float64)


def roundtrip_rows(x) -> np.ndarray:
    """What the attention reads back for rows written as x."""
    codes, scale = quantize_rows(x)
    return dequantize_rows(codes, scale)
