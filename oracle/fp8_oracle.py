"""Plain CPU oracle for the 8-bit storage of a compressed KV cache.

TEST INFRASTRUCTURE ONLY.  The paper (MEDA, arXiv 2502.17599) names quantisation of the KV cache as work that
can be combined with its method (Limitations section) and fixes no scheme, so there is nothing of the paper to pin
here; the scheme below is this build's choice and its oracle is pinned against the definition of the number format
and against an independent library conversion.  It shares no code with the HIP path and imports nothing from it.

Format: the 8-bit floating-point format "E4M3" of the OCP 8-bit floating point specification: 1 sign bit,
4 exponent bits (bias 7), 3 mantissa bits; no infinities; the all-ones pattern S.1111.111 is NaN; the largest
finite magnitude is S.1111.110 = 448; subnormals are m * 2^-9.

Scheme (per row of head_dim elements, the unit a decoding step reads):
  scale  = max|x| / 448                computed in float32 (1 when the row is all zero)
  code_i = E4M3(clamp(x_i / scale, -448, 448))   division in float32, round to nearest, ties to even
  x_i   ~= value(code_i) * scale
Both sides take the quantisation decision in float32, as the kernel does.

Pins (tests/test_oracle_fp8.py): the code table against the format's definition (named values, monotone, symmetric),
the encoder against brute-force nearest-neighbour search over the table with the tie rule, encode(decode(c)) == c,
saturation, the encoder against torch's float8_e4m3fn conversion, and for rows: the largest element maps to 448,
zero rows, the relative error bound 2^-4 per element.
"""
from __future__ import annotations

import numpy as np

E4M3_MAX = 448.0


def e4m3_decode_table() -> np.ndarray:
    """Value of each of the 256 codes as float64 (NaN for the two NaN codes), from the format's definition."""
    out = np.empty(256, dtype=np.float64)
    for c in range(256):
        sign = -1.0 if c & 0x80 else 1.0
        e = (c >> 3) & 0xF
        m = c & 0x7
        if e == 0xF and m == 0x7:
            out[c] = np.nan
        elif e == 0:
            out[c] = sign * m * 2.0 ** -9            # subnormal: 0.m * 2^(1 - 7)
        else:
            out[c] = sign * (1.0 + m / 8.0) * 2.0 ** (e - 7)
    return out


def e4m3_encode(x) -> np.ndarray:
    """Codes of the finite values ``x``: nearest representable value, ties to the even mantissa, magnitudes
    above 448 saturate to 448.  Arithmetic on exact binary fractions (frexp / ldexp), no table search."""
    x = np.asarray(x, dtype=np.float64)
    a = np.minimum(np.abs(x), E4M3_MAX)
    sign = np.where(np.signbit(x), 0x80, 0).astype(np.int64)
    # exponent of the binade the value lies in, not below the smallest normal binade (2^-6): below it the
    # grid keeps the subnormal spacing 2^-9
    mant, ex = np.frexp(a)                       # a = mant * 2^ex, mant in [0.5, 1)
    e = np.maximum(ex - 1, -6)                   # a in [2^e, 2^(e+1)) for normals
    step = np.ldexp(1.0, e - 3)                  # spacing of the grid in that binade (3 mantissa bits)
    q = np.rint(a / step).astype(np.int64)       # numpy rint rounds half to even; a / step is exact
    # q in [0, 16]: q < 8 subnormal (code = q), q = 16 carries into the next binade
    carry = q == 16
    e = np.where(carry, e + 1, e)
    q = np.where(carry, 8, q)
    code = np.where(q < 8, q, ((e + 7) << 3) | (q - 8))
    return (sign | code).astype(np.uint8)


def quantize_rows(x) -> tuple:
    """``x`` [n, d] (values that float32 holds exactly): returns (codes uint8 [n, d], scales float32 [n])."""
    x32 = np.asarray(x, dtype=np.float32)
    absmax = np.abs(x32).max(axis=1)
    scales = np.where(absmax > 0, absmax / np.float32(E4M3_MAX), np.float32(1.0)).astype(np.float32)
    y = (x32 / scales[:, None]).astype(np.float32)            # float32 division, round to nearest even
    y = np.clip(y, np.float32(-E4M3_MAX), np.float32(E4M3_MAX))
    return e4m3_encode(y.astype(np.float64)), scales


def dequantize_rows(codes, scales) -> np.ndarray:
    """float64 values of quantised rows: table value times the row's scale (exact in float64)."""
    table = e4m3_decode_table()
    return table[np.asarray(codes, dtype=np.uint8)] * np.asarray(scales, dtype=np.float64)[:, None]
