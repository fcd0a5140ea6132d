"""Oracle (test infrastructure): a latent cache stored as 8-bit floats.

The paper treats quantisation of the cache as orthogonal to its dimensional
compression and reports the two combined (Section 6.2, the rows that add
KVQuant to FDC); it fixes no number format. Reading taken here: the latent rows
K' = x.A_k, V' = x.A_v are stored as OCP "E4M3" codes (1 sign, 4 exponent bits
with bias 7, 3 mantissa bits; no infinities, the all-ones exponent with
mantissa 111 is NaN, largest finite value 448), rounded to nearest, ties to
even, values beyond +-448 saturating to +-448. Per-head scales are the caller's:
they fold into A (divide), B_k and B_v.W_o (multiply), so what attention sees is
exactly the decoded code values.

Everything below is written from the format's definition with integer
arithmetic on the binary expansion of the input; no library conversion is used.
"""
from __future__ import annotations

import math

import numpy as np

E4M3_MAX = 448.0
_BIAS = 7
_MANT = 3


def e4m3_decode(codes) -> np.ndarray:
    """uint8 codes -> float64 values (NaN for 0x7f / 0xff)."""
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    sign = np.where(c & 0x80, -1.0, 1.0)
    e = (c >> _MANT) & 0xF
    m = c & 0x7
    normal = np.ldexp(1.0 + m / 8.0, e - _BIAS)
    sub = np.ldexp(m / 8.0, 1 - _BIAS)
    v = np.where(e == 0, sub, normal)
    v = np.where((e == 0xF) & (m == 0x7), np.nan, v)
    return sign * v


def _encode_one(x: float) -> int:
    """One finite value -> code: saturate, then round to nearest representable, ties to even."""
    s = 0x80 if math.copysign(1.0, x) < 0 else 0
    a = min(abs(x), E4M3_MAX)
    if a == 0.0:
        return s
    # spacing of the grid around a: 2^(e-3) for normals with exponent e >= -6, 2^-9 below 2^-6
    e = max(math.floor(math.log2(a)), 1 - _BIAS)
    if 2.0 ** e > a:          # guard against log2 rounding up at powers of two
        e -= 1
    e = max(e, 1 - _BIAS)
    q = a / 2.0 ** (e - _MANT)            # in [8, 16) for normals, [0, 8) for subnormals; exact in float64
    n = math.floor(q)
    r = q - n
    if r > 0.5 or (r == 0.5 and n % 2 == 1):
        n += 1
    if n == 16:               # rounded up into the next binade
        n, e = 8, e + 1
    if n < 8:                 # subnormal (e == -6): code exponent field 0, mantissa n
        return s | n
    return s | ((e + _BIAS) << _MANT) | (n - 8)


def e4m3_encode(x) -> np.ndarray:
    """float array -> uint8 codes (saturating, round to nearest even). NaN is not accepted."""
    a = np.asarray(x, dtype=np.float64)
    assert not np.isnan(a).any()
    flat = a.ravel()
    out = np.fromiter((_encode_one(float(v)) for v in flat), dtype=np.uint8, count=flat.size)
    return out.reshape(a.shape)


def quantise_latent(rows, compute_dtype=np.float32) -> np.ndarray:
    """Codes of latent rows as a kernel stores them: the product is first held in the kernel's
    accumulator precision (fp32), the code decision is taken on that value."""
    return e4m3_encode(np.asarray(rows, dtype=np.float64).astype(compute_dtype).astype(np.float64))
