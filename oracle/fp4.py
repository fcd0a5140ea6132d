"""Oracle (test infrastructure): a latent cache stored as 4-bit floats.

The paper reports its compression combined with 4-bit cache quantisation
(Section 6.2, the rows that add KVQuant, a non-uniform 4-bit scheme, to FDC) and
fixes no number format for the combination. Reading taken here: the latent rows
K' = x.A_k, V' = x.A_v are stored as OCP "E2M1" codes, the 4-bit element type of
the Microscaling formats: 1 sign bit, 2 exponent bits with bias 1, 1 mantissa
bit, no infinities and no NaN, i.e. the sixteen values +-{0, 0.5, 1, 1.5, 2, 3,
4, 6}. Rounding is to the nearest value, ties to the even mantissa; values
beyond +-6 saturate. Two codes share a byte: the element with the even column
index sits in bits 3..0, its right neighbour in bits 7..4. No block scales are
stored: a scale per (head, latent column) folds into the factors (the column of
A divided, the row of B_k or of B_v.W_o multiplied by it), so attention sees
exactly the decoded code values.

Written from the format's definition (value table, integer comparisons against
the midpoints of the grid); no library conversion is used.
"""
from __future__ import annotations

import numpy as np

E2M1_MAX = 6.0
# magnitudes of the codes 0..7 (exponent field e, mantissa bit m): e = 0 is subnormal, m * 0.5; otherwise
# (1 + m / 2) * 2^(e - 1)
_MAGNITUDE = [(m * 0.5) if e == 0 else (1.0 + m / 2.0) * 2.0 ** (e - 1) for e in range(4) for m in range(2)]


def e2m1_decode(codes) -> np.ndarray:
    """4-bit codes (0..15, sign in bit 3) -> float64 values."""
    c = np.asarray(codes).astype(np.int64)
    assert ((c >= 0) & (c <= 15)).all()
    mag = np.array(_MAGNITUDE, dtype=np.float64)[c & 7]
    return np.where(c & 8, -mag, mag)


def _encode_one(x: float) -> int:
    s = 8 if np.signbit(x) else 0
    a = min(abs(float(x)), E2M1_MAX)
    best = 0
    for code in range(1, 8):           # walk up the grid: move on while a is past the midpoint (or on it, towards even)
        lo, hi = _MAGNITUDE[code - 1], _MAGNITUDE[code]
        mid = (lo + hi) / 2.0
        if a > mid or (a == mid and code % 2 == 0):      # even code = mantissa bit 0
            best = code
        else:
            break
    return s | best


def e2m1_encode(x) -> np.ndarray:
    """float array -> codes 0..15 (uint8), saturating, round to nearest, ties to even. NaN is not accepted."""
    a = np.asarray(x, dtype=np.float64)
    assert not np.isnan(a).any()
    flat = a.ravel()
    out = np.fromiter((_encode_one(v) for v in flat), dtype=np.uint8, count=flat.size)
    return out.reshape(a.shape)


def pack_rows(codes) -> np.ndarray:
    """Codes [..., r] (r even) -> bytes [..., r / 2]: column 2 j in the low nibble, 2 j + 1 in the high one."""
    c = np.asarray(codes, dtype=np.uint8)
    assert c.shape[-1] % 2 == 0 and (c <= 15).all()
    return (c[..., 0::2] | (c[..., 1::2] << 4)).astype(np.uint8)


def unpack_rows(packed) -> np.ndarray:
    """Inverse of pack_rows: bytes [..., n] -> codes [..., 2 n]."""
    p = np.asarray(packed, dtype=np.uint8)
    out = np.empty(p.shape[:-1] + (2 * p.shape[-1],), dtype=np.uint8)
    out[..., 0::2] = p & 0xF
    out[..., 1::2] = p >> 4
    return out


def quantise_latent(rows, compute_dtype=np.float32) -> np.ndarray:
    """Codes of latent rows: the product is first held in fp32 (the precision the paper's setting, bf16 storage
    with fp32 sums, accumulates in), the code decision is taken on that value."""
    return e2m1_encode(np.asarray(rows, dtype=np.float64).astype(compute_dtype).astype(np.float64))
