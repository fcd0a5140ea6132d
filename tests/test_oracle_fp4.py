"""Pins of the oracle's E2M1 encoder / decoder (oracle/fp4.py) against facts other than itself: the
format's published value table, the nearest-value property by brute force over the grid (every tie and
its neighbours included), saturation, the nibble order of a packed byte, and the size of the error."""
import numpy as np

from oracle import attention as oa
from oracle import fp4

# the sixteen E2M1 values in code order (OCP Microscaling formats, element type FP4 E2M1)
TABLE = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0, -0.0, -0.5, -1.0, -1.5, -2.0, -3.0, -4.0, -6.0]


def test_decode_is_the_format_table():
    v = fp4.e2m1_decode(np.arange(16))
    assert v.tolist() == TABLE and np.signbit(v[8])
    # the same table from the bit fields: sign s, exponent e (bias 1), mantissa m
    for c in range(16):
        s, e, m = c >> 3, (c >> 1) & 3, c & 1
        mag = m * 0.5 if e == 0 else (1 + m / 2) * 2.0 ** (e - 1)
        assert v[c] == (-mag if s else mag)


def test_every_code_round_trips():
    codes = np.arange(16, dtype=np.uint8)
    assert np.array_equal(fp4.e2m1_encode(fp4.e2m1_decode(codes)), codes)     # -0 keeps its sign bit


def test_encode_is_the_nearest_value_ties_to_even_by_brute_force():
    grid = np.array(TABLE[:8])
    g = np.random.default_rng(0)
    mids = (grid[:-1] + grid[1:]) / 2
    xs = np.concatenate([g.uniform(0, 7, 2000), g.uniform(0, 0.6, 500), mids, np.nextafter(mids, 0), np.nextafter(mids, 9),
                         grid, [6.0, 6.5, 1e9, np.inf, 2.0 ** -20]])
    for x in xs:
        d = np.abs(grid - min(x, 6.0))
        best = np.flatnonzero(d == d.min())
        want = best[0] if len(best) == 1 else [b for b in best if b % 2 == 0][0]     # tie: mantissa bit 0
        assert fp4.e2m1_encode([x])[0] == want, (x, want)
        assert fp4.e2m1_encode([-x])[0] == (want | 8)
    # the ties written out: 0.25 -> 0, 0.75 -> 1, 1.25 -> 1, 1.75 -> 2, 2.5 -> 2, 3.5 -> 4, 5 -> 4
    assert fp4.e2m1_decode(fp4.e2m1_encode(mids)).tolist() == [0.0, 1.0, 1.0, 2.0, 2.0, 4.0, 4.0]


def test_packing_puts_the_even_column_in_the_low_nibble():
    codes = np.array([[1, 2, 3, 15], [8, 0, 7, 9]], dtype=np.uint8)
    packed = fp4.pack_rows(codes)
    assert packed.tolist() == [[0x21, 0xF3], [0x08, 0x97]]
    assert np.array_equal(fp4.unpack_rows(packed), codes)
    g = np.random.default_rng(3)
    c = g.integers(0, 16, (5, 7, 32)).astype(np.uint8)
    assert np.array_equal(fp4.unpack_rows(fp4.pack_rows(c)), c)


def test_attention_over_decoded_codes_with_column_scales_folded_into_the_factors():
    """A scale per latent column moves into the query (K' side) and the output (V' side); attention over the decoded
    codes then approximates the unquantised result with the error of a 1-bit mantissa, and is exact on grid values."""
    g = np.random.default_rng(2)
    S, r = 400, 32
    sig = np.exp(-np.arange(r) / 32.0)
    K, V, q = g.standard_normal((S, r)) * sig, g.standard_normal((S, r)) * sig, g.standard_normal(r)
    sk, sv = np.abs(K).max(axis=0) / 6.0, np.abs(V).max(axis=0) / 6.0            # per column
    Kc = fp4.e2m1_decode(fp4.quantise_latent(K / sk))
    Vc = fp4.e2m1_decode(fp4.quantise_latent(V / sv))
    ref = oa.latent_attn_decode(q, K, V, 0.2)
    got = sv * oa.latent_attn_decode(q * sk, Kc, Vc, 0.2)
    err = np.linalg.norm(got - ref) / np.linalg.norm(ref)
    assert 0.01 < err < 0.5              # coarse (sixteen levels), but the same attention
    Kg = fp4.e2m1_decode(g.integers(0, 16, (S, r)))
    Vg = fp4.e2m1_decode(g.integers(0, 16, (S, r)))
    a = oa.latent_attn_decode(q, Kg, Vg, 0.05)
    b = oa.latent_attn_decode(q, fp4.e2m1_decode(fp4.quantise_latent(Kg)), fp4.e2m1_decode(fp4.quantise_latent(Vg)), 0.05)
    assert np.array_equal(a, b)
