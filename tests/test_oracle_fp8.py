"""Pins of the oracle's E4M3 encoder / decoder (oracle/fp8.py) against facts other than itself:
the format's published constants, torch's own float8_e4m3fn conversion (an independent library
routine), exhaustive round trips and the nearest-value property checked by brute force."""
import numpy as np
import pytest
import torch

from oracle import fp8
from oracle import attention as oa


def test_decode_matches_the_format_constants_and_torch():
    v = fp8.e4m3_decode(np.arange(256, dtype=np.uint8))
    assert v[0x00] == 0.0 and v[0x80] == 0.0 and np.signbit(v[0x80])
    assert v[0x01] == 2.0 ** -9             # smallest subnormal
    assert v[0x07] == 7 * 2.0 ** -9         # largest subnormal
    assert v[0x08] == 2.0 ** -6             # smallest normal
    assert v[0x38] == 1.0 and v[0x3C] == 1.5 and v[0x40] == 2.0
    assert v[0x7E] == 448.0 and v[0xFE] == -448.0
    assert np.isnan(v[0x7F]) and np.isnan(v[0xFF])
    ref = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    ok = (v == ref) | (np.isnan(v) & np.isnan(ref))
    assert ok.all()


def test_every_code_round_trips():
    codes = np.array([c for c in range(256) if c not in (0x7F, 0xFF)], dtype=np.uint8)
    assert np.array_equal(fp8.e4m3_encode(fp8.e4m3_decode(codes)), codes)


def test_encode_is_the_nearest_code_ties_to_even_by_brute_force():
    finite = np.array([c for c in range(0x7F)], dtype=np.uint8)            # non-negative finite codes, ascending
    grid = fp8.e4m3_decode(finite)
    g = np.random.default_rng(0)
    xs = np.concatenate([g.uniform(0, 460, 400), g.uniform(0, 0.05, 400), np.ldexp(g.uniform(1, 2, 400), g.integers(-12, 9, 400)),
                         (grid[:-1] + grid[1:]) / 2,                       # every tie
                         np.nextafter((grid[:-1] + grid[1:]) / 2, 0), np.nextafter((grid[:-1] + grid[1:]) / 2, 1e9)])
    for x in xs:
        d = np.abs(grid - min(x, 448.0))
        best = np.flatnonzero(d == d.min())
        want = best[0] if len(best) == 1 else [b for b in best if b % 2 == 0][0]   # tie: even mantissa = even code
        assert fp8.e4m3_encode([x])[0] == want, (x, want)
        assert fp8.e4m3_encode([-x])[0] == (want | 0x80)


def test_encode_matches_torch_on_fp32_inputs_and_saturates():
    g = np.random.default_rng(1)
    x = np.concatenate([g.standard_normal(5000) * 3, g.standard_normal(2000) * 200, g.standard_normal(2000) * 0.01,
                        [0.0, -0.0, 448.0, 464.0, -464.0, 2.0 ** -10, 3 * 2.0 ** -11, 2.0 ** -9]]).astype(np.float32)
    inside = np.abs(x) <= 464.0          # torch rounds |x| in (448, 464] to 448 and turns anything larger into NaN
    ref = torch.from_numpy(x[inside]).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(fp8.e4m3_encode(x[inside]), ref)
    assert np.array_equal(fp8.e4m3_encode([465.0, 1e9, -1e9, np.inf, -np.inf]), [0x7E, 0x7E, 0xFE, 0x7E, 0xFE])


def test_attention_over_decoded_codes_approaches_the_unquantised_result():
    """Scales folded into the factors: with K'/s_k and V'/s_v stored as codes and s_k, s_v moved into the
    query and the output, attention over the decoded codes stays close to the unquantised one (3 mantissa
    bits: a few percent), and is exact when the rows are already on the grid."""
    g = np.random.default_rng(2)
    S, r = 300, 32
    K, V, q = g.standard_normal((S, r)), g.standard_normal((S, r)), g.standard_normal(r)
    sk, sv = np.abs(K).max() / 448.0, np.abs(V).max() / 448.0
    Kc, Vc = fp8.e4m3_decode(fp8.quantise_latent(K / sk)), fp8.e4m3_decode(fp8.quantise_latent(V / sv))
    ref = oa.latent_attn_decode(q, K, V, 0.2)
    got = sv * oa.latent_attn_decode(q * sk, Kc, Vc, 0.2)
    assert np.linalg.norm(got - ref) / np.linalg.norm(ref) < 0.08
    Kg, Vg = fp8.e4m3_decode(g.integers(0, 0x7E, (S, r)).astype(np.uint8)), fp8.e4m3_decode(g.integers(0x80, 0xFE, (S, r)).astype(np.uint8))
    a = oa.latent_attn_decode(q, Kg, Vg, 0.01)
    b = oa.latent_attn_decode(q, fp8.e4m3_decode(fp8.quantise_latent(Kg)), fp8.e4m3_decode(fp8.quantise_latent(Vg)), 0.01)
    assert np.array_equal(a, b)
