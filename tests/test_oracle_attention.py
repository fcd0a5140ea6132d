"""Pins for the float64 oracle's numerics: each test ties the oracle to a fact that is
fixed by the paper's identities or by mathematics, computed by another route
(torch's scaled_dot_product_attention on uncompressed K/V, closed forms, explicit
Python loops), never by re-typing the oracle's own expression.
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import attention as oa
from oracle.factors import truncated_svd_factors
from workloads import generators as gen


def _std_mha(x_q, x_kv, Wq, Wk, Wv, Wo, d_h, causal):
    """Standard multi-head attention from the uncompressed weights (library routine)."""
    H = len(Wk)
    q = torch.stack([torch.from_numpy(x_q @ Wq[h]) for h in range(H)])[None]      # [1,H,Sq,d_h]
    k = torch.stack([torch.from_numpy(x_kv @ Wk[h]) for h in range(H)])[None]
    v = torch.stack([torch.from_numpy(x_kv @ Wv[h]) for h in range(H)])[None]
    Sq, Skv = q.shape[2], k.shape[2]
    mask = None
    if causal:
        pos = (Skv - Sq) + torch.arange(Sq)[:, None]
        mask = torch.arange(Skv)[None, :] <= pos
    o = F.scaled_dot_product_attention(q, k, v, attn_mask=mask)                   # scale 1/sqrt(d_h)
    o = o[0].permute(1, 0, 2).reshape(Sq, H * d_h).numpy()
    return o @ Wo


def _latent_chain(x_q, x_kv, Wq, Wk, Wv, Wo, d_h, ranks_k, ranks_v, causal, decode):
    H = len(Wk)
    Ak, Bk, Av, Bv = [], [], [], []
    for h in range(H):
        a, b, _ = truncated_svd_factors(Wk[h], ranks_k[h])
        Ak.append(a), Bk.append(b)
        a, b, _ = truncated_svd_factors(Wv[h], ranks_v[h])
        Av.append(a), Bv.append(b)
    K_lat = oa.project_latent_kv(x_kv, Ak)
    V_lat = oa.project_latent_kv(x_kv, Av)
    q = np.stack([x_q @ Wq[h] for h in range(H)], axis=1)                        # [T,H,d_h]
    q_lat = oa.absorb_query(q, Bk)
    scale = 1.0 / math.sqrt(d_h)
    if decode:
        o_lat = [oa.latent_attn_decode(q_lat[h][0], K_lat[h], V_lat[h], scale)[None, :] for h in range(H)]
    else:
        o_lat = [oa.latent_attn_prefill(q_lat[h], K_lat[h], V_lat[h], scale, causal) for h in range(H)]
    M = oa.fold_output(Bv, Wo, d_h)
    return oa.apply_output(o_lat, M)


def _weights(d, d_h, H, decay, g, exact_rank=None):
    Wk = [gen.planted_weight(d, d_h, decay, g, exact_rank).W for _ in range(H)]
    Wv = [gen.planted_weight(d, d_h, decay, g, exact_rank).W for _ in range(H)]
    Wq = [g.standard_normal((d, d_h)) / math.sqrt(d) for _ in range(H)]
    Wo = g.standard_normal((H * d_h, d)) / math.sqrt(H * d_h)
    return Wq, Wk, Wv, Wo


@pytest.mark.parametrize("decode,causal", [(True, False), (False, True), (False, False)])
def test_full_rank_equals_standard_attention(decode, causal):
    # Section 3 (R R^T = I): with every dimension kept and orthogonal B the latent path is exact.
    g = gen.make_rng(11)
    d, d_h, H, S = 48, 16, 3, 23
    Wq, Wk, Wv, Wo = _weights(d, d_h, H, 4.0, g)
    x = gen.hidden_states(S, d, g)
    x_q = x[-1:] if decode else x[-9:]          # decode: one query; prefill: last 9 positions
    ref = _std_mha(x_q, x, Wq, Wk, Wv, Wo, d_h, causal and not decode)
    got = _latent_chain(x_q, x, Wq, Wk, Wv, Wo, d_h, [d_h] * H, [d_h] * H, causal, decode)
    assert np.max(np.abs(got - ref)) <= 1e-10 * max(1.0, np.max(np.abs(ref)))


@pytest.mark.parametrize("decode", [True, False])
def test_exact_low_rank_equals_uncompressed(decode):
    # Section 2: K' B ~= K, with equality when W has exactly r non-zero singular values.
    g = gen.make_rng(5)
    d, d_h, H, S, r = 40, 16, 2, 17, 5
    Wq, Wk, Wv, Wo = _weights(d, d_h, H, 4.0, g, exact_rank=r)
    x = gen.hidden_states(S, d, g)
    x_q = x[-1:] if decode else x
    ref = _std_mha(x_q, x, Wq, Wk, Wv, Wo, d_h, not decode)
    got = _latent_chain(x_q, x, Wq, Wk, Wv, Wo, d_h, [r] * H, [r + 2] * H, True, decode)
    assert np.max(np.abs(got - ref)) <= 1e-10 * max(1.0, np.max(np.abs(ref)))


def test_truncation_changes_result_and_rk_rv_are_independent():
    # guards against a chain that silently ignores the rank (would make the two pins above vacuous)
    g = gen.make_rng(6)
    d, d_h, H, S = 40, 16, 2, 17
    Wq, Wk, Wv, Wo = _weights(d, d_h, H, 4.0, g)
    x = gen.hidden_states(S, d, g)
    full = _latent_chain(x[-1:], x, Wq, Wk, Wv, Wo, d_h, [16] * H, [16] * H, False, True)
    cut_k = _latent_chain(x[-1:], x, Wq, Wk, Wv, Wo, d_h, [4] * H, [16] * H, False, True)
    cut_v = _latent_chain(x[-1:], x, Wq, Wk, Wv, Wo, d_h, [16] * H, [4] * H, False, True)
    assert np.max(np.abs(full - cut_k)) > 1e-6
    assert np.max(np.abs(full - cut_v)) > 1e-6
    assert np.max(np.abs(cut_k - cut_v)) > 1e-6


def test_eckart_young_closed_form():
    # ||W - A B||_F^2 = sum_{i >= r} s_i^2; for s_i = e^{-i/8}, d_h = 64 the tail is geometric.
    g = gen.make_rng(0)
    pw = gen.planted_weight(96, 64, 8.0, g)
    for r in (16, 32, 48, 64):
        A, B, sigma = truncated_svd_factors(pw.W, r)
        err = np.linalg.norm(pw.W - A @ B, "fro") ** 2
        closed = (math.exp(-r / 4) - math.exp(-16.0)) / (1 - math.exp(-0.25))
        assert abs(err - closed) <= 1e-10
        assert np.allclose(sigma, pw.s, atol=1e-12)
        # A.B equals the product of the generator's own leading factors (signs cancel in the product)
        planted = (pw.U[:, :r] * pw.s[None, :r]) @ pw.V[:, :r].T
        assert np.max(np.abs(A @ B - planted)) <= 1e-10
        # the reading "B has orthonormal rows, sigma sits in A"
        assert np.max(np.abs(B @ B.T - np.eye(r))) <= 1e-12
        assert np.allclose(np.linalg.norm(A, axis=0), pw.s[:r], atol=1e-12)


def test_eckart_young_closed_form_decay32():
    g = gen.make_rng(1)
    pw = gen.planted_weight(160, 128, 32.0, g)
    for r in (16, 64, 112):
        A, B, _ = truncated_svd_factors(pw.W, r)
        err = np.linalg.norm(pw.W - A @ B, "fro") ** 2
        closed = (math.exp(-r / 16) - math.exp(-8.0)) / (1 - math.exp(-1 / 16))
        assert abs(err - closed) <= 1e-9


def test_score_error_bound():
    # |q.k - q'.k'| <= ||q|| ||x|| s_r  (spectral norm of W - A B is the first dropped singular value)
    g = gen.make_rng(2)
    d, d_h, r = 64, 32, 12
    pw = gen.planted_weight(d, d_h, 6.0, g)
    A, B, sigma = truncated_svd_factors(pw.W, r)
    x = gen.hidden_states(50, d, g)
    q = g.standard_normal((7, d_h))
    exact = q @ (x @ pw.W).T
    lat = oa.absorb_query(q[:, None, :], [B])[0] @ oa.project_latent_kv(x, [A])[0].T
    bound = np.linalg.norm(q, axis=1)[:, None] * np.linalg.norm(x, axis=1)[None, :] * sigma[r]
    assert np.all(np.abs(exact - lat) <= bound + 1e-12)
    assert np.max(np.abs(exact - lat)) > 1e-3 * np.max(bound)   # bound is not vacuous


def test_softmax_properties_and_limits():
    g = gen.make_rng(3)
    S, rk, rv = 37, 6, 5
    K = g.standard_normal((S, rk))
    V = g.standard_normal((S, rv))
    q = g.standard_normal(rk)
    o, p = oa.latent_attn_decode(q, K, V, 0.7, return_probs=True)
    assert abs(p.sum() - 1.0) <= 1e-14 and np.all(p >= 0)
    assert np.all(o <= V.max(axis=0) + 1e-14) and np.all(o >= V.min(axis=0) - 1e-14)
    # zero keys -> uniform weights -> mean of the values
    o0 = oa.latent_attn_decode(q, np.zeros_like(K), V, 0.7)
    assert np.max(np.abs(o0 - V.mean(axis=0))) <= 1e-14
    # one dominating key -> its value row
    Kd = K.copy()
    Kd[11] = 1e3 * q
    od = oa.latent_attn_decode(q, Kd, V, 0.7)
    assert np.max(np.abs(od - V[11])) <= 1e-12
    # a single key
    assert np.array_equal(oa.latent_attn_decode(q, K[:1], V[:1], 0.7), V[0])
    # no keys
    assert np.array_equal(oa.latent_attn_decode(q, K[:0], V[:0], 0.7), np.zeros(rv))
    # ordering of the keys does not matter, as long as values move with them
    perm = g.permutation(S)
    op = oa.latent_attn_decode(q, K[perm], V[perm], 0.7)
    assert np.max(np.abs(op - o)) <= 1e-14
    # scale matters (a dropped scale would pass the tests above)
    assert np.max(np.abs(oa.latent_attn_decode(q, K, V, 1.4) - o)) > 1e-3


def test_shift_and_chunk_invariance():
    g = gen.make_rng(4)
    S, rk, rv = 101, 8, 7
    K = g.standard_normal((S, rk)) * 3
    V = g.standard_normal((S, rv))
    q = g.standard_normal(rk)
    scale = 0.9
    whole = oa.latent_attn_decode(q, K, V, scale)
    # adding a constant to every score: append a constant latent column hit by a unit query entry
    K1 = np.concatenate([K, np.full((S, 1), 5.0)], axis=1)
    q1 = np.concatenate([q, [3.0]])
    assert np.max(np.abs(oa.latent_attn_decode(q1, K1, V, scale) - whole)) <= 1e-13
    # any partition of the key range, merged by log-sum-exp, gives the same output
    for cuts in ([0, 101], [0, 1, 101], [0, 17, 64, 100, 101], list(range(0, 102, 1))):
        ms, ls, accs = [], [], []
        for a, b in zip(cuts[:-1], cuts[1:]):
            s = [scale * sum(q[i] * K[t, i] for i in range(rk)) for t in range(a, b)]
            m = max(s)
            e = [math.exp(v - m) for v in s]
            ms.append(m), ls.append(sum(e))
            accs.append(sum(e[t - a] * V[t] for t in range(a, b)))
        merged = oa.lse_merge(ms, ls, accs)
        assert np.max(np.abs(merged - whole)) <= 1e-12


def test_brute_force_tiny_chain():
    # H <= 2, d <= 8, d_h <= 4, S <= 5: reconstruct K, V and do dense softmax with explicit loops
    g = gen.make_rng(9)
    d, d_h, H, S = 8, 4, 2, 5
    rk, rv = [2, 3], [3, 1]
    Wq, Wk, Wv, Wo = _weights(d, d_h, H, 2.0, g)
    x = gen.hidden_states(S, d, g)
    got = _latent_chain(x, x, Wq, Wk, Wv, Wo, d_h, rk, rv, True, False)

    y = [[0.0] * d for _ in range(S)]
    for h in range(H):
        Ak, Bk, _ = truncated_svd_factors(Wk[h], rk[h])
        Av, Bv, _ = truncated_svd_factors(Wv[h], rv[h])
        Kh = [[sum(x[t, a] * (Ak @ Bk)[a, j] for a in range(d)) for j in range(d_h)] for t in range(S)]
        Vh = [[sum(x[t, a] * (Av @ Bv)[a, j] for a in range(d)) for j in range(d_h)] for t in range(S)]
        # query projected onto the kept right-singular subspace: q Bk^T Bk
        P = Bk.T @ Bk
        for i in range(S):
            qi = [sum(x[i, a] * Wq[h][a, j] for a in range(d)) for j in range(d_h)]
            qp = [sum(qi[a] * P[a, j] for a in range(d_h)) for j in range(d_h)]
            sc = [sum(qp[j] * Kh[t][j] for j in range(d_h)) / math.sqrt(d_h) for t in range(i + 1)]
            mx = max(sc)
            e = [math.exp(v - mx) for v in sc]
            z = sum(e)
            oh = [sum(e[t] / z * Vh[t][j] for t in range(i + 1)) for j in range(d_h)]
            for c in range(d):
                y[i][c] += sum(oh[j] * Wo[h * d_h + j, c] for j in range(d_h))
    assert np.max(np.abs(got - np.array(y))) <= 1e-11


def test_causal_prefill_last_row_is_decode_and_rows_are_prefixes():
    g = gen.make_rng(12)
    S, rk, rv = 33, 16, 16
    Q = g.standard_normal((S, rk))
    K = g.standard_normal((S, rk))
    V = g.standard_normal((S, rv))
    O = oa.latent_attn_prefill(Q, K, V, 0.3, causal=True)
    for i in (0, 1, 15, 16, 32):
        assert np.max(np.abs(O[i] - oa.latent_attn_decode(Q[i], K[:i + 1], V[:i + 1], 0.3))) <= 1e-14
    # chunked prefill: the last 5 queries against the full key range
    O5 = oa.latent_attn_prefill(Q[-5:], K, V, 0.3, causal=True)
    assert np.max(np.abs(O5 - O[-5:])) <= 1e-14


def test_direct_latent_statistics():
    # column i of x.(U_r diag(s_r)) has variance s_i^2 for x ~ N(0, I): the fast generator matches
    g = gen.make_rng(13)
    d, d_h, r, T = 256, 64, 32, 20000
    pw = gen.planted_weight(d, d_h, 8.0, g)
    A, _, _ = truncated_svd_factors(pw.W, r)
    K = oa.project_latent_kv(gen.hidden_states(T, d, g), [A])[0]
    Kd = gen.direct_latent(T, r, 8.0, g)
    s2 = pw.s[:r] ** 2
    assert np.allclose(K.var(axis=0), s2, rtol=0.06)
    assert np.allclose(Kd.var(axis=0), s2, rtol=0.06)


def test_bf16_packing_round_trip():
    g = gen.make_rng(14)
    x = g.standard_normal(4096)
    bits = gen.f64_to_bf16_bits(x)
    back = gen.bf16_bits_to_f64(bits)
    ref = torch.from_numpy(x).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(back, ref)
