"""Pins for the post-RoPE oracle (Sections 3 and 5.1): RoPE against the complex-number form and its
relative-position property, the rotation identity (Q_p R)(K_p R)^T = Q_p K_p^T, the equivalence of
full-rank post-RoPE latent attention with standard RoPE attention, and the truncation error in
terms of the dropped singular values.
"""
import math

import numpy as np
import torch
import torch.nn.functional as F

from oracle import attention as oa
from oracle import rope as orp
from workloads import generators as gen


def _rope_complex(x, pos, base=10000.0):
    """Independent route: pairs as complex numbers times e^{i pos theta}."""
    d = x.shape[1]
    theta = base ** (-2.0 * np.arange(d // 2) / d)
    z = (x[:, 0::2] + 1j * x[:, 1::2]) * np.exp(1j * np.asarray(pos)[:, None] * theta[None, :])
    y = np.empty_like(x)
    y[:, 0::2], y[:, 1::2] = z.real, z.imag
    return y


def test_rope_matches_complex_form_and_hand_case():
    g = gen.make_rng(1)
    d, T = 16, 9
    cos, sin = orp.rope_tables(50, d)
    x = g.standard_normal((T, d))
    pos = g.integers(0, 50, T)
    assert np.max(np.abs(orp.rope(x, pos, cos, sin) - _rope_complex(x, pos))) <= 1e-13
    # d_h = 2, position 3, base irrelevant (theta_0 = 1): rotation of (1, 0) by 3 rad
    c2, s2 = orp.rope_tables(4, 2)
    y = orp.rope(np.array([[1.0, 0.0]]), [3], c2, s2)
    assert np.allclose(y, [[math.cos(3.0), math.sin(3.0)]], atol=1e-15)
    # position 0 is the identity; norms are preserved
    assert np.array_equal(orp.rope(x, np.zeros(T, int), cos, sin), x)
    assert np.allclose(np.linalg.norm(orp.rope(x, pos, cos, sin), axis=1), np.linalg.norm(x, axis=1), rtol=1e-14)


def test_rope_scores_depend_on_relative_position_only():
    g = gen.make_rng(2)
    d = 32
    cos, sin = orp.rope_tables(200, d)
    q, k = g.standard_normal((1, d)), g.standard_normal((1, d))
    ref = (orp.rope(q, [17], cos, sin) @ orp.rope(k, [5], cos, sin).T)[0, 0]
    for shift in (1, 40, 150):
        got = (orp.rope(q, [17 + shift], cos, sin) @ orp.rope(k, [5 + shift], cos, sin).T)[0, 0]
        assert abs(got - ref) <= 1e-12
    other = (orp.rope(q, [18], cos, sin) @ orp.rope(k, [5], cos, sin).T)[0, 0]
    assert abs(other - ref) > 1e-6


def _post_rope_inputs(seed, d=48, d_h=16, S=40, n_cal=300):
    g = gen.make_rng(seed)
    Wq = g.standard_normal((d, d_h)) / math.sqrt(d)
    Wk = gen.planted_weight(d, d_h, 4.0, g).W
    cos, sin = orp.rope_tables(max(S, n_cal), d_h)
    # calibration on random tokens (Section 5.1: R does not depend on the tokens)
    xc = gen.hidden_states(n_cal, d, g)
    pc = np.arange(n_cal)
    R, sigma = orp.common_rotation(orp.rope(xc @ Wq, pc, cos, sin), orp.rope(xc @ Wk, pc, cos, sin))
    x = gen.hidden_states(S, d, g)
    pos = np.arange(S)
    Qp, Kp = orp.rope(x @ Wq, pos, cos, sin), orp.rope(x @ Wk, pos, cos, sin)
    V = g.standard_normal((S, d_h))
    return R, sigma, Qp, Kp, V, d_h


def test_rotation_identity_and_orthogonality():
    R, sigma, Qp, Kp, V, d_h = _post_rope_inputs(3)
    assert np.max(np.abs(R.T @ R - np.eye(d_h))) <= 1e-12
    assert np.all(np.diff(sigma) <= 1e-12)
    full = orp.rotate_truncate(Qp, R, d_h) @ orp.rotate_truncate(Kp, R, d_h).T
    assert np.max(np.abs(full - Qp @ Kp.T)) <= 1e-11          # (Q_p R)(K_p R)^T = Q_p K_p^T
    # truncation = deleting the rightmost columns: the first k columns are unchanged
    assert np.array_equal(orp.rotate_truncate(Kp, R, 5), orp.rotate_truncate(Kp, R, d_h)[:, :5])


def test_full_rank_post_rope_attention_equals_standard_rope_attention():
    R, sigma, Qp, Kp, V, d_h = _post_rope_inputs(4)
    scale = 1 / math.sqrt(d_h)
    got = oa.latent_attn_prefill(orp.rotate_truncate(Qp, R, d_h), orp.rotate_truncate(Kp, R, d_h), V, scale, True)
    t = lambda a: torch.from_numpy(a)[None, None]
    ref = F.scaled_dot_product_attention(t(Qp), t(Kp), t(V), is_causal=True)[0, 0].numpy()
    assert np.max(np.abs(got - ref)) <= 1e-11


def test_truncation_error_is_the_dropped_singular_mass():
    # on the calibration matrix itself: ||X - X R_k R_k^T||_F^2 = sum_{i >= k} sigma_i^2
    g = gen.make_rng(5)
    d, d_h, n = 40, 16, 200
    Wq, Wk = g.standard_normal((d, d_h)), gen.planted_weight(d, d_h, 3.0, g).W
    cos, sin = orp.rope_tables(n, d_h)
    x = gen.hidden_states(n, d, g)
    Qp, Kp = orp.rope(x @ Wq, np.arange(n), cos, sin), orp.rope(x @ Wk, np.arange(n), cos, sin)
    R, sigma = orp.common_rotation(Qp, Kp)
    X = np.concatenate([Qp, Kp])
    for k in (4, 9, 16):
        err = np.linalg.norm(X - orp.rotate_truncate(X, R, k) @ R[:, :k].T, "fro") ** 2
        assert abs(err - np.sum(sigma[k:] ** 2)) <= 1e-9 * np.sum(sigma ** 2)
    # compressed scores approach the exact ones as k grows
    exact = Qp @ Kp.T
    errs = [np.max(np.abs(orp.rotate_truncate(Qp, R, k) @ orp.rotate_truncate(Kp, R, k).T - exact)) for k in (4, 8, 12, 16)]
    assert errs[0] > errs[1] > errs[2] > errs[3] and errs[3] <= 1e-10
