"""Pins for the grouped-query oracle (Section 5.1, GQA paragraph): at full rank it is the library
GQA attention of PyTorch; g = 1 is the multi-head oracle; expanding the key/value heads g times
gives the multi-head result; the offsets are a partition; the group rotation keeps every query
head's scores."""
import math

import numpy as np
import torch
import torch.nn.functional as F

from oracle import attention as oa
from oracle import gqa as og
from oracle import factors as of
from oracle import rope as orp
from workloads import generators as gen


def _model(seed, H_kv=2, g=3, d=48, d_h=16, S=37):
    rng = gen.make_rng(seed)
    Hq = H_kv * g
    Wq = rng.standard_normal((d, Hq * d_h)) / math.sqrt(d)
    Wk = [gen.planted_weight(d, d_h, 4.0, rng).W for _ in range(H_kv)]
    Wv = [gen.planted_weight(d, d_h, 4.0, rng).W for _ in range(H_kv)]
    Wo = rng.standard_normal((Hq * d_h, d)) / math.sqrt(Hq * d_h)
    x = gen.hidden_states(S, d, rng)
    return rng, Hq, Wq, Wk, Wv, Wo, x


def test_full_rank_gqa_chain_equals_torch_gqa_attention():
    H_kv, g, d, d_h, S = 2, 3, 48, 16, 37
    rng, Hq, Wq, Wk, Wv, Wo, x = _model(1, H_kv, g, d, d_h, S)
    fk = [of.truncated_svd_factors(W, d_h) for W in Wk]
    fv = [of.truncated_svd_factors(W, d_h) for W in Wv]
    K_lat = oa.project_latent_kv(x, [f[0] for f in fk])
    V_lat = oa.project_latent_kv(x, [f[0] for f in fv])
    q = (x @ Wq).reshape(S, Hq, d_h)
    scale = 1 / math.sqrt(d_h)
    Q_lat = og.absorb_query(q, [f[1] for f in fk], g)
    O_lat = og.latent_attn_prefill(Q_lat, K_lat, V_lat, scale, True, g)
    M = og.fold_output([f[1] for f in fv], Wo, d_h, g)
    y = oa.apply_output(O_lat, M)
    # library route: uncompressed K, V with H_kv heads, queries with H_q heads
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(np.stack([x @ W for W in Wk]))[None]
    tv = torch.from_numpy(np.stack([x @ W for W in Wv]))[None]
    ref = F.scaled_dot_product_attention(tq, tk, tv, is_causal=True, enable_gqa=True)[0]   # [Hq, S, d_h]
    y_ref = ref.permute(1, 0, 2).reshape(S, Hq * d_h).numpy() @ Wo
    assert np.max(np.abs(y - y_ref)) <= 1e-10
    # decode = last row
    o_dec = og.latent_attn_decode([Q[-1] for Q in Q_lat], K_lat, V_lat, scale, g)
    for hq in range(Hq):
        assert np.max(np.abs(o_dec[hq] - O_lat[hq][-1])) <= 1e-12


def test_group_size_one_is_the_multi_head_oracle_and_expansion_equivalence():
    H_kv, g, d, d_h, S = 3, 2, 40, 16, 21
    rng, Hq, Wq, Wk, Wv, Wo, x = _model(2, H_kv, g, d, d_h, S)
    rk, rv = [8, 16, 4], [16, 4, 8]
    fk = [of.truncated_svd_factors(W, r) for W, r in zip(Wk, rk)]
    fv = [of.truncated_svd_factors(W, r) for W, r in zip(Wv, rv)]
    K_lat = oa.project_latent_kv(x, [f[0] for f in fk])
    V_lat = oa.project_latent_kv(x, [f[0] for f in fv])
    q = (x @ Wq).reshape(S, Hq, d_h)
    Q_lat = og.absorb_query(q, [f[1] for f in fk], g)
    got = og.latent_attn_prefill(Q_lat, K_lat, V_lat, 0.3, True, g)
    # expanding every key/value head g times turns GQA into plain multi-head attention
    Bk_x = [fk[h // g][1] for h in range(Hq)]
    K_x = [K_lat[h // g] for h in range(Hq)]
    V_x = [V_lat[h // g] for h in range(Hq)]
    Q_x = oa.absorb_query(q, Bk_x)
    for hq in range(Hq):
        ref = oa.latent_attn_prefill(Q_x[hq], K_x[hq], V_x[hq], 0.3, True)
        assert np.array_equal(got[hq], ref)
    # g = 1 is the multi-head oracle itself
    one = og.latent_attn_prefill(Q_x, K_x, V_x, 0.3, True, 1)
    for hq in range(Hq):
        assert np.array_equal(one[hq], got[hq])
    # a query head really uses ITS key/value head: query head g (first of group 1) against head 0 differs
    wrong = oa.latent_attn_prefill(Q_lat[g][:, :rk[0]], K_lat[0], V_lat[0], 0.3, True)
    right = oa.latent_attn_prefill(Q_lat[g], K_lat[1], V_lat[1], 0.3, True)
    assert np.array_equal(right, got[g]) and wrong.shape != right.shape


def test_query_offsets_partition_the_columns():
    rk = [16, 48, 32]
    for g in (1, 2, 4):
        off = og.query_offsets(rk, g)
        assert len(off) == len(rk) * g + 1 and off[0] == 0 and off[-1] == g * sum(rk)
        covered = np.zeros(off[-1], dtype=int)
        for hq in range(len(rk) * g):
            w = rk[og.kv_head_of(hq, g)]
            assert off[hq + 1] - off[hq] == w
            covered[off[hq]:off[hq] + w] += 1
        assert np.all(covered == 1)
    assert og.query_offsets([16, 32], 2) == [0, 16, 32, 64, 96]
    assert [og.kv_head_of(h, 4) for h in range(8)] == [0, 0, 0, 0, 1, 1, 1, 1]


def test_group_rotation_keeps_scores_of_every_query_head():
    rng = gen.make_rng(4)
    d, d_h, n, g = 40, 16, 120, 3
    cos, sin = orp.rope_tables(n, d_h)
    x = gen.hidden_states(n, d, rng)
    pos = np.arange(n)
    Wk = gen.planted_weight(d, d_h, 3.0, rng).W
    Qp = [orp.rope(x @ (rng.standard_normal((d, d_h)) / math.sqrt(d)), pos, cos, sin) for _ in range(g)]
    Kp = orp.rope(x @ Wk, pos, cos, sin)
    R, sigma = og.common_rotation(Qp, Kp)
    assert np.max(np.abs(R.T @ R - np.eye(d_h))) <= 1e-12 and np.all(np.diff(sigma) <= 1e-12)
    for j in range(g):
        assert np.max(np.abs((Qp[j] @ R) @ (Kp @ R).T - Qp[j] @ Kp.T)) <= 1e-10
    # the stacked matrix has (g + 1) n rows; dropped mass = sum of the dropped sigma^2
    X = np.concatenate(Qp + [Kp])
    k = 9
    err = np.linalg.norm(X - (X @ R[:, :k]) @ R[:, :k].T, "fro") ** 2
    assert abs(err - np.sum(sigma[k:] ** 2)) <= 1e-9 * np.sum(sigma ** 2)
    # g = 1 reduces to the single-head rotation (same subspace ordering: equal singular values)
    R1, s1 = og.common_rotation(Qp[:1], Kp)
    R0, s0 = orp.common_rotation(Qp[0], Kp)
    assert np.allclose(s1, s0, rtol=1e-12)
