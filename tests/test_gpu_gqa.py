"""GPU parity of the grouped-query path (layouts with q_per_kv > 1) against the float64 oracle:
decode attention (MFMA tile kernel + split-K merge), query absorption, output fold / apply, the
post-RoPE query rotation and prefill attention. Inputs are the stored bits; q' enters the decode
tile kernel's matrix product rounded to bf16, so the oracle is fed the same rounded q'.
"""
import math
import sys

import numpy as np
import pytest
import torch

import paper_2408_04107_amd as fdc
from oracle import attention as oa
from oracle import gqa as og
from oracle import rope as orp
from tests.gpu_util import Cache, assert_close, workspace_for
from workloads import generators as gen

pytestmark = pytest.mark.gpu
BF = torch.bfloat16


def say(msg):
    print(f"[gqa-parity] {msg}", flush=True)
    sys.stdout.flush()


def dev(a, dt):
    return torch.from_numpy(np.ascontiguousarray(a)).to(dt).cuda().contiguous()


def f64(t):
    return t.to(torch.float64).cpu().numpy()


def run_gqa_decode(rk, rv, g, seq, W, min_split=1, split=1, granule=64, q_gain=1.0, seed=0, d_head=128,
                   decay=32.0, device_fill=False, check_units=None):
    H, B = len(rk), len(seq)
    S_max = max(max(seq), 1)
    lay = fdc.Layout(1, H, 256, d_head, [rk], [rv], B, S_max, fdc.FDC_BF16, q_per_kv=g)
    cache = Cache(lay)
    rng = gen.make_rng(seed)
    tg = torch.Generator(device="cuda:0").manual_seed(seed)
    for b in range(B):
        for h in range(H):
            if seq[b] == 0:
                continue
            if device_fill:
                for side, r in (("k", rk[h]), ("v", rv[h])):
                    sig = torch.exp(-torch.arange(r, device="cuda:0", dtype=torch.float32) / decay)
                    u = cache.unit(side, b, h)
                    u[:seq[b]] = (torch.randn(seq[b], r, generator=tg, device="cuda:0") * sig).to(u.dtype)
            else:
                cache.fill_unit("k", b, h, gen.direct_latent(seq[b], rk[h], decay, rng))
                cache.fill_unit("v", b, h, gen.direct_latent(seq[b], rv[h], decay, rng))
    q_lat = torch.from_numpy((rng.standard_normal((B, g * cache.RK)) * q_gain).astype(np.float32)).cuda()
    o_lat = torch.full((B, g * cache.RV), float("nan"), dtype=torch.float32, device="cuda:0")
    pp = fdc.fdc_plan_params_default()
    pp.n_workers, pp.min_split, pp.split, pp.granule = W, min_split, split, granule
    plan = fdc.fdc_plan_decode(lay, 0, seq, pp)
    ws = workspace_for(plan)
    scale = 1.0 / math.sqrt(d_head)
    fdc.fdc_latent_attn_decode(lay, plan, q_lat, cache.k, cache.v, scale, o_lat, ws)
    torch.cuda.synchronize()
    out = o_lat.cpu().numpy().astype(np.float64)
    q_used = f64(q_lat)      # the fp32 q' the caller passed (the kernel's bf16 operand rounding is inside the tolerance)
    qo, oo = og.query_offsets(rk, g), og.query_offsets(rv, g)
    units = check_units if check_units is not None else [(b, h) for b in range(B) for h in range(H)]
    got_all, ref_all = [], []
    for b, h in units:
        K, V = cache.unit_f64("k", b, h, seq[b]), cache.unit_f64("v", b, h, seq[b])
        for j in range(g):
            hq = h * g + j
            ref = oa.latent_attn_decode(q_used[b, qo[hq]:qo[hq + 1]], K, V, scale)
            got = out[b, oo[hq]:oo[hq + 1]]
            assert_close(got, ref, f"b={b} h={h} j={j} rk={rk[h]} rv={rv[h]} S={seq[b]}")
            got_all.append(got), ref_all.append(ref)
    if check_units is None:   # nothing outside the written columns
        assert np.all(np.isfinite(out))
    ma, rl = assert_close(np.concatenate(got_all), np.concatenate(ref_all), "all query heads")
    return ma, rl, plan.export()["n_items"], (lay, plan, cache, q_lat, o_lat, ws, scale)


MIX_K = [16, 32, 48, 64, 80, 96, 112, 128]
MIX_V = [128, 16, 48, 64, 32, 112, 96, 80]


@pytest.mark.parametrize("g", [2, 3, 4, 8, 16])
@pytest.mark.parametrize("W,min_split,split", [(1, 1, 1), (7, 1, 1), (64, 1, 1), (1000, 1, 1), (5, 3, 0), (64, 4, 1)])
def test_gqa_decode_mixed_ranks(g, W, min_split, split):
    say(f"decode mixed ranks g={g} W={W} min_split={min_split} split={split}")
    ma, rl, n, _ = run_gqa_decode(MIX_K, MIX_V, g, [777, 64, 1300], W, min_split=min_split, split=split, seed=W + g)
    say(f"  tiles={n} max_abs={ma:.2e} rel_l2={rl:.2e}")


def test_gqa_decode_ragged_and_empty_sequences():
    say("decode ragged and empty sequences")
    ma, rl, n, _ = run_gqa_decode(MIX_K, MIX_V, 4, [0, 1, 31, 32, 33, 63, 65, 127, 129, 300, 0], 33, granule=16, seed=3)
    say(f"  tiles={n} max_abs={ma:.2e} rel_l2={rl:.2e}")
    # all empty: zeros
    lay = fdc.Layout(1, 2, 256, 128, [[16, 64]], [[32, 16]], 2, 8, fdc.FDC_BF16, q_per_kv=4)
    cache = Cache(lay)
    pp = fdc.fdc_plan_params_default()
    pp.n_workers = 8
    plan = fdc.fdc_plan_decode(lay, 0, [0, 0], pp)
    ws = workspace_for(plan)
    q = torch.randn(2, 4 * cache.RK, device="cuda:0")
    o = torch.full((2, 4 * cache.RV), float("nan"), device="cuda:0")
    fdc.fdc_latent_attn_decode(lay, plan, q, cache.k, cache.v, 0.1, o, ws)
    torch.cuda.synchronize()
    assert torch.count_nonzero(o).item() == 0


def test_gqa_decode_peaked_queries_and_repeat_calls():
    say("decode peaked queries (q x 8), called twice on one workspace")
    ma, rl, n, st = run_gqa_decode(MIX_K, MIX_K, 4, [2048, 500], 256, q_gain=8.0, seed=5)
    say(f"  tiles={n} max_abs={ma:.2e} rel_l2={rl:.2e}")
    lay, plan, cache, q_lat, o_lat, ws, scale = st
    first = o_lat.clone()
    o_lat.fill_(float("nan"))
    fdc.fdc_latent_attn_decode(lay, plan, q_lat, cache.k, cache.v, scale, o_lat, ws)
    torch.cuda.synchronize()
    assert torch.equal(first, o_lat)   # deterministic


def test_gqa_decode_bench_shape_sampled_units():
    """8 key/value heads x 4 query heads, adaptive ranks, batch 16, context 8192, in the launch
    configuration bench.py uses for the grouped kernel; 24 sampled units, all their query heads."""
    say("decode at the grouped bench shape (sampled units)")
    g, H, B, S = 4, 8, 16, 8192
    r = [int(x) for x in gen.adaptive_ranks(1, H, 11)[0]]
    W = fdc.fdc_suggest_workers(2)
    rs = gen.make_rng(1)
    units = [(int(rs.integers(0, B)), int(rs.integers(0, H))) for _ in range(24)]
    ma, rl, n, _ = run_gqa_decode(r, r, g, [S] * B, W, seed=9, device_fill=True, check_units=units)
    say(f"  W={W} ranks={r} tiles={n} max_abs={ma:.2e} rel_l2={rl:.2e}")


def test_gqa_decode_on_an_fp32_layout_runs_one_pass_per_query_head():
    """fp32 caches have no grouped tile kernel: the multi-head kernel runs once per query head of the group.
    Plain fp32 arithmetic, so the result sits at fp32 rounding distance from the oracle."""
    rk, rv, g = [16, 32, 64], [32, 16, 48], 3
    seq = [700, 0, 65]
    H, d_h, B, S = len(rk), 64, len(seq), max(seq)
    lay = fdc.Layout(1, H, 64, d_h, [rk], [rv], B, S, fdc.FDC_F32, q_per_kv=g)
    cache = Cache(lay)
    rng = gen.make_rng(77)
    koff, voff = np.concatenate([[0], np.cumsum(rk)]), np.concatenate([[0], np.cumsum(rv)])
    kb, vb = np.zeros(cache.k.numel(), np.float32), np.zeros(cache.v.numel(), np.float32)
    Ks, Vs = {}, {}
    for b, n in enumerate(seq):
        for h in range(H):
            Ks[b, h] = gen.direct_latent(n, rk[h], 32.0, rng).astype(np.float32)
            Vs[b, h] = gen.direct_latent(n, rv[h], 32.0, rng).astype(np.float32)
            k0, v0 = b * S * cache.RK + S * koff[h], b * S * cache.RV + S * voff[h]
            kb[k0:k0 + n * rk[h]], vb[v0:v0 + n * rv[h]] = Ks[b, h].ravel(), Vs[b, h].ravel()
    cache.k.copy_(torch.from_numpy(kb)), cache.v.copy_(torch.from_numpy(vb))
    q = torch.from_numpy(rng.standard_normal((B, g * cache.RK)).astype(np.float32)).cuda()
    o = torch.full((B, g * cache.RV), float("nan"), device="cuda:0")
    pp = fdc.fdc_plan_params_default()
    pp.n_workers = 11
    plan = fdc.fdc_plan_decode(lay, 0, seq, pp)
    ws = workspace_for(plan)
    scale = 1 / math.sqrt(d_h)
    fdc.fdc_latent_attn_decode(lay, plan, q, cache.k, cache.v, scale, o, ws)
    torch.cuda.synchronize()
    out, q64 = o.cpu().numpy().astype(np.float64), q.cpu().numpy().astype(np.float64)
    qo, oo = og.query_offsets(rk, g), og.query_offsets(rv, g)
    for b, n in enumerate(seq):
        for hq in range(H * g):
            got = out[b, oo[hq]:oo[hq + 1]]
            if n == 0:
                assert not got.any()
                continue
            ref = oa.latent_attn_decode(q64[b, qo[hq]:qo[hq + 1]], Ks[b, hq // g].astype(np.float64),
                                        Vs[b, hq // g].astype(np.float64), scale)
            assert_close(got, ref, f"b={b} hq={hq}", rel_l2_tol=1e-5)


@pytest.mark.parametrize("g,T", [(2, 5), (4, 300), (8, 70)])
def test_gqa_absorb_query_fold_apply_and_rope(g, T):
    say(f"projections g={g} T={T}")
    rng = gen.make_rng(20 + g)
    H, d, d_h = 3, 256, 64
    rk, rv = [16, 64, 32], [48, 16, 64]
    Hq = H * g
    lay = fdc.Layout(1, H, d, d_h, [rk], [rv], 2, 64, fdc.FDC_BF16, q_per_kv=g)
    RK, RV = sum(rk), sum(rv)
    koff, voff = np.concatenate([[0], np.cumsum(rk)]), np.concatenate([[0], np.cumsum(rv)])
    Bk = dev(rng.standard_normal((RK, d_h)) / math.sqrt(d_h), BF)
    Bv = dev(rng.standard_normal((RV, d_h)) / math.sqrt(d_h), BF)
    q = dev(rng.standard_normal((T, Hq, d_h)), BF)
    Bk_heads = [f64(Bk)[koff[h]:koff[h + 1]] for h in range(H)]
    Bv_heads = [f64(Bv)[voff[h]:voff[h + 1]] for h in range(H)]
    # query absorption
    for dt, tdt in ((fdc.FDC_F32, torch.float32), (fdc.FDC_BF16, BF)):
        q_lat = torch.full((T, g * RK), float("nan"), dtype=tdt, device="cuda:0")
        fdc.fdc_absorb_query(lay, 0, q, Bk, q_lat, dt)
        torch.cuda.synchronize()
        ref = np.concatenate(og.absorb_query(f64(q), Bk_heads, g), axis=1)
        ma, rl = assert_close(f64(q_lat), ref, "q_lat")
        say(f"  absorb_query dtype={dt} max_abs={ma:.2e} rel_l2={rl:.2e}")
    # fold and apply
    Wo_t = dev(rng.standard_normal((d, Hq * d_h)) / math.sqrt(Hq * d_h), BF)
    Mt = torch.full((d, g * RV), float("nan"), dtype=BF, device="cuda:0")
    fdc.fdc_absorb_output(lay, 0, fdc.FDC_FOLD, Bv, Wo_t, Mt, None, fdc.FDC_BF16, 0, None, fdc.FDC_BF16)
    torch.cuda.synchronize()
    M_ref = og.fold_output(Bv_heads, f64(Wo_t).T, d_h, g)          # list of [rv, d]
    ma, rl = assert_close(f64(Mt), np.concatenate(M_ref, axis=0).T, "Mt")
    say(f"  fold max_abs={ma:.2e} rel_l2={rl:.2e}")
    for dt, tdt in ((fdc.FDC_F32, torch.float32), (fdc.FDC_BF16, BF)):
        o_lat = dev(rng.standard_normal((T, g * RV)), tdt)
        y = torch.full((T, d), float("nan"), dtype=BF, device="cuda:0")
        fdc.fdc_absorb_output(lay, 0, fdc.FDC_APPLY, None, None, Mt, o_lat, dt, T, y, fdc.FDC_BF16)
        torch.cuda.synchronize()
        ref = f64(o_lat) @ f64(Mt).T                               # o' as passed (fp32 o' becomes a bf16 operand inside the call)
        ma, rl = assert_close(f64(y), ref, "y")
        say(f"  apply dtype={dt} max_abs={ma:.2e} rel_l2={rl:.2e}")
    # post-RoPE query rotation with the rotation of the key/value head
    n_pos = 128
    cos, sin = orp.rope_tables(n_pos, d_h)
    cos32, sin32 = cos.astype(np.float32).astype(np.float64), sin.astype(np.float32).astype(np.float64)
    pos = rng.integers(0, n_pos, T).astype(np.int32)
    q_lat = torch.full((T, g * RK), float("nan"), dtype=torch.float32, device="cuda:0")
    fdc.fdc_rope_absorb_query(lay, 0, q, dev(pos, torch.int32), dev(cos, torch.float32), dev(sin, torch.float32),
                              Bk, q_lat, fdc.FDC_F32)
    torch.cuda.synchronize()
    ref = np.concatenate([orp.rope(f64(q)[:, hq, :], pos, cos32, sin32) @ Bk_heads[hq // g].T for hq in range(Hq)], axis=1)
    ma, rl = assert_close(f64(q_lat), ref, "rope q_lat")
    say(f"  rope_absorb_query max_abs={ma:.2e} rel_l2={rl:.2e}")


def test_gqa_prefill_attention():
    say("prefill attention g=4")
    rng = gen.make_rng(31)
    g, H, d_h = 4, 3, 128
    rk, rv = [16, 128, 48], [64, 32, 128]
    q_len, kv_len = [200, 77], [330, 77]
    B = len(q_len)
    lay = fdc.Layout(1, H, 256, d_h, [rk], [rv], B, max(kv_len), fdc.FDC_BF16, q_per_kv=g)
    cache = Cache(lay)
    for b in range(B):
        for h in range(H):
            cache.fill_unit("k", b, h, gen.direct_latent(kv_len[b], rk[h], 32.0, rng))
            cache.fill_unit("v", b, h, gen.direct_latent(kv_len[b], rv[h], 32.0, rng))
    T = sum(q_len)
    q_lat = dev(rng.standard_normal((T, g * cache.RK)) * 2.0, BF)
    o_lat = torch.full((T, g * cache.RV), float("nan"), dtype=BF, device="cuda:0")
    pp = fdc.fdc_plan_params_default()
    pp.n_workers, pp.cost_mode = 16, 1
    plan = fdc.fdc_plan_prefill(lay, 0, q_len, kv_len, pp)
    ws = workspace_for(plan)
    scale = 1 / math.sqrt(d_h)
    fdc.fdc_latent_attn_prefill(lay, plan, q_lat, cache.k, cache.v, scale, True, o_lat, ws)
    torch.cuda.synchronize()
    qo, oo = og.query_offsets(rk, g), og.query_offsets(rv, g)
    Q, O = f64(q_lat), f64(o_lat)
    assert np.all(np.isfinite(O))
    row0 = 0
    got_all, ref_all = [], []
    for b in range(B):
        for h in range(H):
            K, V = cache.unit_f64("k", b, h, kv_len[b]), cache.unit_f64("v", b, h, kv_len[b])
            for j in range(g):
                hq = h * g + j
                ref = oa.latent_attn_prefill(Q[row0:row0 + q_len[b], qo[hq]:qo[hq + 1]], K, V, scale, True)
                got = O[row0:row0 + q_len[b], oo[hq]:oo[hq + 1]]
                assert_close(got, ref, f"prefill b={b} hq={hq}")
                got_all.append(got.ravel()), ref_all.append(ref.ravel())
        row0 += q_len[b]
    ma, rl = assert_close(np.concatenate(got_all), np.concatenate(ref_all), "prefill all")
    say(f"  max_abs={ma:.2e} rel_l2={rl:.2e}")
