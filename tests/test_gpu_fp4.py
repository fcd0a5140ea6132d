"""GPU parity of the E2M1 latent cache (FDC_FP4 layouts: 4-bit float codes, two per byte) through the C ABI.

Projection: products chosen to be exact hit every grid value, every tie and the saturating range, so the
stored codes must be the oracle's, nibble for nibble; random products are compared like the E4M3 ones (the
code decision is taken on the fp32 value on both sides, the library's fp32 sum is MFMA-ordered, so a value on
a rounding boundary may land on the neighbouring code: rare and exactly one grid step apart). Decode and
prefill attention: the oracle works on the decoded values of the very bytes the kernel reads.
"""
import math
import sys

import numpy as np
import pytest
import torch

import paper_2408_04107_amd as fdc
from oracle import attention as oa
from oracle import fp4
from tests.gpu_util import assert_close, workspace_for
from workloads import generators as gen

pytestmark = pytest.mark.gpu
BF = torch.bfloat16


def say(msg):
    print(f"[fp4-parity] {msg}", flush=True)
    sys.stdout.flush()


def grid_index(codes):
    """Position of a code on the ordered grid of values (sign-magnitude -> signed integer; +0 and -0 coincide)."""
    c = np.asarray(codes).astype(np.int64)
    return np.where(c & 8, -(c & 7), c & 7)


def unit_rows(buf, R, S, off_h, r, b, positions):
    """Unpacked codes [len(positions), r] of unit (b, h) at the given token positions; buf holds bytes."""
    out = []
    for p in positions:
        e0 = (b * S) * R + S * off_h + p * r          # element offset, even
        out.append(fp4.unpack_rows(buf[e0 // 2:(e0 + r) // 2]))
    return np.stack(out)


@pytest.mark.parametrize("T", [3, 16, 40, 300])
def test_exact_products_store_exactly_the_oracles_codes(T):
    """x rows are one-hot times a value, A rows one-hot: every latent element is one exact product, so grid
    values, ties (0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5), their neighbours and values beyond +-6 are all
    decided without rounding noise. Checks rounding, saturation and which nibble a column lands in."""
    rk, rv = [16, 48], [32, 16]
    H, d, B, S = 2, 128, 2, 320
    lay = fdc.Layout(1, H, d, 64, [rk], [rv], B, S, fdc.FDC_FP4)
    t = lay.tables()
    RK, RV = sum(rk), sum(rv)
    assert int(t["k_bytes"][0]) == B * S * RK // 2 and int(t["v_bytes"][0]) == B * S * RV // 2   # half a byte per element
    kc = torch.zeros(B * S * RK // 2, dtype=torch.uint8, device="cuda:0")
    vc = torch.zeros(B * S * RV // 2, dtype=torch.uint8, device="cuda:0")
    # latent column n of every token = value[token] * weight[n]: x[t, n] = value, A[n, n] = weight (d >= RK + RV)
    ties = [0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0]
    vals = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0, 7.0, 100.0, 2.0 ** -10] + ties + \
        [float(gen.round_to_bf16(np.array([m * f]))[0]) for m in ties for f in (1 - 1 / 128, 1 + 1 / 128)]   # bf16 neighbours
    g = gen.make_rng(T)
    v_tok = np.array([vals[i % len(vals)] * (-1.0) ** (i // len(vals)) for i in range(T)])
    w_col = np.where(g.random(RK + RV) < 0.5, 1.0, -1.0) * np.where(g.random(RK + RV) < 0.3, 0.5, 1.0)
    x = np.zeros((T, d))
    x[:, :RK + RV] = v_tok[:, None]
    A = np.zeros((RK + RV, d))
    A[np.arange(RK + RV), np.arange(RK + RV)] = w_col
    assert np.array_equal(gen.round_to_bf16(x), x) and np.array_equal(gen.round_to_bf16(A), A)
    slots = g.permutation(B * S)[:T]
    tb = torch.tensor(slots // S, dtype=torch.int32, device="cuda:0")
    tp = torch.tensor(slots % S, dtype=torch.int32, device="cuda:0")
    fdc.fdc_project_latent_kv(lay, 0, torch.from_numpy(x).to(BF).cuda(), tb, tp, torch.from_numpy(A).to(BF).cuda(), kc, vc)
    torch.cuda.synchronize()
    kb, vb = kc.cpu().numpy(), vc.cpu().numpy()
    for buf, ranks, R, col0 in ((kb, rk, RK, 0), (vb, rv, RV, RK)):
        off = np.concatenate([[0], np.cumsum(ranks)])
        for h in range(H):
            want = fp4.quantise_latent(v_tok[:, None] * w_col[None, col0 + off[h]:col0 + off[h + 1]])
            for i, (b, p) in enumerate(zip(slots // S, slots % S)):
                got = unit_rows(buf, R, S, off[h], ranks[h], b, [p])[0]
                # the sign of a zero is not part of the contract: compare values
                assert np.array_equal(fp4.e2m1_decode(got), fp4.e2m1_decode(want[i])), (h, i, v_tok[i], got, want[i])
    assert kb.any() and vb.any()


@pytest.mark.parametrize("T", [1, 16, 40, 300])
def test_projection_stores_the_oracles_codes(T):
    rk, rv = [16, 48, 128, 64], [64, 16, 128, 32]
    H, d, B, S = len(rk), 512, 3, 200
    say(f"project T={T}")
    lay = fdc.Layout(1, H, d, 128, [rk], [rv], B, S, fdc.FDC_FP4)
    RK, RV = sum(rk), sum(rv)
    kc = torch.zeros(B * S * RK // 2, dtype=torch.uint8, device="cuda:0")
    vc = torch.zeros(B * S * RV // 2, dtype=torch.uint8, device="cuda:0")
    g = gen.make_rng(700 + T)
    x = torch.from_numpy(gen.round_to_bf16(gen.hidden_states(T, d, g))).to(BF).cuda()
    # weights scaled so that the rows spread over the whole E2M1 range, some beyond 6 (saturation)
    A = torch.from_numpy(gen.round_to_bf16(g.standard_normal((RK + RV, d)) * (3.0 / math.sqrt(d)))).to(BF).cuda()
    slots = g.permutation(B * S)[:T]
    tb = torch.tensor(slots // S, dtype=torch.int32, device="cuda:0")
    tp = torch.tensor(slots % S, dtype=torch.int32, device="cuda:0")
    fdc.fdc_project_latent_kv(lay, 0, x, tb, tp, A, kc, vc)
    torch.cuda.synchronize()
    x64, A64 = x.to(torch.float64).cpu().numpy(), A.to(torch.float64).cpu().numpy()
    kb, vb = kc.cpu().numpy(), vc.cpu().numpy()
    n_total = n_off = sat = 0
    for buf, ranks, R, row0 in ((kb, rk, RK, 0), (vb, rv, RV, RK)):
        off = np.concatenate([[0], np.cumsum(ranks)])
        for h in range(H):
            want = fp4.quantise_latent(x64 @ A64[row0 + off[h]:row0 + off[h + 1]].T)       # [T, r] codes
            got = np.concatenate([unit_rows(buf, R, S, off[h], ranks[h], b, [p]) for b, p in zip(slots // S, slots % S)])
            diff = np.abs(grid_index(got) - grid_index(want))
            assert diff.max() <= 1, (h, int(diff.max()))
            n_total += diff.size
            n_off += int((diff == 1).sum())
            sat += int(((want & 7) == 7).sum())
    assert n_off <= max(2, n_total // 500), (n_off, n_total)
    assert sat > 0
    written = np.zeros(B * S, bool)
    written[slots] = True
    assert kb.any() and not kb.reshape(B, -1)[~written.reshape(B, S).any(axis=1)].any()      # untouched sequences stay zero
    say(f"  {n_total} codes, {n_off} one grid step apart, {sat} saturated")


def build_cache(rk, rv, seq, rng, k_gain=2.0, v_gain=2.5):
    """Packed code buffers of a dense layout filled with quantised latent rows, plus the decoded rows per unit."""
    H, B, S = len(rk), len(seq), max(max(seq), 1)
    RK, RV = sum(rk), sum(rv)
    kcodes = np.zeros(B * S * RK, dtype=np.uint8)
    vcodes = np.zeros(B * S * RV, dtype=np.uint8)
    ko, vo = np.concatenate([[0], np.cumsum(rk)]), np.concatenate([[0], np.cumsum(rv)])
    Ks, Vs = {}, {}
    for b, n in enumerate(seq):
        for h in range(H):
            kq = fp4.quantise_latent(gen.direct_latent(n, rk[h], 32.0, rng) * k_gain)
            vq = fp4.quantise_latent(gen.direct_latent(n, rv[h], 32.0, rng) * v_gain)
            Ks[b, h], Vs[b, h] = fp4.e2m1_decode(kq), fp4.e2m1_decode(vq)
            k0, v0 = b * S * RK + S * ko[h], b * S * RV + S * vo[h]
            kcodes[k0:k0 + n * rk[h]] = kq.ravel()
            vcodes[v0:v0 + n * rv[h]] = vq.ravel()
    pack = lambda c: torch.from_numpy(fp4.pack_rows(c.reshape(-1, 2)).ravel()).cuda()
    return pack(kcodes), pack(vcodes), Ks, Vs


@pytest.mark.parametrize("W,granule,min_split", [(1, 64, 1), (37, 64, 1), (700, 32, 2), (4096, 64, 1)])
def test_decode_attention_on_e2m1_codes(W, granule, min_split):
    """Multi-head decode over E2M1 codes, every rank class on both sides, through the three decode entry points."""
    rk = [16, 32, 48, 64, 80, 96, 112, 128]
    rv = [128, 16, 112, 32, 96, 48, 64, 80]
    H, d_h = len(rk), 128
    seq = [0, 1, 63, 257, 1500, 700]
    B, S = len(seq), max(seq)
    say(f"decode W={W} granule={granule} min_split={min_split}")
    lay = fdc.Layout(1, H, 256, d_h, [rk], [rv], B, S, fdc.FDC_FP4)
    RK, RV = sum(rk), sum(rv)
    rng = gen.make_rng(19 * W + granule)
    kc, vc, Ks, Vs = build_cache(rk, rv, seq, rng)
    q_lat = torch.from_numpy((rng.standard_normal((B, RK)) * 0.7).astype(np.float32)).cuda()
    o_lat = torch.full((B, RV), float("nan"), dtype=torch.float32, device="cuda:0")
    pp = fdc.fdc_plan_params_default()
    pp.n_workers, pp.granule, pp.min_split = W, granule, min_split
    plan = fdc.fdc_plan_decode(lay, 0, seq, pp)
    ws = workspace_for(plan)
    scale = 1 / math.sqrt(d_h)
    for _ in range(2):      # twice on the same workspace
        fdc.fdc_latent_attn_decode(lay, plan, q_lat, kc, vc, scale, o_lat, ws)
    torch.cuda.synchronize()
    out = o_lat.cpu().numpy().astype(np.float64)
    q64 = q_lat.to(torch.float64).cpu().numpy()
    ko, vo = np.concatenate([[0], np.cumsum(rk)]), np.concatenate([[0], np.cumsum(rv)])
    got_all, ref_all = [], []
    for b, n in enumerate(seq):
        for h in range(H):
            got = out[b, vo[h]:vo[h + 1]]
            if n == 0:
                assert not got.any()
                continue
            ref = oa.latent_attn_decode(q64[b, ko[h]:ko[h + 1]], Ks[b, h], Vs[b, h], scale)
            assert_close(got, ref, f"b={b} h={h} n={n}", rel_l2_tol=2e-4)     # fp32 sums of exactly decoded values
            got_all.append(got), ref_all.append(ref)
    ma, rl = assert_close(np.concatenate(got_all), np.concatenate(ref_all), "all", rel_l2_tol=5e-5)
    say(f"  tiles={plan.export()['n_items']} max_abs={ma:.2e} rel_l2={rl:.2e}")
    # the entry point on the built-in workspace and the one for actual lengths give the same bits
    o2 = torch.full_like(o_lat, float("nan"))
    fdc.fdc_latent_attn_decode_static(lay, plan, q_lat, kc, vc, scale, o2)
    o3 = torch.full_like(o_lat, float("nan"))
    lens = torch.tensor(seq, dtype=torch.int32, device="cuda:0")
    fdc.fdc_latent_attn_decode_at(lay, plan, lens, q_lat, kc, vc, scale, o3, ws)
    torch.cuda.synchronize()
    assert torch.equal(o2, o_lat) and torch.equal(o3, o_lat)


@pytest.mark.parametrize("g,W", [(2, 5), (4, 300)])
def test_grouped_decode_over_e2m1_codes(g, W):
    """Grouped queries over an E2M1 cache: the multi-head kernel runs once per query head of the group, each pass
    with that head's q', o' and partial slots; split units, unsplit units, an empty sequence."""
    from oracle import gqa as og
    rk, rv = [16, 64, 128, 48], [32, 16, 80, 128]
    H, d_h = len(rk), 128
    seq = [100, 0, 1300, 64]
    B, S = len(seq), max(seq)
    say(f"grouped decode g={g} W={W}")
    lay = fdc.Layout(1, H, 256, d_h, [rk], [rv], B, S, fdc.FDC_FP4, q_per_kv=g)
    RK, RV = sum(rk), sum(rv)
    rng = gen.make_rng(31 * g + W)
    kc, vc, Ks, Vs = build_cache(rk, rv, seq, rng)
    q_lat = torch.from_numpy((rng.standard_normal((B, g * RK)) * 0.7).astype(np.float32)).cuda()
    o_lat = torch.full((B, g * RV), float("nan"), dtype=torch.float32, device="cuda:0")
    pp = fdc.fdc_plan_params_default()
    pp.n_workers = W
    plan = fdc.fdc_plan_decode(lay, 0, seq, pp)
    ws = workspace_for(plan)
    scale = 1 / math.sqrt(d_h)
    fdc.fdc_latent_attn_decode(lay, plan, q_lat, kc, vc, scale, o_lat, ws)
    torch.cuda.synchronize()
    out, q64 = o_lat.cpu().numpy().astype(np.float64), q_lat.cpu().numpy().astype(np.float64)
    qo, oo = og.query_offsets(rk, g), og.query_offsets(rv, g)
    for b, n in enumerate(seq):
        for hq in range(H * g):
            h = hq // g
            got = out[b, oo[hq]:oo[hq + 1]]
            if n == 0:
                assert not got.any()
                continue
            ref = oa.latent_attn_decode(q64[b, qo[hq]:qo[hq + 1]], Ks[b, h], Vs[b, h], scale)
            assert_close(got, ref, f"b={b} hq={hq} n={n}", rel_l2_tol=2e-4)
    o2 = torch.full_like(o_lat, float("nan"))
    fdc.fdc_latent_attn_decode_static(lay, plan, q_lat, kc, vc, scale, o2)
    torch.cuda.synchronize()
    assert torch.equal(o2, o_lat)
    say(f"  tiles={plan.export()['n_items']}")


@pytest.mark.parametrize("g", [1, 2])
@pytest.mark.parametrize("W,br,chunked", [(5, 64, False), (40, 256, True), (256, 512, False)])
def test_prefill_attention_on_e2m1_codes(W, br, chunked, g):
    """Causal prefill over E2M1 codes (whole and chunked prompts): the kernel widens the codes to bf16 while
    staging, which is exact, so the bf16 tolerance applies."""
    rk, rv = [16, 48, 128, 64, 32], [64, 16, 128, 32, 48]
    H, d_h = len(rk), 128
    kv = [1, 129, 700, 1300, 333]
    ql = [1, 129, 300, 1300, 0] if chunked else [1, 129, 700, 1300, 333]
    say(f"prefill W={W} br={br} chunked={chunked} g={g}")
    rng = gen.make_rng(7 * W + br)
    RK, RV = sum(rk), sum(rv)
    lay = fdc.Layout(1, H, 256, d_h, [rk], [rv], len(kv), max(kv), fdc.FDC_FP4, q_per_kv=g)
    kc, vc, Ks, Vs = build_cache(rk, rv, kv, rng)
    T = int(np.sum(ql))
    q_lat = torch.from_numpy(gen.round_to_bf16(rng.standard_normal((T, g * RK)) * 0.5)).to(BF).cuda()
    o_lat = torch.full((T, g * RV), float("nan"), dtype=BF, device="cuda:0")
    pp = fdc.fdc_plan_params_default()
    pp.n_workers, pp.br_base, pp.br_cap, pp.cost_mode = W, br, br, 1
    plan = fdc.fdc_plan_prefill(lay, 0, ql, kv, pp)
    ws = workspace_for(plan)
    scale = 1 / math.sqrt(d_h)
    fdc.fdc_latent_attn_prefill(lay, plan, q_lat, kc, vc, scale, True, o_lat, ws)
    torch.cuda.synchronize()
    out, q64 = o_lat.to(torch.float64).cpu().numpy(), q_lat.to(torch.float64).cpu().numpy()
    assert np.all(np.isfinite(out))
    from oracle import gqa as og
    ko, vo = og.query_offsets(rk, g), og.query_offsets(rv, g)
    row0 = np.concatenate([[0], np.cumsum(ql)])
    got_all, ref_all = [], []
    for b in range(len(kv)):
        if ql[b] == 0:
            continue
        for hq in range(H * g):
            h = hq // g
            ref = oa.latent_attn_prefill(q64[row0[b]:row0[b + 1], ko[hq]:ko[hq + 1]], Ks[b, h], Vs[b, h], scale, True)
            got = out[row0[b]:row0[b + 1], vo[hq]:vo[hq + 1]]
            assert_close(got, ref, f"b={b} hq={hq}", max_abs_tol=3e-2)     # values reach +-6
            got_all.append(got.ravel()), ref_all.append(ref.ravel())
    ma, rl = assert_close(np.concatenate(got_all), np.concatenate(ref_all), "all", max_abs_tol=3e-2)
    say(f"  tasks={plan.export()['n_items']} max_abs={ma:.2e} rel_l2={rl:.2e}")


def test_post_rope_keys_and_one_launch_prologue_store_e2m1_codes():
    """fdc_rope_compress_keys on an FDC_FP4 layout: every decoded element lies within half a grid step (plus the
    bf16-operand error of the rotated key) of the oracle's value. fdc_project_and_absorb_query writes the very
    bytes of fdc_project_latent_kv and the queries of fdc_absorb_query."""
    from oracle import rope as orp
    H, d_h, rk, T, n_pos = 4, 64, [16, 64, 32, 48], 130, 256
    g = gen.make_rng(43)
    B, S = 2, 200
    lay = fdc.Layout(1, H, 128, d_h, [rk], [rk], B, S, fdc.FDC_FP4)
    RK = sum(rk)
    kc = torch.zeros(B * S * RK // 2, dtype=torch.uint8, device="cuda:0")
    R_t = np.concatenate([np.linalg.qr(g.standard_normal((d_h, d_h)))[0][:, :r].T for r in rk], axis=0)   # [RK, d_h]
    cos, sin = orp.rope_tables(n_pos, d_h)
    k = torch.from_numpy(gen.round_to_bf16(g.standard_normal((T, H, d_h)) * 2.0)).to(BF).cuda()
    R_d = torch.from_numpy(gen.round_to_bf16(R_t)).to(BF).cuda()
    slots = g.permutation(B * S)[:T]
    tb, tp = (slots // S).astype(np.int32), (slots % S).astype(np.int32)
    fdc.fdc_rope_compress_keys(lay, 0, k, torch.from_numpy(tb).cuda(), torch.from_numpy(tp).cuda(),
                               torch.from_numpy(np.ascontiguousarray(cos, dtype=np.float32)).cuda(),
                               torch.from_numpy(np.ascontiguousarray(sin, dtype=np.float32)).cuda(), R_d, kc)
    torch.cuda.synchronize()
    cos32, sin32 = cos.astype(np.float32).astype(np.float64), sin.astype(np.float32).astype(np.float64)
    off = np.concatenate([[0], np.cumsum(rk)])
    R64, k64, kb = R_d.to(torch.float64).cpu().numpy(), k.to(torch.float64).cpu().numpy(), kc.cpu().numpy()
    n_total = n_same = 0
    for h in range(H):
        want_rows = orp.rope(k64[:, h, :], tp, cos32, sin32) @ R64[off[h]:off[h + 1]].T
        want = fp4.quantise_latent(want_rows)
        got = np.concatenate([unit_rows(kb, RK, S, off[h], rk[h], b, [p]) for b, p in zip(tb, tp)])
        clipped = np.clip(want_rows, -6.0, 6.0)
        # half the largest grid step around the value (1 between 4 and 6, 0.5 between 2 and 4, 0.25 below) + operand error
        half_step = np.where(np.abs(clipped) >= 4, 1.0, np.where(np.abs(clipped) >= 2, 0.5, 0.25))
        err = np.abs(fp4.e2m1_decode(got) - clipped)
        assert np.all(err <= half_step + 0.03), (h, float(err.max()))
        n_total += got.size
        n_same += int((grid_index(got) == grid_index(want)).sum())
    assert kb.any() and n_same >= 0.97 * n_total, (n_same, n_total)
    say(f"  rope keys: {n_total} codes, {n_same} equal to the oracle's")

    rk2, rv2 = [16, 48, 128, 64], [64, 16, 128, 32]
    H2, d, S2, T2 = 4, 512, 64, 12
    lay4 = fdc.Layout(1, H2, d, 128, [rk2], [rv2], 2, S2, fdc.FDC_FP4)
    RK2, RV2 = sum(rk2), sum(rv2)
    x = torch.from_numpy(gen.round_to_bf16(gen.hidden_states(T2, d, g))).to(BF).cuda()
    A = torch.from_numpy(gen.round_to_bf16(g.standard_normal((RK2 + RV2, d)) * (2.0 / math.sqrt(d)))).to(BF).cuda()
    q = torch.from_numpy(gen.round_to_bf16(g.standard_normal((T2, H2, 128)))).to(BF).cuda()
    Bk = torch.from_numpy(gen.round_to_bf16(g.standard_normal((RK2, 128)) / math.sqrt(128))).to(BF).cuda()
    sl = g.permutation(2 * S2)[:T2]
    tb2 = torch.tensor(sl // S2, dtype=torch.int32, device="cuda:0")
    tp2 = torch.tensor(sl % S2, dtype=torch.int32, device="cuda:0")
    mk = lambda n: torch.zeros(n, dtype=torch.uint8, device="cuda:0")
    k1, v1, k2, v2 = mk(2 * S2 * RK2 // 2), mk(2 * S2 * RV2 // 2), mk(2 * S2 * RK2 // 2), mk(2 * S2 * RV2 // 2)
    q1 = torch.full((T2, RK2), float("nan"), dtype=torch.float32, device="cuda:0")
    q2 = torch.full_like(q1, float("nan"))
    fdc.fdc_project_latent_kv(lay4, 0, x, tb2, tp2, A, k1, v1)
    fdc.fdc_absorb_query(lay4, 0, q, Bk, q1, fdc.FDC_F32)
    fdc.fdc_project_and_absorb_query(lay4, 0, x, tb2, tp2, A, k2, v2, q, Bk, q2, fdc.FDC_F32)
    torch.cuda.synchronize()
    assert torch.equal(k1, k2) and torch.equal(v1, v2) and torch.equal(q1, q2) and bool(k1.any())


def build_paged_cache(rk, rv, seq, P, bt, n_pages, rng, k_gain=2.0, v_gain=2.5):
    """Packed code buffers of a paged layout (pages scattered by the block table) and the decoded rows per unit."""
    from oracle import layout as ol
    H, RK, RV = len(rk), sum(rk), sum(rv)
    kcodes = np.zeros(n_pages * P * RK, dtype=np.uint8)
    vcodes = np.zeros(n_pages * P * RV, dtype=np.uint8)
    Ks, Vs = {}, {}
    for b, n in enumerate(seq):
        for h in range(H):
            kq = fp4.quantise_latent(gen.direct_latent(n, rk[h], 32.0, rng) * k_gain)
            vq = fp4.quantise_latent(gen.direct_latent(n, rv[h], 32.0, rng) * v_gain)
            Ks[b, h], Vs[b, h] = fp4.e2m1_decode(kq), fp4.e2m1_decode(vq)
            for t in range(n):
                k0 = ol.paged_element_index(rk, P, bt[b], h, t, 0)
                v0 = ol.paged_element_index(rv, P, bt[b], h, t, 0)
                kcodes[k0:k0 + rk[h]], vcodes[v0:v0 + rv[h]] = kq[t], vq[t]
    pack = lambda c: torch.from_numpy(fp4.pack_rows(c.reshape(-1, 2)).ravel()).cuda()
    return pack(kcodes), pack(vcodes), Ks, Vs


@pytest.mark.parametrize("P,W,granule", [(128, 19, 64), (64, 300, 32)])
def test_paged_decode_on_e2m1_codes(P, W, granule):
    """Decode over a paged E2M1 cache: tiles are cut at page boundaries and every address is in half bytes."""
    from tests.test_gpu_paged import build_block_table
    rk, rv = [16, 64, 128, 48], [32, 128, 16, 80]
    H, d_h = len(rk), 128
    seq = [5, 300, 0, 129, 64]
    say(f"paged decode P={P} W={W} granule={granule}")
    rng = gen.make_rng(123 + P)
    bt, n_pages = build_block_table(seq, P, rng)
    lay = fdc.Layout(1, H, 256, d_h, [rk], [rv], n_pages, P, fdc.FDC_FP4)
    RK, RV = sum(rk), sum(rv)
    kc, vc, Ks, Vs = build_paged_cache(rk, rv, seq, P, bt, n_pages, rng)
    B = len(seq)
    q_lat = torch.from_numpy((rng.standard_normal((B, RK)) * 0.5).astype(np.float32)).cuda()
    o_lat = torch.full((B, RV), float("nan"), dtype=torch.float32, device="cuda:0")
    pp = fdc.fdc_plan_params_default()
    pp.n_workers, pp.granule = W, granule
    plan = fdc.fdc_plan_decode_paged(lay, 0, seq, bt, pp)
    ws = workspace_for(plan)
    scale = 1 / math.sqrt(d_h)
    fdc.fdc_latent_attn_decode(lay, plan, q_lat, kc, vc, scale, o_lat, ws)
    torch.cuda.synchronize()
    out, q64 = o_lat.cpu().numpy().astype(np.float64), q_lat.cpu().numpy().astype(np.float64)
    ko, vo = np.concatenate([[0], np.cumsum(rk)]), np.concatenate([[0], np.cumsum(rv)])
    for b, n in enumerate(seq):
        for h in range(H):
            got = out[b, vo[h]:vo[h + 1]]
            if n == 0:
                assert not got.any()
                continue
            ref = oa.latent_attn_decode(q64[b, ko[h]:ko[h + 1]], Ks[b, h], Vs[b, h], scale)
            assert_close(got, ref, f"paged b={b} h={h} n={n}", rel_l2_tol=2e-4)
    say(f"  tiles={plan.export()['n_items']}")


def test_paged_prefill_on_e2m1_codes():
    """Causal prefill over a paged E2M1 cache, chunked prompts, lengths that end inside a page."""
    from tests.test_gpu_paged import build_block_table
    rk, rv = [16, 48, 128, 64], [64, 16, 128, 32]
    H, d_h, P = len(rk), 128, 256
    kv = [1, 129, 700, 1300, 333]
    ql = [1, 129, 300, 1300, 0]
    rng = gen.make_rng(77)
    bt, n_pages = build_block_table(kv, P, rng)
    lay = fdc.Layout(1, H, 256, d_h, [rk], [rv], n_pages, P, fdc.FDC_FP4)
    RK, RV = sum(rk), sum(rv)
    kc, vc, Ks, Vs = build_paged_cache(rk, rv, kv, P, bt, n_pages, rng)
    T = int(np.sum(ql))
    q_lat = torch.from_numpy(gen.round_to_bf16(rng.standard_normal((T, RK)) * 0.5)).to(BF).cuda()
    o_lat = torch.full((T, RV), float("nan"), dtype=BF, device="cuda:0")
    pp = fdc.fdc_plan_params_default()
    pp.n_workers, pp.br_base, pp.br_cap, pp.cost_mode = 40, 256, 256, 1
    plan = fdc.fdc_plan_prefill_paged(lay, 0, ql, kv, bt, pp)
    ws = workspace_for(plan)
    scale = 1 / math.sqrt(d_h)
    fdc.fdc_latent_attn_prefill(lay, plan, q_lat, kc, vc, scale, True, o_lat, ws)
    torch.cuda.synchronize()
    out, q64 = o_lat.to(torch.float64).cpu().numpy(), q_lat.to(torch.float64).cpu().numpy()
    assert np.all(np.isfinite(out))
    ko, vo = np.concatenate([[0], np.cumsum(rk)]), np.concatenate([[0], np.cumsum(rv)])
    row0 = np.concatenate([[0], np.cumsum(ql)])
    got_all, ref_all = [], []
    for b in range(len(kv)):
        if ql[b] == 0:
            continue
        for h in range(H):
            ref = oa.latent_attn_prefill(q64[row0[b]:row0[b + 1], ko[h]:ko[h + 1]], Ks[b, h], Vs[b, h], scale, True)
            got = out[row0[b]:row0[b + 1], vo[h]:vo[h + 1]]
            assert_close(got, ref, f"b={b} h={h}", max_abs_tol=3e-2)     # values reach +-6
            got_all.append(got.ravel()), ref_all.append(ref.ravel())
    ma, rl = assert_close(np.concatenate(got_all), np.concatenate(ref_all), "all", max_abs_tol=3e-2)
    say(f"  paged prefill tasks={plan.export()['n_items']} max_abs={ma:.2e} rel_l2={rl:.2e}")


def test_decode_on_e2m1_codes_at_config3_size_sampled_units():
    """Layer 0 of the adaptive-rank decode config (batch 16, context 8192, 32 heads) with an E2M1 cache, in the
    launch configuration bench.py times (fdc_suggest_workers(4)): random bytes on the device (every byte is two
    valid codes), the oracle on ~60 sampled (sequence, head) units including the narrowest and the widest head."""
    wl = gen.CONFIGS["c3_adaptive_decode"]
    r = wl.ranks()[0].tolist()
    H, B, S, d_h = wl.n_heads, wl.batch, wl.context, wl.d_head
    W = fdc.fdc_suggest_workers(4)
    say(f"config 3 layer 0, E2M1: B={B} S={S} W={W}")
    lay = fdc.Layout(1, H, wl.d_model, d_h, [r], [r], B, S, fdc.FDC_FP4)
    R = sum(r)
    tg = torch.Generator(device="cuda:0").manual_seed(4)
    mk = lambda: torch.randint(0, 256, (B * S * R // 2,), generator=tg, device="cuda:0", dtype=torch.uint8)
    kc, vc = mk(), mk()
    rng = gen.make_rng(9)
    q_lat = torch.from_numpy((rng.standard_normal((B, R)) * 0.3).astype(np.float32)).cuda()     # codes reach +-6
    o_lat = torch.full((B, R), float("nan"), dtype=torch.float32, device="cuda:0")
    pp = fdc.fdc_plan_params_default()
    pp.n_workers = W
    plan = fdc.fdc_plan_decode(lay, 0, [S] * B, pp)
    ws = workspace_for(plan)
    scale = 1 / math.sqrt(d_h)
    fdc.fdc_latent_attn_decode(lay, plan, q_lat, kc, vc, scale, o_lat, ws)
    torch.cuda.synchronize()
    assert not torch.isnan(o_lat).any()
    units = {(int(b), int(h)) for b, h in zip(rng.integers(0, B, 60), rng.integers(0, H, 60))}
    units |= {(0, int(np.argmax(r))), (B - 1, int(np.argmin(r)))}
    off = np.concatenate([[0], np.cumsum(r)])
    out, q64 = o_lat.cpu().numpy().astype(np.float64), q_lat.cpu().numpy().astype(np.float64)
    for b, h in sorted(units):
        e0 = b * S * R + S * off[h]                       # element offset of the unit, even
        K = fp4.e2m1_decode(fp4.unpack_rows(kc[e0 // 2:(e0 + S * r[h]) // 2].cpu().numpy())).reshape(S, r[h])
        V = fp4.e2m1_decode(fp4.unpack_rows(vc[e0 // 2:(e0 + S * r[h]) // 2].cpu().numpy())).reshape(S, r[h])
        ref = oa.latent_attn_decode(q64[b, off[h]:off[h + 1]], K, V, scale)
        assert_close(out[b, off[h]:off[h + 1]], ref, f"b={b} h={h} r={r[h]}")
    say(f"  tiles={plan.export()['n_items']} units checked={len(units)}")


def test_prefill_reads_every_e2m1_code_exactly():
    """The prefill staging widens E2M1 codes to bf16 with the hardware's packed conversion. Row i is peaked on
    token i (weights exactly one-hot in bf16), so output row i is V' row i decoded: all sixteen codes, in every
    nibble position of a word, must come back as the format's values, bit for bit."""
    n, r = 16, 16
    rows = (np.arange(n)[:, None] + np.arange(r)[None, :]) % 16          # every code in every column
    lay = fdc.Layout(1, 1, 256, 128, [[r]], [[r]], 1, n, fdc.FDC_FP4)
    key_vals = np.zeros((n, r))
    key_vals[np.arange(n), np.arange(n)] = 6.0                            # K'[t] = 6 e_t (the largest code)
    kc = torch.from_numpy(fp4.pack_rows(fp4.quantise_latent(key_vals)).ravel()).cuda()
    vc = torch.from_numpy(fp4.pack_rows(rows.astype(np.uint8)).ravel()).cuda()
    q_lat = (torch.eye(n, r) * 512.0).to(BF).cuda()                       # score 3072 * scale on the diagonal
    o_lat = torch.full((n, r), float("nan"), dtype=BF, device="cuda:0")
    pp = fdc.fdc_plan_params_default()
    pp.n_workers, pp.br_base, pp.br_cap = 2, 64, 64
    plan = fdc.fdc_plan_prefill(lay, 0, [n], [n], pp)
    ws = workspace_for(plan)
    fdc.fdc_latent_attn_prefill(lay, plan, q_lat, kc, vc, 1 / math.sqrt(128), True, o_lat, ws)
    torch.cuda.synchronize()
    assert np.array_equal(o_lat.to(torch.float64).cpu().numpy(), fp4.e2m1_decode(rows))
