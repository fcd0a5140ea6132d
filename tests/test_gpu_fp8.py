"""GPU parity of the E4M3 latent cache (FDC_FP8 layouts) through the C ABI.

Projection: the codes the library stores are compared with the oracle's codes of the same products
(the code decision is taken on the fp32 value on both sides; the library's fp32 sum is MFMA-ordered,
so a value that sits on a rounding boundary may land on the neighbouring code: such elements must be
rare and exactly one code apart). Decode attention: the oracle works on the decoded values of the
very bytes the kernel reads, so the usual tolerance applies; the same for prefill attention.
"""
import math
import sys

import numpy as np
import pytest
import torch

import paper_2408_04107_amd as fdc
from oracle import attention as oa
from oracle import fp8
from tests.gpu_util import assert_close, workspace_for
from workloads import generators as gen

pytestmark = pytest.mark.gpu
BF = torch.bfloat16


def say(msg):
    print(f"[fp8-parity] {msg}", flush=True)
    sys.stdout.flush()


def magnitude_index(codes):
    """Position of a code on the ordered grid of values (sign-magnitude -> signed integer)."""
    c = np.asarray(codes).astype(np.int64)
    return np.where(c & 0x80, -(c & 0x7F), c & 0x7F)


@pytest.mark.parametrize("T", [1, 16, 40, 300])
def test_projection_stores_the_oracles_codes(T):
    rk, rv = [16, 48, 128, 64], [64, 16, 128, 32]
    H, d, B, S = len(rk), 512, 3, 200
    say(f"project T={T}")
    lay = fdc.Layout(1, H, d, 128, [rk], [rv], B, S, fdc.FDC_FP8)
    t = lay.tables()
    RK, RV = int(t["koff_r"][0, -1]), int(t["voff_r"][0, -1])
    assert int(t["k_bytes"][0]) == B * S * RK and int(t["v_bytes"][0]) == B * S * RV    # one byte per element
    kc = torch.zeros(B * S * RK, dtype=torch.uint8, device="cuda:0")
    vc = torch.zeros(B * S * RV, dtype=torch.uint8, device="cuda:0")
    g = gen.make_rng(900 + T)
    x = torch.from_numpy(gen.round_to_bf16(gen.hidden_states(T, d, g))).to(BF).cuda()
    # weights scaled so that the rows spread over the whole E4M3 range, some beyond 448 (saturation)
    A = torch.from_numpy(gen.round_to_bf16(g.standard_normal((RK + RV, d)) * (150.0 / math.sqrt(d)))).to(BF).cuda()
    slots = g.permutation(B * S)[:T]
    tb = torch.tensor(slots // S, dtype=torch.int32, device="cuda:0")
    tp = torch.tensor(slots % S, dtype=torch.int32, device="cuda:0")
    fdc.fdc_project_latent_kv(lay, 0, x, tb, tp, A, kc, vc)
    torch.cuda.synchronize()
    x64, A64 = x.to(torch.float64).cpu().numpy(), A.to(torch.float64).cpu().numpy()
    kb, vb = kc.cpu().numpy(), vc.cpu().numpy()
    n_total = n_off = 0
    sat = 0
    for side, buf, ranks, R, row0 in (("k", kb, rk, RK, 0), ("v", vb, rv, RV, RK)):
        off = np.concatenate([[0], np.cumsum(ranks)])
        for h in range(H):
            want = fp8.quantise_latent(x64 @ A64[row0 + off[h]:row0 + off[h + 1]].T)       # [T, r] codes
            got = np.stack([buf[(b * S) * R + S * off[h] + p * ranks[h]:(b * S) * R + S * off[h] + (p + 1) * ranks[h]]
                            for b, p in zip(slots // S, slots % S)])
            diff = np.abs(magnitude_index(got) - magnitude_index(want))
            assert diff.max() <= 1, (side, h, int(diff.max()))
            n_total += diff.size
            n_off += int((diff == 1).sum())
            sat += int(((want & 0x7F) == 0x7E).sum())
    assert n_off <= max(2, n_total // 500), (n_off, n_total)
    assert sat > 0                      # the saturating branch was exercised
    written = np.zeros(B * S, bool)
    written[slots] = True
    view = kb.reshape(B, -1)
    assert kb.any() and not view[~written.reshape(B, S).any(axis=1)].any()      # untouched sequences stay zero
    say(f"  {n_total} codes, {n_off} one code apart, {sat} saturated")


@pytest.mark.parametrize("g", [1, 4, 16])
@pytest.mark.parametrize("W,granule,min_split", [(1, 64, 1), (37, 64, 1), (700, 32, 2)])
def test_decode_attention_on_e4m3_codes(W, granule, min_split, g):
    """Multi-head (g = 1) and grouped-query decode over E4M3 codes, every rank class on both sides."""
    from oracle import gqa as og
    rk = [16, 32, 48, 64, 80, 96, 112, 128]
    rv = [128, 16, 112, 32, 96, 48, 64, 80]
    H, d_h = len(rk), 128
    seq = [0, 1, 63, 257, 1500, 700]
    B, S = len(seq), max(seq)
    say(f"decode g={g} W={W} granule={granule} min_split={min_split}")
    lay = fdc.Layout(1, H, 256, d_h, [rk], [rv], B, S, fdc.FDC_FP8, q_per_kv=g)
    t = lay.tables()
    RK, RV = int(t["koff_r"][0, -1]), int(t["voff_r"][0, -1])
    rng = gen.make_rng(17 * W + granule + g)
    # codes of latent rows with the decaying spectrum of the workloads, scaled into the format's range
    kcodes = np.zeros(B * S * RK, dtype=np.uint8)
    vcodes = np.zeros(B * S * RV, dtype=np.uint8)
    Ks, Vs = {}, {}
    ko, vo = np.concatenate([[0], np.cumsum(rk)]), np.concatenate([[0], np.cumsum(rv)])
    for b, n in enumerate(seq):
        for h in range(H):
            kq = fp8.quantise_latent(gen.direct_latent(n, rk[h], 32.0, rng) * 6.0)
            vq = fp8.quantise_latent(gen.direct_latent(n, rv[h], 32.0, rng) * 100.0)
            Ks[b, h], Vs[b, h] = fp8.e4m3_decode(kq), fp8.e4m3_decode(vq)
            k0, v0 = b * S * RK + S * ko[h], b * S * RV + S * vo[h]
            kcodes[k0:k0 + n * rk[h]] = kq.ravel()
            vcodes[v0:v0 + n * rv[h]] = vq.ravel()
    kc, vc = torch.from_numpy(kcodes).cuda(), torch.from_numpy(vcodes).cuda()
    q_lat = torch.from_numpy((rng.standard_normal((B, g * RK)) * 0.5).astype(np.float32)).cuda()
    o_lat = torch.full((B, g * RV), float("nan"), dtype=torch.float32, device="cuda:0")
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
    qo, oo = og.query_offsets(rk, g), og.query_offsets(rv, g)
    got_all, ref_all = [], []
    for b, n in enumerate(seq):
        for hq in range(H * g):
            h = hq // g
            got = out[b, oo[hq]:oo[hq + 1]]
            if n == 0:
                assert not got.any()
                continue
            ref = oa.latent_attn_decode(q64[b, qo[hq]:qo[hq + 1]], Ks[b, h], Vs[b, h], scale)
            # values reach +-448: the absolute bound scales with the largest value a head can output
            assert_close(got / 100.0, ref / 100.0, f"b={b} hq={hq} n={n}")
            got_all.append(got), ref_all.append(ref)
    ma, rl = assert_close(np.concatenate(got_all) / 100.0, np.concatenate(ref_all) / 100.0, "all")
    say(f"  tiles={plan.export()['n_items']} max_abs/100={ma:.2e} rel_l2={rl:.2e}")


@pytest.mark.parametrize("g", [1, 2])
@pytest.mark.parametrize("W,br,paged", [(5, 64, False), (40, 256, False), (9, 512, True)])
def test_prefill_attention_on_e4m3_codes(W, br, paged, g):
    """Causal prefill over E4M3 codes (dense and paged, chunked prompts, grouped queries): the kernel
    widens the codes to bf16 while staging, which is exact, so the bf16 tolerance applies."""
    from tests.test_gpu_paged import build_block_table
    from oracle import gqa as og
    from oracle import layout as ol
    rk, rv = [16, 48, 128, 64], [64, 16, 128, 32]
    H, d_h, P = len(rk), 128, 256
    kv = [1, 129, 700, 1300, 333]
    ql = [1, 129, 300, 1300, 0]
    say(f"prefill W={W} br={br} paged={paged} g={g}")
    rng = gen.make_rng(5 * W + br + g)
    RK, RV = sum(rk), sum(rv)
    if paged:
        bt, n_rows = build_block_table(kv, P, rng)
        lay = fdc.Layout(1, H, 256, d_h, [rk], [rv], n_rows, P, fdc.FDC_FP8, q_per_kv=g)
        row_len = P
    else:
        n_rows, row_len = len(kv), max(kv)
        lay = fdc.Layout(1, H, 256, d_h, [rk], [rv], n_rows, row_len, fdc.FDC_FP8, q_per_kv=g)
    kcodes, vcodes = np.zeros(n_rows * row_len * RK, np.uint8), np.zeros(n_rows * row_len * RV, np.uint8)
    ko, vo = np.concatenate([[0], np.cumsum(rk)]), np.concatenate([[0], np.cumsum(rv)])
    Ks, Vs = {}, {}
    for b, n in enumerate(kv):
        for h in range(H):
            kq = fp8.quantise_latent(gen.direct_latent(n, rk[h], 32.0, rng) * 6.0)
            vq = fp8.quantise_latent(gen.direct_latent(n, rv[h], 32.0, rng) * 100.0)
            Ks[b, h], Vs[b, h] = fp8.e4m3_decode(kq), fp8.e4m3_decode(vq)
            for tkn in range(n):
                if paged:
                    k0 = ol.paged_element_index(rk, P, bt[b], h, tkn, 0)
                    v0 = ol.paged_element_index(rv, P, bt[b], h, tkn, 0)
                else:
                    k0 = b * row_len * RK + row_len * ko[h] + tkn * rk[h]
                    v0 = b * row_len * RV + row_len * vo[h] + tkn * rv[h]
                kcodes[k0:k0 + rk[h]], vcodes[v0:v0 + rv[h]] = kq[tkn], vq[tkn]
    kc, vc = torch.from_numpy(kcodes).cuda(), torch.from_numpy(vcodes).cuda()
    T = int(np.sum(ql))
    q_lat = torch.from_numpy(gen.round_to_bf16(rng.standard_normal((T, g * RK)) * 0.3)).to(BF).cuda()
    o_lat = torch.full((T, g * RV), float("nan"), dtype=BF, device="cuda:0")
    pp = fdc.fdc_plan_params_default()
    pp.n_workers, pp.br_base, pp.br_cap, pp.cost_mode = W, br, br, 1
    plan = fdc.fdc_plan_prefill_paged(lay, 0, ql, kv, bt, pp) if paged else fdc.fdc_plan_prefill(lay, 0, ql, kv, pp)
    ws = workspace_for(plan)
    scale = 1 / math.sqrt(d_h)
    fdc.fdc_latent_attn_prefill(lay, plan, q_lat, kc, vc, scale, True, o_lat, ws)
    torch.cuda.synchronize()
    out, q64 = o_lat.to(torch.float64).cpu().numpy(), q_lat.to(torch.float64).cpu().numpy()
    assert np.all(np.isfinite(out))
    qo, oo = og.query_offsets(rk, g), og.query_offsets(rv, g)
    row0 = np.concatenate([[0], np.cumsum(ql)])
    got_all, ref_all = [], []
    for b in range(len(kv)):
        if ql[b] == 0:
            continue
        for hq in range(H * g):
            h = hq // g
            ref = oa.latent_attn_prefill(q64[row0[b]:row0[b + 1], qo[hq]:qo[hq + 1]], Ks[b, h], Vs[b, h], scale, True)
            got = out[row0[b]:row0[b + 1], oo[hq]:oo[hq + 1]]
            assert_close(got / 100.0, ref / 100.0, f"b={b} hq={hq}")
            got_all.append(got.ravel()), ref_all.append(ref.ravel())
    ma, rl = assert_close(np.concatenate(got_all) / 100.0, np.concatenate(ref_all) / 100.0, "all")
    say(f"  tasks={plan.export()['n_items']} max_abs/100={ma:.2e} rel_l2={rl:.2e}")


def test_post_rope_keys_are_stored_as_e4m3_codes():
    """fdc_rope_compress_keys on an FDC_FP8 layout. The kernel rounds the rotated keys to bf16 before its
    MFMA product, the oracle does not, so values near a rounding boundary (and, in absolute terms, values near zero where the codes are fine)
    can take another code: every decoded element must lie within half a code spacing plus the bf16-operand
    error of the oracle's value, and most codes must be the oracle's."""
    from oracle import rope as orp
    H, d_h, rk, T, n_pos = 4, 64, [16, 64, 32, 48], 130, 256
    g = gen.make_rng(41)
    B, S = 2, 200
    lay = fdc.Layout(1, H, 128, d_h, [rk], [rk], B, S, fdc.FDC_FP8)
    RK = sum(rk)
    kc = torch.zeros(B * S * RK, dtype=torch.uint8, device="cuda:0")
    R_t = np.concatenate([np.linalg.qr(g.standard_normal((d_h, d_h)))[0][:, :r].T for r in rk], axis=0)   # [RK, d_h]
    cos, sin = orp.rope_tables(n_pos, d_h)
    k = torch.from_numpy(gen.round_to_bf16(g.standard_normal((T, H, d_h)) * 20.0)).to(BF).cuda()
    R_d = torch.from_numpy(gen.round_to_bf16(R_t)).to(BF).cuda()
    slots = g.permutation(B * S)[:T]
    tb, tp = (slots // S).astype(np.int32), (slots % S).astype(np.int32)
    fdc.fdc_rope_compress_keys(lay, 0, k, torch.from_numpy(tb).cuda(), torch.from_numpy(tp).cuda(),
                               torch.from_numpy(cos.astype(np.float32)).cuda(), torch.from_numpy(sin.astype(np.float32)).cuda(),
                               R_d, kc)
    torch.cuda.synchronize()
    cos32, sin32 = cos.astype(np.float32).astype(np.float64), sin.astype(np.float32).astype(np.float64)
    off = np.concatenate([[0], np.cumsum(rk)])
    R64, k64, kb = R_d.to(torch.float64).cpu().numpy(), k.to(torch.float64).cpu().numpy(), kc.cpu().numpy()
    n_total = n_same = 0
    for h in range(H):
        want_rows = orp.rope(k64[:, h, :], tp, cos32, sin32) @ R64[off[h]:off[h + 1]].T
        want = fp8.quantise_latent(want_rows)
        got = np.stack([kb[b * S * RK + S * off[h] + p * rk[h]: b * S * RK + S * off[h] + (p + 1) * rk[h]] for b, p in zip(tb, tp)])
        # half a code spacing (at most 1/16 of the value) plus the error of the bf16 operands (values reach 60,
        # 64 terms: a few hundredths), which near zero spans several of the fine codes there
        err = np.abs(fp8.e4m3_decode(got) - want_rows)
        assert np.all(err <= np.abs(want_rows) / 16 + 0.15), (h, float(err.max()))
        n_total += got.size
        n_same += int((got == want).sum())
    assert kb.any() and n_same >= 0.85 * n_total, (n_same, n_total)
    say(f"  rope keys: {n_total} codes, {n_same} equal to the oracle's")


def test_one_launch_prologue_and_bf16_side_calls_on_an_e4m3_layout():
    """fdc_project_and_absorb_query writes the same codes and queries as the two calls; query absorption
    and output projection of an FDC_FP8 layout are those of the bf16 layout (only the cache differs)."""
    rk, rv = [16, 48, 128, 64], [64, 16, 128, 32]
    H, d, d_h, B, S, T = len(rk), 512, 128, 2, 64, 12
    lay8 = fdc.Layout(1, H, d, d_h, [rk], [rv], B, S, fdc.FDC_FP8)
    lay16 = fdc.Layout(1, H, d, d_h, [rk], [rv], B, S, fdc.FDC_BF16)
    RK, RV = sum(rk), sum(rv)
    g = gen.make_rng(77)
    x = torch.from_numpy(gen.round_to_bf16(gen.hidden_states(T, d, g))).to(BF).cuda()
    A = torch.from_numpy(gen.round_to_bf16(g.standard_normal((RK + RV, d)) * (40.0 / math.sqrt(d)))).to(BF).cuda()
    q = torch.from_numpy(gen.round_to_bf16(g.standard_normal((T, H, d_h)))).to(BF).cuda()
    Bk = torch.from_numpy(gen.round_to_bf16(g.standard_normal((RK, d_h)) / math.sqrt(d_h))).to(BF).cuda()
    slots = g.permutation(B * S)[:T]
    tb = torch.tensor(slots // S, dtype=torch.int32, device="cuda:0")
    tp = torch.tensor(slots % S, dtype=torch.int32, device="cuda:0")
    k2, v2 = torch.zeros(B * S * RK, dtype=torch.uint8, device="cuda:0"), torch.zeros(B * S * RV, dtype=torch.uint8, device="cuda:0")
    k1, v1 = torch.zeros_like(k2), torch.zeros_like(v2)
    q2 = torch.full((T, RK), float("nan"), dtype=torch.float32, device="cuda:0")
    q1, q16 = torch.full_like(q2, float("nan")), torch.full_like(q2, float("nan"))
    fdc.fdc_project_latent_kv(lay8, 0, x, tb, tp, A, k2, v2)
    fdc.fdc_absorb_query(lay8, 0, q, Bk, q2, fdc.FDC_F32)
    fdc.fdc_project_and_absorb_query(lay8, 0, x, tb, tp, A, k1, v1, q, Bk, q1, fdc.FDC_F32)
    fdc.fdc_absorb_query(lay16, 0, q, Bk, q16, fdc.FDC_F32)
    Mt = torch.from_numpy(gen.round_to_bf16(g.standard_normal((d, RV)) / math.sqrt(RV))).to(BF).cuda()
    o = torch.from_numpy(g.standard_normal((T, RV)).astype(np.float32)).cuda()
    y8 = torch.empty(T, d, dtype=BF, device="cuda:0")
    y16 = torch.empty(T, d, dtype=BF, device="cuda:0")
    fdc.fdc_absorb_output(lay8, 0, fdc.FDC_APPLY, None, None, Mt, o, fdc.FDC_F32, T, y8, fdc.FDC_BF16)
    fdc.fdc_absorb_output(lay16, 0, fdc.FDC_APPLY, None, None, Mt, o, fdc.FDC_F32, T, y16, fdc.FDC_BF16)
    torch.cuda.synchronize()
    assert k1.any() and torch.equal(k1, k2) and torch.equal(v1, v2)
    assert torch.equal(q1, q2) and torch.equal(q1, q16) and not torch.isnan(q1).any()
    assert torch.equal(y8, y16)


def test_paged_decode_on_e4m3_codes():
    from tests.test_gpu_paged import build_block_table
    from oracle import layout as ol
    rk, rv = [16, 64, 128], [32, 128, 16]
    H, d_h, P = len(rk), 128, 128
    seq = [5, 300, 0, 129]
    g = gen.make_rng(123)
    bt, n_pages = build_block_table(seq, P, g)
    lay = fdc.Layout(1, H, 256, d_h, [rk], [rv], n_pages, P, fdc.FDC_FP8)
    RK, RV = sum(rk), sum(rv)
    kcodes, vcodes = np.zeros(n_pages * P * RK, np.uint8), np.zeros(n_pages * P * RV, np.uint8)
    Ks, Vs = {}, {}
    for b, n in enumerate(seq):
        for h in range(H):
            kq = fp8.quantise_latent(gen.direct_latent(n, rk[h], 32.0, g) * 6.0)
            vq = fp8.quantise_latent(gen.direct_latent(n, rv[h], 32.0, g) * 50.0)
            Ks[b, h], Vs[b, h] = fp8.e4m3_decode(kq), fp8.e4m3_decode(vq)
            for tkn in range(n):
                k0 = ol.paged_element_index(rk, P, bt[b], h, tkn, 0)
                v0 = ol.paged_element_index(rv, P, bt[b], h, tkn, 0)
                kcodes[k0:k0 + rk[h]], vcodes[v0:v0 + rv[h]] = kq[tkn], vq[tkn]
    kc, vc = torch.from_numpy(kcodes).cuda(), torch.from_numpy(vcodes).cuda()
    B = len(seq)
    q_lat = torch.from_numpy((g.standard_normal((B, RK)) * 0.5).astype(np.float32)).cuda()
    o_lat = torch.full((B, RV), float("nan"), dtype=torch.float32, device="cuda:0")
    pp = fdc.fdc_plan_params_default()
    pp.n_workers = 19
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
            assert_close(got / 50.0, ref / 50.0, f"paged b={b} h={h}")


def test_decode_on_e4m3_codes_at_config3_size_sampled_units():
    """Layer 0 of the adaptive-rank decode config (batch 16, context 8192, 32 heads) with an E4M3 cache, in the
    launch configuration bench.py times (fdc_suggest_workers(3)): random finite codes on the device, the
    oracle on ~60 sampled (sequence, head) units including the narrowest and the widest head."""
    wl = gen.CONFIGS["c3_adaptive_decode"]
    r = wl.ranks()[0].tolist()
    H, B, S, d_h = wl.n_heads, wl.batch, wl.context, wl.d_head
    W = fdc.fdc_suggest_workers(3)
    say(f"config 3 layer 0, E4M3: B={B} S={S} W={W}")
    lay = fdc.Layout(1, H, wl.d_model, d_h, [r], [r], B, S, fdc.FDC_FP8)
    R = sum(r)
    tg = torch.Generator(device="cuda:0").manual_seed(3)
    mk = lambda: torch.randint(0, 0x7F, (B * S * R,), generator=tg, device="cuda:0", dtype=torch.uint8) | \
        (torch.randint(0, 2, (B * S * R,), generator=tg, device="cuda:0", dtype=torch.uint8) << 7)
    kc, vc = mk(), mk()
    rng = gen.make_rng(8)
    # codes are uniform over the grid, so values reach 448: small queries keep the scores in a softmax's range
    q_lat = torch.from_numpy((rng.standard_normal((B, R)) * 0.01).astype(np.float32)).cuda()
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
        k0 = b * S * R + S * off[h]
        K = fp8.e4m3_decode(kc[k0:k0 + S * r[h]].cpu().numpy()).reshape(S, r[h])
        V = fp8.e4m3_decode(vc[k0:k0 + S * r[h]].cpu().numpy()).reshape(S, r[h])
        ref = oa.latent_attn_decode(q64[b, off[h]:off[h + 1]], K, V, scale)
        assert_close(out[b, off[h]:off[h + 1]] / 100.0, ref / 100.0, f"b={b} h={h} r={r[h]}")
    say(f"  tiles={plan.export()['n_items']} units checked={len(units)}")


def _all_codes_rows():
    """[16, 16] uint8: every E4M3 code once (the two NaN codes replaced by zero), row t = codes 16 t .. 16 t + 15."""
    c = np.arange(256, dtype=np.uint8).reshape(16, 16).copy()
    c[c == 0x7F] = 0
    c[c == 0xFF] = 0
    return c


@pytest.mark.parametrize("g", [4, 16])
def test_grouped_decode_reads_every_e4m3_code_exactly(g):
    """The grouped kernel widens codes to bf16 operands with the hardware's packed conversion. Each query is peaked
    on one token (weights exactly one-hot in bf16), so an output row is that token's V' row decoded: all 254
    finite codes must come back as the format's values, bit for bit."""
    rows = _all_codes_rows()
    n, r = 16, 16
    B = n // g if g <= n else 1
    lay = fdc.Layout(1, 1, 256, 128, [[r]], [[r]], B, n, fdc.FDC_FP8, q_per_kv=g)
    key_codes = np.zeros((n, r), np.uint8)
    key_codes[np.arange(n), np.arange(n)] = fp8.quantise_latent(np.array([[64.0]]))[0, 0]      # K'[t] = 64 e_t
    kc = torch.from_numpy(np.tile(key_codes.ravel(), B)).cuda()
    vc = torch.from_numpy(np.tile(rows.ravel(), B)).cuda()
    q = np.zeros((B, g, r), np.float32)
    for b in range(B):
        for j in range(g):
            q[b, j, (b * g + j) % n] = 64.0                  # query (b, j) selects token b g + j: score 4096 * scale
    q_lat = torch.from_numpy(q.reshape(B, g * r)).cuda()
    o_lat = torch.full((B, g * r), float("nan"), dtype=torch.float32, device="cuda:0")
    pp = fdc.fdc_plan_params_default()
    pp.n_workers = 3
    plan = fdc.fdc_plan_decode(lay, 0, [n] * B, pp)
    ws = workspace_for(plan)
    fdc.fdc_latent_attn_decode(lay, plan, q_lat, kc, vc, 1 / math.sqrt(128), o_lat, ws)
    torch.cuda.synchronize()
    out = o_lat.cpu().numpy().reshape(B, g, r)
    want = fp8.e4m3_decode(rows)
    for b in range(B):
        for j in range(g):
            assert np.array_equal(out[b, j].astype(np.float64), want[(b * g + j) % n]), (b, j)


def test_prefill_reads_every_e4m3_code_exactly():
    """Same for the prefill kernel's staging (codes widened to bf16 on the way into LDS): row i is peaked on token i."""
    rows = _all_codes_rows()
    n, r = 16, 16
    lay = fdc.Layout(1, 1, 256, 128, [[r]], [[r]], 1, n, fdc.FDC_FP8)
    key_codes = np.zeros((n, r), np.uint8)
    key_codes[np.arange(n), np.arange(n)] = fp8.quantise_latent(np.array([[64.0]]))[0, 0]
    kc, vc = torch.from_numpy(key_codes.ravel()).cuda(), torch.from_numpy(rows.ravel().copy()).cuda()
    q_lat = (torch.eye(n, r) * 64.0).to(BF).cuda()
    o_lat = torch.full((n, r), float("nan"), dtype=BF, device="cuda:0")
    pp = fdc.fdc_plan_params_default()
    pp.n_workers, pp.br_base, pp.br_cap = 2, 64, 64
    plan = fdc.fdc_plan_prefill(lay, 0, [n], [n], pp)
    ws = workspace_for(plan)
    fdc.fdc_latent_attn_prefill(lay, plan, q_lat, kc, vc, 1 / math.sqrt(128), True, o_lat, ws)
    torch.cuda.synchronize()
    assert np.array_equal(o_lat.to(torch.float64).cpu().numpy(), fp8.e4m3_decode(rows))
