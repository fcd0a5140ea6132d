"""GPU parity of decode and prefill attention over a paged latent cache (fdc_plan_decode_paged,
fdc_plan_prefill_paged). Decode: tokens are
written page by page through fdc_project_latent_kv (tok_batch = page, tok_pos = offset), pages are
scattered over the buffer by a random block table, and the result is compared with the float64
oracle on the rows gathered back in sequence order. Multi-head and grouped-query layouts.
"""
import math
import sys

import numpy as np
import pytest
import torch

import paper_2408_04107_amd as fdc
from oracle import attention as oa
from oracle import gqa as og
from oracle import layout as ol
from tests.gpu_util import Cache, assert_close, workspace_for
from workloads import generators as gen

pytestmark = pytest.mark.gpu
BF = torch.bfloat16


def say(msg):
    print(f"[paged-parity] {msg}", flush=True)
    sys.stdout.flush()


def build_block_table(seq, P, rng, spare=3):
    max_pages = max(1, max(-(-s // P) for s in seq))
    n_pages = sum(-(-s // P) for s in seq) + spare
    perm = rng.permutation(n_pages)
    bt = np.zeros((len(seq), max_pages), dtype=np.int32)
    k = 0
    for b, S in enumerate(seq):
        for i in range(-(-S // P)):
            bt[b, i] = perm[k]
            k += 1
    return bt, n_pages


@pytest.mark.parametrize("g", [1, 4])
@pytest.mark.parametrize("P,granule,W,min_split", [(64, 64, 33, 1), (256, 64, 500, 2), (128, 32, 7, 1)])
def test_paged_decode(g, P, granule, W, min_split):
    say(f"paged decode g={g} P={P} granule={granule} W={W} min_split={min_split}")
    rng = gen.make_rng(P + W + g)
    rk, rv = [16, 48, 128, 64], [64, 16, 128, 32]
    H, d, d_h = len(rk), 256, 128
    seq = [0, 1, 63, 64, 65, 700, 1300]
    bt, n_pages = build_block_table(seq, P, rng)
    lay = fdc.Layout(1, H, d, d_h, [rk], [rv], n_pages, P, fdc.FDC_BF16, q_per_kv=g)
    cache = Cache(lay)
    # write every token through the projection, with page / offset addressing
    A_cat_t = torch.from_numpy((rng.standard_normal((cache.RK + cache.RV, d)) / math.sqrt(d)).astype(np.float32)).to(BF).cuda()
    x_all, tb, tp = [], [], []
    for b, S in enumerate(seq):
        xs = gen.hidden_states(S, d, rng)
        x_all.append(xs)
        tb += [int(bt[b, t // P]) for t in range(S)]
        tp += [t % P for t in range(S)]
    x = torch.from_numpy(np.concatenate(x_all, axis=0).astype(np.float32)).to(BF).cuda()
    order = rng.permutation(len(tb))     # token order is irrelevant
    fdc.fdc_project_latent_kv(lay, 0, x[torch.from_numpy(order).cuda()].contiguous(),
                              torch.tensor(np.asarray(tb)[order], dtype=torch.int32, device="cuda:0"),
                              torch.tensor(np.asarray(tp)[order], dtype=torch.int32, device="cuda:0"),
                              A_cat_t, cache.k, cache.v)
    B = len(seq)
    q_lat = torch.from_numpy((rng.standard_normal((B, g * cache.RK)) * 3.0).astype(np.float32)).cuda()
    o_lat = torch.full((B, g * cache.RV), float("nan"), dtype=torch.float32, device="cuda:0")
    pp = fdc.fdc_plan_params_default()
    pp.n_workers, pp.granule, pp.min_split = W, granule, min_split
    plan = fdc.fdc_plan_decode_paged(lay, 0, seq, bt, pp)
    ws = workspace_for(plan)
    scale = 1 / math.sqrt(d_h)
    fdc.fdc_latent_attn_decode(lay, plan, q_lat, cache.k, cache.v, scale, o_lat, ws)
    torch.cuda.synchronize()
    out = o_lat.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(out))
    q_used = q_lat.to(torch.float64).cpu().numpy()
    qo, oo = og.query_offsets(rk, g), og.query_offsets(rv, g)
    kbuf, vbuf = cache.k.to(torch.float64).cpu().numpy(), cache.v.to(torch.float64).cpu().numpy()
    got_all, ref_all = [], []
    for b, S in enumerate(seq):
        for h in range(H):
            # gather the unit's rows through the oracle's paged index
            K = np.array([[kbuf[ol.paged_element_index(rk, P, bt[b], h, t, i)] for i in range(rk[h])] for t in range(S)]).reshape(S, rk[h])
            V = np.array([[vbuf[ol.paged_element_index(rv, P, bt[b], h, t, i)] for i in range(rv[h])] for t in range(S)]).reshape(S, rv[h])
            for j in range(g):
                hq = h * g + j
                ref = oa.latent_attn_decode(q_used[b, qo[hq]:qo[hq + 1]], K, V, scale)
                got = out[b, oo[hq]:oo[hq + 1]]
                assert_close(got, ref, f"b={b} hq={hq} S={S}")
                got_all.append(got), ref_all.append(ref)
    ma, rl = assert_close(np.concatenate(got_all), np.concatenate(ref_all), "all")
    # the projection itself landed where the oracle's paged index says
    x64, A64 = x.to(torch.float64).cpu().numpy(), A_cat_t.to(torch.float64).cpu().numpy()
    koff = np.concatenate([[0], np.cumsum(rk)])
    row0 = int(np.sum(seq[:5]))          # first token of the 700-token sequence
    for h in (0, 2):
        for t in (0, P - 1, P, 699):
            ref = x64[row0 + t] @ A64[koff[h]:koff[h + 1]].T
            got = np.array([kbuf[ol.paged_element_index(rk, P, bt[5], h, t, i)] for i in range(rk[h])])
            assert_close(got, ref, f"projected K' row t={t} h={h}")
    # the entry point on the library's own workspace takes paged plans as well: same tables, same bits
    o_static = torch.full_like(o_lat, float("nan"))
    fdc.fdc_latent_attn_decode_static(lay, plan, q_lat, cache.k, cache.v, scale, o_static)
    torch.cuda.synchronize()
    assert torch.equal(o_static, o_lat)
    say(f"  tiles={plan.export()['n_items']} max_abs={ma:.2e} rel_l2={rl:.2e}")


@pytest.mark.parametrize("g", [1, 2])
@pytest.mark.parametrize("P,W,br", [(128, 9, 64), (256, 40, 256), (512, 3, 512)])
def test_paged_prefill(g, P, W, br):
    """Causal prefill over a paged cache (fdc_plan_prefill_paged): chunked prompts (q_len < kv_len),
    lengths that end inside a page and inside a staged block, pages scattered by a random block table."""
    say(f"paged prefill g={g} P={P} W={W} br={br}")
    rng = gen.make_rng(7 * P + W + g)
    rk, rv = [16, 48, 128, 64], [64, 16, 128, 32]
    H, d_h = len(rk), 128
    kv = [1, 127, 128, 129, 700, 1300, 333]
    ql = [1, 100, 128, 129, 700, 300, 0]
    bt, n_pages = build_block_table(kv, P, rng)
    lay = fdc.Layout(1, H, 256, d_h, [rk], [rv], n_pages, P, fdc.FDC_BF16, q_per_kv=g)
    cache = Cache(lay)
    RK, RV = cache.RK, cache.RV
    koff, voff = np.concatenate([[0], np.cumsum(rk)]), np.concatenate([[0], np.cumsum(rv)])
    # latent rows per (sequence, head), rounded to bf16, written into their pages on the host
    kbuf = np.zeros(cache.k.numel(), dtype=np.float64)
    vbuf = np.zeros(cache.v.numel(), dtype=np.float64)
    Ks, Vs = {}, {}
    for b, S in enumerate(kv):
        for h in range(H):
            Ks[b, h] = gen.round_to_bf16(gen.direct_latent(S, rk[h], 32.0, rng))
            Vs[b, h] = gen.round_to_bf16(gen.direct_latent(S, rv[h], 32.0, rng))
            for t in range(S):
                k0 = ol.paged_element_index(rk, P, bt[b], h, t, 0)
                v0 = ol.paged_element_index(rv, P, bt[b], h, t, 0)
                kbuf[k0:k0 + rk[h]] = Ks[b, h][t]
                vbuf[v0:v0 + rv[h]] = Vs[b, h][t]
    cache.k.copy_(torch.from_numpy(kbuf).to(BF))
    cache.v.copy_(torch.from_numpy(vbuf).to(BF))
    T = int(np.sum(ql))
    q_lat = torch.from_numpy(gen.round_to_bf16(rng.standard_normal((T, g * RK)) * 2.0)).to(BF).cuda()
    o_lat = torch.full((T, g * RV), float("nan"), dtype=BF, device="cuda:0")
    pp = fdc.fdc_plan_params_default()
    pp.n_workers, pp.br_base, pp.br_cap, pp.cost_mode = W, br, max(br, 16), 1
    plan = fdc.fdc_plan_prefill_paged(lay, 0, ql, kv, bt, pp)
    ws = workspace_for(plan)
    scale = 1 / math.sqrt(d_h)
    fdc.fdc_latent_attn_prefill(lay, plan, q_lat, cache.k, cache.v, scale, True, o_lat, ws)
    torch.cuda.synchronize()
    out = o_lat.to(torch.float64).cpu().numpy()
    assert np.all(np.isfinite(out))
    q64 = q_lat.to(torch.float64).cpu().numpy()
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
            assert_close(got, ref, f"b={b} hq={hq}")
            got_all.append(got.ravel()), ref_all.append(ref.ravel())
    ma, rl = assert_close(np.concatenate(got_all), np.concatenate(ref_all), "all")
    # the schedule is the dense one: pages do not cut query blocks
    dense = fdc.Layout(1, H, 256, d_h, [rk], [rv], len(kv), max(kv), fdc.FDC_BF16, q_per_kv=g)
    tp, td = plan.export(), fdc.fdc_plan_prefill(dense, 0, ql, kv, pp).export()
    for key in ("item_b", "item_h", "item_lo", "item_hi", "item_cost", "worker_ptr", "worker_items", "worker_load"):
        assert np.array_equal(tp[key], td[key]), key
    say(f"  tasks={tp['n_items']} max_abs={ma:.2e} rel_l2={rl:.2e}")


def test_paged_prefill_rejects_a_page_that_splits_a_staged_block():
    lay = fdc.Layout(1, 2, 64, 32, [[16, 32]], [[16, 16]], 8, 64, fdc.FDC_BF16)   # 64-token pages
    pp = fdc.fdc_plan_params_default()
    pp.n_workers = 4
    with pytest.raises(fdc.FdcError):
        fdc.fdc_plan_prefill_paged(lay, 0, [10], [100], np.array([[0, 1]], dtype=np.int32), pp)
