"""GPU parity of decode attention over a paged latent cache (fdc_plan_decode_paged): tokens are
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
    q_used = q_lat.to(torch.float64).cpu().numpy() if g == 1 else q_lat.to(BF).to(torch.float64).cpu().numpy()
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
    say(f"  tiles={plan.export()['n_items']} max_abs={ma:.2e} rel_l2={rl:.2e}")
