"""GPU parity of fdc_latent_attn_prefill (MFMA, causal) against the float64 oracle on identical
stored bf16 inputs: whole outputs at small sizes, sampled query rows at the config-5 size.
"""
import math
import sys

import numpy as np
import pytest
import torch

import paper_2408_04107_amd as fdc
from oracle import attention as oa
from tests.gpu_util import Cache, assert_close, workspace_for
from workloads import generators as gen

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[prefill-parity] {msg}", flush=True)
    sys.stdout.flush()


def run_prefill(rk, rv, q_len, kv_len, W, cost_mode=1, causal=True, seed=0, br_base=64, br_cap=256,
                decay=32.0, sample_rows=None, device_fill=False, q_gain=1.0, softmax_cost=1):
    H, B = len(rk), len(q_len)
    S_max = max(max(kv_len), 1)
    lay = fdc.Layout(1, H, 256, 128, [rk], [rv], B, S_max, fdc.FDC_BF16)
    cache = Cache(lay)
    g = gen.make_rng(seed)
    tg = torch.Generator(device="cuda:0").manual_seed(seed)
    for b in range(B):
        for h in range(H):
            if kv_len[b] == 0:
                continue
            if device_fill:
                for side, r in (("k", rk[h]), ("v", rv[h])):
                    sig = torch.exp(-torch.arange(r, device="cuda:0", dtype=torch.float32) / decay)
                    u = cache.unit(side, b, h)
                    u[:kv_len[b]] = (torch.randn(kv_len[b], r, generator=tg, device="cuda:0") * sig).to(u.dtype)
            else:
                cache.fill_unit("k", b, h, gen.direct_latent(kv_len[b], rk[h], decay, g))
                cache.fill_unit("v", b, h, gen.direct_latent(kv_len[b], rv[h], decay, g))
    T = int(sum(q_len))
    q_lat = (torch.randn(T, cache.RK, generator=tg, device="cuda:0") * q_gain).to(torch.bfloat16)
    o_lat = torch.full((T, cache.RV), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    pp = fdc.fdc_plan_params_default()
    pp.n_workers, pp.cost_mode, pp.br_base, pp.br_cap, pp.softmax_cost = W, cost_mode, br_base, br_cap, softmax_cost
    plan = fdc.fdc_plan_prefill(lay, 0, q_len, kv_len, pp)
    ws = workspace_for(plan)
    scale = 1.0 / math.sqrt(128)
    fdc.fdc_latent_attn_prefill(lay, plan, q_lat, cache.k, cache.v, scale, causal, o_lat, ws)
    torch.cuda.synchronize()
    out = o_lat.to(torch.float64).cpu().numpy()
    q64 = q_lat.to(torch.float64).cpu().numpy()
    kr, vr = cache.t["koff_r"][0], cache.t["voff_r"][0]
    row0 = np.concatenate([[0], np.cumsum(q_len)])
    got_all, ref_all = [], []
    for b in range(B):
        if q_len[b] == 0:
            continue
        for h in range(H):
            K = cache.unit_f64("k", b, h, kv_len[b])
            V = cache.unit_f64("v", b, h, kv_len[b])
            Q = q64[row0[b]:row0[b + 1], kr[h]:kr[h + 1]]
            O = out[row0[b]:row0[b + 1], vr[h]:vr[h + 1]]
            if sample_rows is None:
                ref = oa.latent_attn_prefill(Q, K, V, scale, causal)
                got = O
            else:
                rows = sorted({r for r in sample_rows(b, h) if 0 <= r < q_len[b]})
                ref = np.stack([oa.latent_attn_decode(
                    Q[r], K[:kv_len[b] - q_len[b] + r + 1] if causal else K,
                    V[:kv_len[b] - q_len[b] + r + 1] if causal else V, scale) for r in rows])
                got = O[rows]
            assert_close(got, ref, f"unit b={b} h={h} rk={rk[h]} rv={rv[h]}")
            got_all.append(got.ravel()), ref_all.append(ref.ravel())
    assert not torch.isnan(o_lat.float()).any(), "some output rows were never written"
    ma, rl = assert_close(np.concatenate(got_all), np.concatenate(ref_all), "all units")
    return ma, rl, plan.export()["n_items"]


MIX_K = [16, 32, 48, 64, 80, 96, 112, 128]
MIX_V = [128, 16, 48, 64, 32, 112, 96, 80]


@pytest.mark.parametrize("W,cost_mode", [(1, 1), (8, 0), (8, 1), (300, 0), (300, 1)])
def test_prefill_mixed_ranks(W, cost_mode):
    say(f"mixed ranks W={W} cost_mode={cost_mode}")
    ma, rl, n = run_prefill(MIX_K, MIX_V, [300, 64], [300, 64], W, cost_mode=cost_mode, seed=W)
    say(f"  tasks={n} max_abs={ma:.2e} rel_l2={rl:.2e}")


def test_prefill_ragged_lengths_and_chunked_queries():
    say("ragged lengths, queries = last rows of a longer context")
    ma, rl, n = run_prefill(MIX_K, MIX_V, [0, 5, 130, 17, 1], [0, 9, 130, 400, 1], 16, seed=3)
    say(f"  tasks={n} max_abs={ma:.2e} rel_l2={rl:.2e}")


def test_prefill_non_causal():
    say("non-causal")
    ma, rl, n = run_prefill(MIX_K, MIX_K, [150, 33], [200, 33], 16, causal=False, seed=4)
    say(f"  tasks={n} max_abs={ma:.2e} rel_l2={rl:.2e}")


def test_prefill_peaked_queries():
    say("peaked queries (q x 8): outputs O(1)")
    ma, rl, n = run_prefill(MIX_K, MIX_K, [513], [513], 64, q_gain=8.0, seed=6)
    say(f"  tasks={n} max_abs={ma:.2e} rel_l2={rl:.2e}")


def test_prefill_row_blocks_other_than_default():
    say("row-block parameters: base 128 / cap 256 and base 16 / cap 48")
    run_prefill(MIX_K, MIX_V, [700], [700], 32, br_base=128, br_cap=256, seed=7)
    run_prefill(MIX_K, MIX_V, [100], [100], 32, br_base=16, br_cap=48, seed=8)


def test_prefill_config5_size_sampled_rows():
    wl = gen.CONFIGS["c5_prefill"]
    r = wl.ranks()[0].tolist()
    W = fdc.fdc_suggest_workers(1)
    S = wl.context
    say(f"config 5 size: B={wl.batch} S={S}, W={W}")
    g = gen.make_rng(11)
    fixed = [0, 15, 16, 63, 64, 127, 128, 255, 256, S - 1]

    def rows(b, h):
        return fixed + [int(x) for x in g.integers(0, S, 6)]

    ma, rl, n = run_prefill(r, r, [S] * wl.batch, [S] * wl.batch, W, cost_mode=1, device_fill=True,
                            sample_rows=rows, seed=12, br_base=512, br_cap=512, softmax_cost=150)   # bench.py's launch configuration
    say(f"  tasks={n} max_abs={ma:.2e} rel_l2={rl:.2e}")
