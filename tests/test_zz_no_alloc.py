"""fdc_latent_attn_decode_static (the decode call on the workspace built into the library, for
callers that cannot allocate) against fdc_latent_attn_decode on a caller-allocated workspace:
identical kernels on identical tables, so the outputs must agree bit for bit. Two calls in a row
share the built-in workspace, the second with a smaller input, then the first plan again (its
tables have been overwritten in between and must be brought back)."""
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
    print(f"[no-alloc] {msg}", flush=True)
    sys.stdout.flush()


def make_case(rk, rv, seq, W, seed, min_split=1, dtype=fdc.FDC_BF16, q_per_kv=1):
    H, B = len(rk), len(seq)
    lay = fdc.Layout(1, H, 256, 128, [rk], [rv], B, max(seq), dtype, q_per_kv=q_per_kv)
    cache = Cache(lay)
    g = gen.make_rng(seed)
    for b in range(B):
        for h in range(H):
            if seq[b]:
                cache.fill_unit("k", b, h, gen.direct_latent(seq[b], rk[h], 32.0, g))
                cache.fill_unit("v", b, h, gen.direct_latent(seq[b], rv[h], 32.0, g))
    q_lat = torch.from_numpy((g.standard_normal((B, q_per_kv * cache.RK)) * 4.0).astype(np.float32)).cuda()
    pp = fdc.fdc_plan_params_default()
    pp.n_workers, pp.min_split = W, min_split
    plan = fdc.fdc_plan_decode(lay, 0, seq, pp)
    return dict(lay=lay, cache=cache, q_lat=q_lat, plan=plan, seq=seq, rk=rk, rv=rv, g=q_per_kv,
                scale=1.0 / math.sqrt(128))


def run_both(c, what):
    say(f"{what}: units {len(c['seq'])}x{len(c['rk'])}, tiles {c['plan'].export()['n_items']}, "
        f"workspace {c['plan'].workspace_bytes()} B")
    cache = c["cache"]
    shape = (len(c["seq"]), c["g"] * cache.RV)
    want = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda:0")
    got = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda:0")
    ws = workspace_for(c["plan"])
    fdc.fdc_latent_attn_decode(c["lay"], c["plan"], c["q_lat"], cache.k, cache.v, c["scale"], want, ws)
    fdc.fdc_latent_attn_decode_static(c["lay"], c["plan"], c["q_lat"], cache.k, cache.v, c["scale"], got)
    torch.cuda.synchronize()
    assert torch.isfinite(got).all(), f"{what}: non-finite output"
    assert torch.equal(got, want), f"{what}: differs from fdc_latent_attn_decode"
    return got


def test_static_workspace_decode_two_calls_in_a_row():
    mix_k = [16, 32, 48, 64, 80, 96, 112, 128]
    mix_v = [128, 16, 48, 64, 32, 112, 96, 80]
    big = make_case(mix_k, mix_v, [3000, 777, 0, 4096, 64, 1], W=4096, seed=3, min_split=3)
    small = make_case([48, 128, 16], [32, 128, 64], [257, 130], W=64, seed=4)
    out_big = run_both(big, "first call")
    # against the oracle too (a few units), so the pair cannot agree on a wrong answer
    cache, qh = big["cache"], big["q_lat"].cpu().numpy().astype(np.float64)
    kr, vr = cache.t["koff_r"][0], cache.t["voff_r"][0]
    o = out_big.cpu().numpy().astype(np.float64)
    for b, h in [(0, 0), (0, 7), (3, 4), (5, 2), (1, 1)]:
        S = big["seq"][b]
        ref = oa.latent_attn_decode(qh[b, kr[h]:kr[h + 1]], cache.unit_f64("k", b, h, S), cache.unit_f64("v", b, h, S),
                                    big["scale"])
        assert_close(o[b, vr[h]:vr[h + 1]], ref, f"unit b={b} h={h}", rel_l2_tol=2e-4)
    assert not o[2].any()                      # the empty sequence gives zeros
    run_both(small, "second call, smaller input")
    run_both(small, "third call, tables already resident")
    run_both(big, "fourth call, first plan again")


def test_static_workspace_grouped_queries_then_multi_head():
    grouped = make_case([32, 96], [64, 16], [900, 300, 1500], W=128, seed=5, q_per_kv=4)
    run_both(grouped, "grouped queries")
    plain = make_case([16, 128, 64], [48, 16, 128], [2000, 100], W=256, seed=6)
    run_both(plain, "multi-head after the grouped call")


def test_static_workspace_rejects_what_does_not_fit():
    # a plan whose workspace exceeds the built-in one: many tiles, 132 floats of partial state each
    H, B = 32, 16
    lay = fdc.Layout(1, H, 256, 128, [[16] * H], [[16] * H], B, 8192, fdc.FDC_BF16)
    pp = fdc.fdc_plan_params_default()
    pp.n_workers, pp.min_split = 4096, 64
    plan = fdc.fdc_plan_decode(lay, 0, [8192] * B, pp)
    assert plan.workspace_bytes() > 8 << 20
    cache = Cache(lay)
    q = torch.zeros(B, cache.RK, dtype=torch.float32, device="cuda:0")
    o = torch.full((B, cache.RV), 7.0, dtype=torch.float32, device="cuda:0")
    with pytest.raises(fdc.FdcError) as e:
        fdc.fdc_latent_attn_decode_static(lay, plan, q, cache.k, cache.v, 0.1, o)
    assert e.value.status == -4 and "built-in" in str(e.value)
    torch.cuda.synchronize()
    assert bool((o == 7.0).all())              # nothing was launched
    pp.min_split = 1
    dp = fdc.fdc_plan_decode_device(lay, 0, B, 0, pp)
    with pytest.raises(fdc.FdcError) as e:
        fdc.fdc_latent_attn_decode_static(lay, dp, q, cache.k, cache.v, 0.1, o)
    assert e.value.status == -1
