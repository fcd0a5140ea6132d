"""Caches larger than 4 GiB: the units under test start 4.5 GiB into the K' and V' buffers, past
what 32-bit byte offsets (and 32-bit element offsets) can address. Decode, causal prefill and the
three projection kernels (few rows, up to 64 rows, large) are compared with the float64 oracle on
the bits they read and wrote there.
"""
import math
import sys

import numpy as np
import pytest
import torch

import paper_2408_04107_amd as fdc
from oracle import attention as oa
from tests.gpu_util import Cache, assert_close, workspace_for

pytestmark = pytest.mark.gpu

H, D_MODEL, D_HEAD, RANK = 32, 512, 128, 128
B, S = 10, 65536                      # 512 MiB per sequence and side: sequence 9 starts at 4.5 GiB
LAST = B - 1
HEADS = (0, 17, 31)


def say(msg):
    print(f"[large-offsets] {msg}", flush=True)
    sys.stdout.flush()


def f64(t):
    return t.to(torch.float64).cpu().numpy()


@pytest.fixture(scope="module")
def big():
    free, _ = torch.cuda.mem_get_info()
    if free < 14 << 30:
        pytest.skip("needs 14 GiB of free device memory")
    lay = fdc.Layout(1, H, D_MODEL, D_HEAD, [[RANK] * H], [[RANK] * H], B, S, fdc.FDC_BF16)
    cache = Cache(lay)
    assert cache.k.numel() * 2 > (5 << 30) - 1 and LAST * S * cache.RK > 2 ** 31
    gt = torch.Generator(device="cuda:0").manual_seed(77)
    sig = torch.exp(-torch.arange(RANK, device="cuda:0", dtype=torch.float32) / 32.0)
    for h in HEADS:
        for side in ("k", "v"):
            u = cache.unit(side, LAST, h)
            u.copy_((torch.randn(S, RANK, generator=gt, device="cuda:0") * sig).to(u.dtype))
    yield lay, cache
    del cache
    torch.cuda.empty_cache()


def test_decode_past_4gib(big):
    lay, cache = big
    seq = [0] * LAST + [S]
    say(f"decode: sequence {LAST} of {S} tokens, units start at {LAST * S * cache.RK * 2 / 2**30:.2f} GiB")
    pp = fdc.fdc_plan_params_default()
    pp.n_workers = 4096
    plan = fdc.fdc_plan_decode(lay, 0, seq, pp)
    ws = workspace_for(plan)
    gt = torch.Generator(device="cuda:0").manual_seed(1)
    q_lat = torch.randn(B, cache.RK, generator=gt, device="cuda:0")
    o_lat = torch.full((B, cache.RV), float("nan"), dtype=torch.float32, device="cuda:0")
    scale = 1.0 / math.sqrt(D_HEAD)
    fdc.fdc_latent_attn_decode(lay, plan, q_lat, cache.k, cache.v, scale, o_lat, ws)
    torch.cuda.synchronize()
    out, q = f64(o_lat), f64(q_lat)
    assert np.all(out[:LAST] == 0.0)                       # empty sequences give zeros
    for h in HEADS:
        K, V = cache.unit_f64("k", LAST, h, S), cache.unit_f64("v", LAST, h, S)
        ref = oa.latent_attn_decode(q[LAST, h * RANK:(h + 1) * RANK], K, V, scale)
        ma, rl = assert_close(out[LAST, h * RANK:(h + 1) * RANK], ref, f"decode head {h}", rel_l2_tol=2e-4)
        say(f"  head {h}: max_abs={ma:.2e} rel_l2={rl:.2e}")


def test_prefill_past_4gib(big):
    lay, cache = big
    q_len, kv_len = [0] * LAST + [300], [0] * LAST + [S]
    say(f"prefill: the last {q_len[-1]} rows of sequence {LAST} ({S} keys)")
    pp = fdc.fdc_plan_params_default()
    pp.n_workers, pp.cost_mode = 256, 1
    plan = fdc.fdc_plan_prefill(lay, 0, q_len, kv_len, pp)
    ws = workspace_for(plan)
    gt = torch.Generator(device="cuda:0").manual_seed(2)
    T = q_len[-1]
    q_lat = torch.randn(T, cache.RK, generator=gt, device="cuda:0").to(torch.bfloat16)
    o_lat = torch.full((T, cache.RV), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    scale = 1.0 / math.sqrt(D_HEAD)
    fdc.fdc_latent_attn_prefill(lay, plan, q_lat, cache.k, cache.v, scale, True, o_lat, ws)
    torch.cuda.synchronize()
    assert not torch.isnan(o_lat.float()).any()
    out, q = f64(o_lat), f64(q_lat)
    rows = [0, 1, 15, 16, 255, 256, 299]
    for h in HEADS:
        K, V = cache.unit_f64("k", LAST, h, S), cache.unit_f64("v", LAST, h, S)
        ref = np.stack([oa.latent_attn_decode(q[r, h * RANK:(h + 1) * RANK], K[:S - T + r + 1], V[:S - T + r + 1], scale)
                        for r in rows])
        ma, rl = assert_close(out[rows, h * RANK:(h + 1) * RANK], ref, f"prefill head {h}")
        say(f"  head {h}: max_abs={ma:.2e} rel_l2={rl:.2e}")


@pytest.mark.parametrize("T", [16, 40, 300])
def test_projection_writes_past_4gib(big, T):
    """Runs last: it overwrites the tail rows of sequence 9."""
    lay, cache = big
    say(f"projection of {T} tokens into the last rows of sequence {LAST}")
    gt = torch.Generator(device="cuda:0").manual_seed(10 + T)
    bf = torch.bfloat16
    x = torch.randn(T, D_MODEL, generator=gt, device="cuda:0").to(bf)
    A_cat_t = (torch.randn(cache.RK + cache.RV, D_MODEL, generator=gt, device="cuda:0") / math.sqrt(D_MODEL)).to(bf)
    tb = torch.full((T,), LAST, dtype=torch.int32, device="cuda:0")
    tp = torch.arange(S - T, S, dtype=torch.int32, device="cuda:0")
    before = cache.unit("k", LAST - 1, H - 1)[S - 8:].clone()     # the rows just in front of sequence 9
    fdc.fdc_project_latent_kv(lay, 0, x, tb, tp, A_cat_t, cache.k, cache.v)
    torch.cuda.synchronize()
    assert torch.equal(before.view(torch.int16), cache.unit("k", LAST - 1, H - 1)[S - 8:].view(torch.int16))
    x64, A64 = f64(x), f64(A_cat_t)
    got, ref = [], []
    for h in HEADS:
        Kh = oa.project_latent_kv(x64, [A64[h * RANK:(h + 1) * RANK].T])[0]
        Vh = oa.project_latent_kv(x64, [A64[cache.RK + h * RANK:cache.RK + (h + 1) * RANK].T])[0]
        got.append(f64(cache.unit("k", LAST, h)[S - T:]).ravel()), ref.append(Kh.ravel())
        got.append(f64(cache.unit("v", LAST, h)[S - T:]).ravel()), ref.append(Vh.ravel())
    ma, rl = assert_close(np.concatenate(got), np.concatenate(ref), f"projected rows T={T}")
    say(f"  max_abs={ma:.2e} rel_l2={rl:.2e}")
