"""Decode attention on seeded random combinations of everything the call accepts: head count, unequal
ranks on the two sides, group size, cache type (bf16, fp32, E4M3), dense or paged cache, granule,
min_split, split on/off, worker count, host or GPU planner, planned or actual lengths
(fdc_latent_attn_decode_at). The structured tests cover each feature; these cover their products.
Every unit is compared with the float64 oracle on the stored bits.
"""
import math
import sys

import numpy as np
import pytest
import torch

import paper_2408_04107_amd as fdc
from oracle import attention as oa
from oracle import fp8
from oracle import gqa as og
from tests.gpu_util import assert_close, workspace_for

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[random-shapes] {msg}", flush=True)
    sys.stdout.flush()


def draw_case(seed):
    r = np.random.default_rng(1000 + seed)
    c = {}
    c["H"] = int(r.integers(1, 6))
    c["rk"] = [int(16 * r.integers(1, 9)) for _ in range(c["H"])]
    c["rv"] = [int(16 * r.integers(1, 9)) for _ in range(c["H"])]
    c["g"] = int(r.choice([1, 1, 1, 2, 3, 4, 8]))
    c["dtype"] = int(r.choice([fdc.FDC_BF16, fdc.FDC_BF16, fdc.FDC_FP8] + ([fdc.FDC_F32] if c["g"] == 1 else [])))
    c["B"] = int(r.integers(1, 5))
    c["granule"] = int(r.choice([16, 32, 64]))
    c["len"] = [int(x) for x in np.where(r.random(c["B"]) < 0.15, 0, r.integers(1, 900, c["B"]))]
    c["paged"] = bool(r.random() < 0.5)
    c["P"] = c["granule"] * int(r.choice([1, 2, 4]))
    c["W"] = int(r.choice([1, 5, 40, 333]))
    c["min_split"] = int(r.choice([1, 1, 2, 3]))
    c["split"] = int(r.choice([1, 1, 1, 0]))
    c["at"] = bool(r.random() < 0.5)           # plan for lengths rounded up to the granule, run at the actual ones
    c["device_plan"] = bool(r.random() < 0.5)
    return c, r


@pytest.mark.parametrize("seed", range(32))
def test_decode_random_combination(seed):
    c, r = draw_case(seed)
    say(f"seed {seed}: {c}")
    H, g, B, G, P = c["H"], c["g"], c["B"], c["granule"], c["P"]
    rk, rv, lens = c["rk"], c["rv"], c["len"]
    planned = [-(-n // G) * G for n in lens] if c["at"] else list(lens)
    S_cap = max(max(planned), 1)
    if c["paged"]:
        max_pages = max(1, -(-S_cap // P))
        n_pages = B * max_pages + 2
        bt = r.permutation(n_pages)[:B * max_pages].reshape(B, max_pages).astype(np.int32)
        rows, row_tokens = n_pages, P
    else:
        bt, max_pages, rows, row_tokens = None, 0, B, S_cap
    lay = fdc.Layout(1, H, 256, 128, [rk], [rv], rows, row_tokens, c["dtype"], q_per_kv=g)
    t = lay.tables()
    RK, RV = int(t["koff_r"][0, -1]), int(t["voff_r"][0, -1])
    tg = torch.Generator(device="cuda:0").manual_seed(seed)
    nk, nv = rows * row_tokens * RK, rows * row_tokens * RV
    if c["dtype"] == fdc.FDC_FP8:     # any code but the two NaN patterns, magnitudes up to 30
        mk = lambda n: (torch.randint(0, 0x60, (n,), generator=tg, device="cuda:0", dtype=torch.uint8)
                        | (torch.randint(0, 2, (n,), generator=tg, device="cuda:0", dtype=torch.uint8) << 7))
        kc, vc = mk(nk), mk(nv)
        k64 = fp8.e4m3_decode(kc.cpu().numpy())
        v64 = fp8.e4m3_decode(vc.cpu().numpy())
        vmax = 30.0
    else:
        dt = torch.bfloat16 if c["dtype"] == fdc.FDC_BF16 else torch.float32
        kc = (torch.randn(nk, generator=tg, device="cuda:0") * 0.7).to(dt)
        vc = torch.randn(nv, generator=tg, device="cuda:0").to(dt)
        k64, v64 = kc.to(torch.float64).cpu().numpy(), vc.to(torch.float64).cpu().numpy()
        vmax = 1.0
    q_lat = torch.randn(B, g * RK, generator=tg, device="cuda:0") * 1.5
    o_lat = torch.full((B, g * RV), float("nan"), dtype=torch.float32, device="cuda:0")
    pp = fdc.fdc_plan_params_default()
    pp.n_workers, pp.granule, pp.min_split, pp.split = c["W"], G, c["min_split"], c["split"]
    lens_dev = torch.tensor(lens, dtype=torch.int32, device="cuda:0")
    if c["device_plan"]:
        plan = fdc.fdc_plan_decode_device(lay, 0, B, max_pages, pp)
        ws = workspace_for(plan)
        btd = None if bt is None else torch.tensor(bt, dtype=torch.int32, device="cuda:0").contiguous()
        fdc.fdc_plan_decode_run([plan], [ws], torch.tensor(planned, dtype=torch.int32, device="cuda:0"), btd)
    else:
        plan = fdc.fdc_plan_decode(lay, 0, planned, pp) if bt is None else fdc.fdc_plan_decode_paged(lay, 0, planned, bt, pp)
        ws = workspace_for(plan)
    scale = 1.0 / math.sqrt(128)
    if c["at"]:
        fdc.fdc_latent_attn_decode_at(lay, plan, lens_dev, q_lat, kc, vc, scale, o_lat, ws)
    else:
        fdc.fdc_latent_attn_decode(lay, plan, q_lat, kc, vc, scale, o_lat, ws)
    torch.cuda.synchronize()
    out = o_lat.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(out)), "some output was never written"
    q64 = q_lat.to(torch.float64).cpu().numpy()
    qo, oo = og.query_offsets(rk, g), og.query_offsets(rv, g)
    koff, voff = np.concatenate([[0], np.cumsum(rk)]), np.concatenate([[0], np.cumsum(rv)])

    def unit_rows(buf, R, off, rank, b, n):
        """Rows 0..n-1 of unit (b, h): cache row = the sequence (dense) or the page of the token (paged)."""
        tok = np.arange(n)
        row = np.full(n, b) if bt is None else bt[b][tok // P]
        in_row = tok if bt is None else tok % P
        base = row.astype(np.int64) * row_tokens * R + row_tokens * off + in_row * rank
        return buf[base[:, None] + np.arange(rank)[None, :]]

    got_all, ref_all = [], []
    for b, n in enumerate(lens):
        for h in range(H):
            K = unit_rows(k64, RK, koff[h], rk[h], b, n)
            V = unit_rows(v64, RV, voff[h], rv[h], b, n)
            for j in range(g):
                hq = h * g + j
                got = out[b, oo[hq]:oo[hq + 1]]
                if n == 0:
                    assert not got.any(), f"b={b} hq={hq}: empty sequence must give zeros"
                    continue
                ref = oa.latent_attn_decode(q64[b, qo[hq]:qo[hq + 1]], K, V, scale)
                assert_close(got / vmax, ref / vmax, f"b={b} hq={hq} n={n} rk={rk[h]} rv={rv[h]}")
                got_all.append(got), ref_all.append(ref)
    if got_all:
        ma, rl = assert_close(np.concatenate(got_all) / vmax, np.concatenate(ref_all) / vmax, "all units")
        say(f"  max_abs={ma:.2e} rel_l2={rl:.2e}")


def draw_prefill_case(seed):
    r = np.random.default_rng(5000 + seed)
    c = {}
    c["H"] = int(r.integers(1, 5))
    c["rk"] = [int(16 * r.integers(1, 9)) for _ in range(c["H"])]
    c["rv"] = [int(16 * r.integers(1, 9)) for _ in range(c["H"])]
    c["g"] = int(r.choice([1, 1, 2, 4]))
    c["dtype"] = int(r.choice([fdc.FDC_BF16, fdc.FDC_BF16, fdc.FDC_FP8]))
    c["B"] = int(r.integers(1, 4))
    c["kv"] = [int(x) for x in r.integers(1, 700, c["B"])]
    c["q"] = [int(r.integers(0, n + 1)) if r.random() < 0.5 else n for n in c["kv"]]
    c["paged"] = bool(r.random() < 0.5)
    c["P"] = int(r.choice([128, 256]))
    c["W"] = int(r.choice([1, 7, 64, 300]))
    c["cost_mode"] = int(r.choice([0, 1]))
    c["br"] = int(r.choice([64, 256, 512]))
    c["causal"] = bool(r.random() < 0.8)
    return c, r


@pytest.mark.parametrize("seed", range(16))
def test_prefill_random_combination(seed):
    c, r = draw_prefill_case(seed)
    say(f"prefill seed {seed}: {c}")
    H, g, B, P = c["H"], c["g"], c["B"], c["P"]
    rk, rv, kv, ql = c["rk"], c["rv"], c["kv"], c["q"]
    S_cap = max(kv)
    if c["paged"]:
        max_pages = -(-S_cap // P)
        n_pages = B * max_pages + 2
        bt = r.permutation(n_pages)[:B * max_pages].reshape(B, max_pages).astype(np.int32)
        rows, row_tokens = n_pages, P
    else:
        bt, rows, row_tokens = None, B, S_cap
    lay = fdc.Layout(1, H, 256, 128, [rk], [rv], rows, row_tokens, c["dtype"], q_per_kv=g)
    t = lay.tables()
    RK, RV = int(t["koff_r"][0, -1]), int(t["voff_r"][0, -1])
    tg = torch.Generator(device="cuda:0").manual_seed(100 + seed)
    nk, nv = rows * row_tokens * RK, rows * row_tokens * RV
    if c["dtype"] == fdc.FDC_FP8:
        mk = lambda n: (torch.randint(0, 0x48, (n,), generator=tg, device="cuda:0", dtype=torch.uint8)
                        | (torch.randint(0, 2, (n,), generator=tg, device="cuda:0", dtype=torch.uint8) << 7))
        kc, vc = mk(nk), mk(nv)
        k64, v64 = fp8.e4m3_decode(kc.cpu().numpy()), fp8.e4m3_decode(vc.cpu().numpy())
        vmax = 4.0
    else:
        kc = (torch.randn(nk, generator=tg, device="cuda:0") * 0.7).to(torch.bfloat16)
        vc = torch.randn(nv, generator=tg, device="cuda:0").to(torch.bfloat16)
        k64, v64 = kc.to(torch.float64).cpu().numpy(), vc.to(torch.float64).cpu().numpy()
        vmax = 1.0
    T = int(sum(ql))
    q_lat = torch.randn(max(T, 1), g * RK, generator=tg, device="cuda:0").to(torch.bfloat16)[:T]
    o_lat = torch.full((max(T, 1), g * RV), float("nan"), dtype=torch.bfloat16, device="cuda:0")[:T]
    pp = fdc.fdc_plan_params_default()
    pp.n_workers, pp.cost_mode, pp.br_base, pp.br_cap = c["W"], c["cost_mode"], c["br"], c["br"]
    plan = fdc.fdc_plan_prefill(lay, 0, ql, kv, pp) if bt is None else fdc.fdc_plan_prefill_paged(lay, 0, ql, kv, bt, pp)
    ws = workspace_for(plan)
    scale = 1.0 / math.sqrt(128)
    fdc.fdc_latent_attn_prefill(lay, plan, q_lat, kc, vc, scale, c["causal"], o_lat, ws)
    torch.cuda.synchronize()
    if T == 0:
        return
    assert not torch.isnan(o_lat.float()).any(), "some output rows were never written"
    out, q64 = o_lat.to(torch.float64).cpu().numpy(), q_lat.to(torch.float64).cpu().numpy()
    qo, oo = og.query_offsets(rk, g), og.query_offsets(rv, g)
    koff, voff = np.concatenate([[0], np.cumsum(rk)]), np.concatenate([[0], np.cumsum(rv)])

    def unit_rows(buf, R, off, rank, b, n):
        tok = np.arange(n)
        row = np.full(n, b) if bt is None else bt[b][tok // P]
        in_row = tok if bt is None else tok % P
        base = row.astype(np.int64) * row_tokens * R + row_tokens * off + in_row * rank
        return buf[base[:, None] + np.arange(rank)[None, :]]

    row0 = np.concatenate([[0], np.cumsum(ql)])
    got_all, ref_all = [], []
    for b in range(B):
        if ql[b] == 0:
            continue
        for h in range(H):
            K = unit_rows(k64, RK, koff[h], rk[h], b, kv[b])
            V = unit_rows(v64, RV, voff[h], rv[h], b, kv[b])
            for j in range(g):
                hq = h * g + j
                ref = oa.latent_attn_prefill(q64[row0[b]:row0[b + 1], qo[hq]:qo[hq + 1]], K, V, scale, c["causal"])
                got = out[row0[b]:row0[b + 1], oo[hq]:oo[hq + 1]]
                assert_close(got / vmax, ref / vmax, f"b={b} hq={hq} q={ql[b]} kv={kv[b]} rk={rk[h]} rv={rv[h]}")
                got_all.append(got.ravel()), ref_all.append(ref.ravel())
    ma, rl = assert_close(np.concatenate(got_all) / vmax, np.concatenate(ref_all) / vmax, "all units")
    say(f"  max_abs={ma:.2e} rel_l2={rl:.2e}")
