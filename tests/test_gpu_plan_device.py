"""The decode planner as a GPU kernel (fdc_plan_decode_device / _run / _download) against the integer
oracle planner: every table bit for bit; and decode through a device plan against decode through
the host plan of the same lengths (identical tiles in identical order: identical bits).
"""
import math
import sys

import numpy as np
import pytest
import torch

import paper_2408_04107_amd as fdc
from oracle import planner as op
from tests.gpu_util import Cache, workspace_for
from workloads import generators as gen

pytestmark = pytest.mark.gpu

PAIRS = [("item_b", "tile_b"), ("item_h", "tile_h"), ("item_lo", "tile_t0"), ("item_hi", "tile_t1"),
         ("item_cost", "tile_cost"), ("unit_item_ptr", "unit_tile_ptr"), ("worker_ptr", "worker_ptr"),
         ("worker_items", "worker_tiles"), ("worker_load", "worker_load")]


def say(msg):
    print(f"[device-planner] {msg}", flush=True)
    sys.stdout.flush()


def params(W, granule=64, min_split=1, split=1, softmax_cost=1):
    pp = fdc.fdc_plan_params_default()
    pp.n_workers, pp.granule, pp.min_split, pp.split, pp.softmax_cost = W, granule, min_split, split, softmax_cost
    return pp


def device_tables(lay, layer, seq, pp, max_pages=0, block_table=None):
    plan = fdc.fdc_plan_decode_device(lay, layer, len(seq), max_pages, pp)
    ws = workspace_for(plan)
    s = torch.tensor(seq, dtype=torch.int32, device="cuda:0")
    bt = None if block_table is None else torch.tensor(block_table, dtype=torch.int32, device="cuda:0").contiguous()
    fdc.fdc_plan_decode_run([plan], [ws], s, bt)
    fdc.fdc_plan_download(plan, ws)
    return plan, ws, plan.export()


def check_tables(got, want, what):
    assert got["n_items"] == len(want["tile_b"]), f"{what}: {got['n_items']} tiles, oracle {len(want['tile_b'])}"
    for a, b in PAIRS:
        assert np.array_equal(got[a], want[b]), f"{what}: table {a} differs from the oracle's {b}"


CASES = [
    # rk, rv, seq, W, granule, min_split, split, softmax_cost
    ([16, 32, 48, 64, 16, 32, 48, 64], [16, 32, 48, 64, 16, 32, 48, 64], [512], 64, 64, 1, 1, 1),
    ([16, 128, 64], [32, 16, 128], [1000, 0, 37, 4096, 64], 100, 64, 1, 1, 1),
    ([16, 128, 64], [32, 16, 128], [1000, 0, 37, 4096, 64], 7, 16, 3, 1, 4),
    ([16, 128, 64], [32, 16, 128], [1000, 0, 37, 4096, 64], 5, 64, 3, 0, 1),
    ([48] * 5, [80] * 5, [0, 0, 0], 64, 64, 1, 1, 1),
    ([48] * 5, [80] * 5, [1, 63, 64, 65], 3000, 64, 2, 1, 1),
    ([128] * 8, [128] * 8, [2048] * 4, 8192, 64, 1, 1, 1),
    ([16], [16], [5000], 1, 64, 1, 1, 1),
    # a granule that is no power of two, a worker count that is no multiple of 64
    ([32, 96, 16], [64, 16, 128], [700, 1, 0, 48, 49, 3000], 1000, 48, 2, 1, 7),
    # the most chunks the kernel sorts (8192), many heads; the largest worker count with it
    ([16 + 16 * (h % 8) for h in range(128)], [128 - 16 * (h % 8) for h in range(128)], [200 + 13 * b for b in range(64)], 4096, 64, 1, 1, 1),
    ([16, 64, 128, 32], [32, 16, 64, 128], [(37 * b) % 300 for b in range(2048)], 8192, 64, 1, 1, 1),
]


@pytest.mark.parametrize("case", range(len(CASES)))
def test_device_plan_tables_bit_exact(case):
    rk, rv, seq, W, G, ms, split, sc = CASES[case]
    say(f"tables case {case}: H={len(rk)} seq={seq} W={W} G={G} min_split={ms} split={split} softmax_cost={sc}")
    lay = fdc.Layout(1, len(rk), 256, 128, [rk], [rv], len(seq), max(max(seq), 1), fdc.FDC_BF16)
    _, _, got = device_tables(lay, 0, seq, params(W, G, ms, split, sc))
    want = op.plan_decode(seq, rk, rv, W, G, ms, bool(split), sc)
    check_tables(got, want, f"case {case}")


def test_device_plan_tables_adaptive_config_and_many_layers():
    """The adaptive-rank decode configuration (32 heads, batch 16, context 8192, 4096 workers), three
    layers planned by one launch, lengths ragged inside the last granule."""
    L, H, B = 3, 32, 16
    rk = gen.adaptive_ranks(L, H, 0)
    rv = gen.adaptive_ranks(L, H, 1)
    seq = [8192 - 64 * (b % 5) - (b * 7) % 64 for b in range(B)]
    say(f"adaptive config, {L} layers in one launch, seq={seq}")
    lay = fdc.Layout(L, H, 256, 128, rk, rv, B, 8192, fdc.FDC_BF16)
    pp = params(4096)
    plans = [fdc.fdc_plan_decode_device(lay, l, B, 0, pp) for l in range(L)]
    wss = [workspace_for(p) for p in plans]
    s = torch.tensor(seq, dtype=torch.int32, device="cuda:0")
    fdc.fdc_plan_decode_run(plans, wss, s)
    for l in range(L):
        fdc.fdc_plan_download(plans[l], wss[l])
        check_tables(plans[l].export(), op.plan_decode(seq, rk[l], rv[l], 4096, 64, 1, True, 1), f"layer {l}")
    # a second run on the same workspaces with other lengths replaces the plan
    seq2 = [max(0, s_ - 3000) for s_ in seq]
    s.copy_(torch.tensor(seq2, dtype=torch.int32))
    fdc.fdc_plan_decode_run(plans, wss, s)
    for l in range(L):
        fdc.fdc_plan_download(plans[l], wss[l])
        check_tables(plans[l].export(), op.plan_decode(seq2, rk[l], rv[l], 4096, 64, 1, True, 1), f"re-plan layer {l}")


def test_device_plan_paged_tables_bit_exact():
    rk, rv = [16, 128, 64, 48], [32, 16, 128, 48]
    P, max_pages, n_pages = 128, 9, 48
    seq = [1000, 0, 129, 1152, 128]
    rng = np.random.default_rng(3)
    bt = rng.permutation(n_pages)[: len(seq) * max_pages].reshape(len(seq), max_pages).astype(np.int32)
    say(f"paged tables: P={P} seq={seq}")
    lay = fdc.Layout(1, len(rk), 256, 128, [rk], [rv], n_pages, P, fdc.FDC_BF16)
    for W, G in ((50, 64), (500, 32)):
        _, _, got = device_tables(lay, 0, seq, params(W, G), max_pages, bt)
        want = op.plan_decode(seq, rk, rv, W, G, 1, True, 1, page_tokens=P)
        check_tables(got, want, f"paged W={W} G={G}")


def _decode_pair(lay, cache, seq, pp, max_pages=0, bt=None, g=1):
    """Decode through the host plan and through the device plan of the same lengths."""
    B = len(seq)
    rng = gen.make_rng(11)
    q_lat = torch.from_numpy(rng.standard_normal((B, g * cache.RK)).astype(np.float32)).cuda()
    scale = 1.0 / math.sqrt(128)
    host = fdc.fdc_plan_decode(lay, 0, seq, pp) if bt is None else fdc.fdc_plan_decode_paged(lay, 0, seq, bt, pp)
    ws_h = workspace_for(host)
    o_h = torch.full((B, g * cache.RV), float("nan"), dtype=torch.float32, device="cuda:0")
    fdc.fdc_latent_attn_decode(lay, host, q_lat, cache.k, cache.v, scale, o_h, ws_h)
    dev = fdc.fdc_plan_decode_device(lay, 0, B, max_pages, pp)
    ws_d = workspace_for(dev)
    s = torch.tensor(seq, dtype=torch.int32, device="cuda:0")
    btd = None if bt is None else torch.tensor(bt, dtype=torch.int32, device="cuda:0").contiguous()
    fdc.fdc_plan_decode_run([dev], [ws_d], s, btd)
    o_d = torch.full((B, g * cache.RV), float("nan"), dtype=torch.float32, device="cuda:0")
    fdc.fdc_latent_attn_decode(lay, dev, q_lat, cache.k, cache.v, scale, o_d, ws_d)   # no download in between
    torch.cuda.synchronize()
    return o_h.cpu().numpy(), o_d.cpu().numpy()


# worker counts that are multiples of 64 take the launch-slot order (heavier workers on the even XCDs) on both
# planners: few workers, three and four per planner thread, most of them idle (a tie at load zero)
@pytest.mark.parametrize("W", [100, 128, 3072, 4096])
@pytest.mark.parametrize("g,dtype", [(1, fdc.FDC_BF16), (4, fdc.FDC_BF16), (1, fdc.FDC_FP8)])
def test_decode_through_device_plan_equals_host_plan(g, dtype, W):
    rk, rv = [16, 32, 48, 64, 80, 96, 112, 128], [128, 16, 48, 64, 32, 112, 96, 80]
    seq = [700, 0, 64, 2048, 1]
    say(f"decode through a device plan: g={g} dtype={dtype} W={W} seq={seq}")
    lay = fdc.Layout(1, len(rk), 256, 128, [rk], [rv], len(seq), 2048, dtype, q_per_kv=g)
    t = lay.tables()
    tg = torch.Generator(device="cuda:0").manual_seed(5)
    es = {fdc.FDC_BF16: 2, fdc.FDC_FP8: 1}[dtype]

    class Buf:
        pass
    cache = Buf()
    nk, nv = int(t["k_bytes"][0]) // es, int(t["v_bytes"][0]) // es
    if dtype == fdc.FDC_BF16:
        cache.k = torch.randn(nk, generator=tg, device="cuda:0").to(torch.bfloat16)
        cache.v = torch.randn(nv, generator=tg, device="cuda:0").to(torch.bfloat16)
    else:   # any E4M3 codes except the two NaN patterns
        cache.k = torch.randint(0, 127, (nk,), generator=tg, device="cuda:0", dtype=torch.uint8)
        cache.v = torch.randint(0, 127, (nv,), generator=tg, device="cuda:0", dtype=torch.uint8)
    cache.RK, cache.RV = int(t["koff_r"][0, -1]), int(t["voff_r"][0, -1])
    o_h, o_d = _decode_pair(lay, cache, seq, params(W), g=g)
    assert np.all(np.isfinite(o_h)) and np.array_equal(o_h, o_d)


def test_decode_through_paged_device_plan_equals_host_plan():
    rk, rv = [16, 128, 64, 48], [32, 16, 128, 48]
    P, max_pages, n_pages = 128, 6, 24
    seq = [700, 0, 129, 768]
    rng = np.random.default_rng(4)
    bt = rng.permutation(n_pages).reshape(len(seq), max_pages).astype(np.int32)
    say(f"paged decode through a device plan: P={P} seq={seq}")
    lay = fdc.Layout(1, len(rk), 256, 128, [rk], [rv], n_pages, P, fdc.FDC_BF16)
    cache = Cache(lay)
    tg = torch.Generator(device="cuda:0").manual_seed(6)
    cache.k.copy_(torch.randn(cache.k.numel(), generator=tg, device="cuda:0").to(torch.bfloat16))
    cache.v.copy_(torch.randn(cache.v.numel(), generator=tg, device="cuda:0").to(torch.bfloat16))
    o_h, o_d = _decode_pair(lay, cache, seq, params(64), max_pages, bt)
    assert np.all(np.isfinite(o_h)) and np.array_equal(o_h, o_d)


def test_device_plan_reports_bad_lengths_and_pages():
    rk, rv = [16, 64], [32, 16]
    lay = fdc.Layout(1, 2, 256, 128, [rk], [rv], 3, 512, fdc.FDC_BF16)
    say("bad length on the device")
    plan = fdc.fdc_plan_decode_device(lay, 0, 3, 0, params(16))
    ws = workspace_for(plan)
    fdc.fdc_plan_decode_run([plan], [ws], torch.tensor([100, 513, -4], dtype=torch.int32, device="cuda:0"))
    with pytest.raises(fdc.FdcError, match="outside"):
        fdc.fdc_plan_download(plan, ws)
    # planned as clamped: the tables are those of [100, 512, 0]
    check_tables(plan.export(), op.plan_decode([100, 512, 0], rk, rv, 16, 64, 1, True, 1), "clamped lengths")
    say("bad page on the device")
    layp = fdc.Layout(1, 2, 256, 128, [rk], [rv], 8, 128, fdc.FDC_BF16)
    plan = fdc.fdc_plan_decode_device(layp, 0, 2, 2, params(16))
    ws = workspace_for(plan)
    bt = torch.tensor([[0, 99], [3, -1]], dtype=torch.int32, device="cuda:0")
    fdc.fdc_plan_decode_run([plan], [ws], torch.tensor([256, 128], dtype=torch.int32, device="cuda:0"), bt)
    with pytest.raises(fdc.FdcError, match="page"):
        fdc.fdc_plan_download(plan, ws)


def test_device_plan_export_needs_download():
    lay = fdc.Layout(1, 2, 256, 128, [[16, 64]], [[32, 16]], 3, 512, fdc.FDC_BF16)
    plan = fdc.fdc_plan_decode_device(lay, 0, 3, 0, params(16))
    with pytest.raises(fdc.FdcError, match="download"):
        plan.export()
