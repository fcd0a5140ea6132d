#!/usr/bin/env python3
"""Benchmark of the latent-KV attention hot path on one MI355X.

Default workload: the adaptive-rank decode configuration (32 layers x 32 heads, d_head 128,
per-(layer, head) rank drawn from {16..128} with P(r) ~ 1/r, batch 16, context 8192, bf16 cache).
One step = one decode step through all layers: latent projection of the new token, query
absorption, decode attention on the latent cache (tile kernel + split-K merge) and output
absorption. Inputs are synthetic, seeded, and resident in HBM before the timed region.

Prints ONE JSON line. `value` is the algorithmic HBM bytes of a whole step divided by the step
time; `roofline` describes the dominant kernel (the decode tile kernel) from HIP events recorded
around that kernel alone; `cpu_baseline` is the float64 oracle timed on the host on a bounded
sample; `prefill` reports the MFMA calls of the prefill configuration in TFLOP/s. Further objects of
the same line are side measurements of the other rows (`c2_uniform_decode`, `c4_long_decode`: one layer over
rotating cache copies; `gqa_decode`, `fp8_decode`, `fp4_decode`, `device_planner`, `serving_loop`); each has a --no-... switch
and a failure in one of them is reported in its place.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0       # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16


class HipEvents:
    """hipEvent_t handles through the HIP runtime torch already loaded."""

    def __init__(self, n: int):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.ev = []
        for _ in range(n):
            e = ctypes.c_void_p()
            rc = self.hip.hipEventCreate(ctypes.byref(e))
            if rc != 0:
                raise RuntimeError(f"hipEventCreate failed: {rc}")
            self.ev.append(e)

    def ms(self, i: int, j: int) -> float:
        out = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(out), self.ev[i], self.ev[j])
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed: {rc}")
        return float(out.value)

    def destroy(self):
        for e in self.ev:
            self.hip.hipEventDestroy(e)
        self.ev = []


def fill_latent(buf, lay, tables_off_r, ranks, batch, S, decay, gen_t):
    """Fills a layer buffer [b][h][t][i] with N(0, s_i^2), s_i = exp(-i / decay): the value
    distribution of projected hidden states x ~ N(0, I) through a weight with that spectrum."""
    import torch
    R = int(tables_off_r[-1])
    sig = torch.cat([torch.exp(-torch.arange(int(r), device=buf.device, dtype=torch.float32) / decay).repeat(S)
                     for r in ranks])                       # one sequence: [S * R] in layout order
    view = buf.view(batch, S * R)
    for b in range(batch):
        view[b] = (torch.randn(S * R, generator=gen_t, device=buf.device) * sig).to(buf.dtype)


def decode_bytes(plan_tables, ranks_k, ranks_v, seq_len, RK, RV, batch):
    """Algorithmic bytes of one decode launch: every cached element once (bf16), q' in, o' or the
    partial state out."""
    kv = sum(int(s) * (int(rk) + int(rv)) * 2 for s in seq_len for rk, rv in zip(ranks_k, ranks_v))
    per_unit = np.diff(plan_tables["unit_item_ptr"])
    H = len(ranks_k)
    out = 0
    for u, n in enumerate(per_unit):
        rv = int(ranks_v[u % H])
        out += rv * 4 if n <= 1 else int(n) * (rv + 2) * 4
    return kv + batch * RK * 4 + out


def run_decode_workload(fdc, gen, wl, steps, warmup, args):
    import torch
    dev = "cuda:0"
    ranks = wl.ranks()
    L, H, B, S, d, dh = wl.n_layers, wl.n_heads, wl.batch, wl.context, wl.d_model, wl.d_head
    lay = fdc.Layout(L, H, d, dh, ranks, ranks, B, S, fdc.FDC_BF16)
    t = lay.tables()
    W = args.workers or fdc.fdc_suggest_workers(0)
    gt = torch.Generator(device=dev).manual_seed(wl.seed)
    bf = torch.bfloat16
    kc, vc, A_cat_t, Bk, Mt, plans, wss = [], [], [], [], [], [], []
    pp = fdc.fdc_plan_params_default()
    pp.n_workers, pp.min_split = W, wl.min_split
    pp.granule = args.granule or wl.granule
    t_plan = 0.0
    for l in range(L):
        k = torch.empty(int(t["k_bytes"][l]) // 2, dtype=bf, device=dev)
        v = torch.empty(int(t["v_bytes"][l]) // 2, dtype=bf, device=dev)
        fill_latent(k, lay, t["koff_r"][l], ranks[l], B, S, wl.decay, gt)
        fill_latent(v, lay, t["voff_r"][l], ranks[l], B, S, wl.decay, gt)
        kc.append(k), vc.append(v)
        RK, RV = int(t["koff_r"][l, -1]), int(t["voff_r"][l, -1])
        A_cat_t.append((torch.randn(RK + RV, d, generator=gt, device=dev) / math.sqrt(d)).to(bf))
        Bk.append((torch.randn(RK, dh, generator=gt, device=dev) / math.sqrt(dh)).to(bf))
        Mt.append((torch.randn(d, RV, generator=gt, device=dev) / math.sqrt(RV)).to(bf))
        t0 = time.perf_counter()
        plan = fdc.fdc_plan_decode(lay, l, [S] * B, pp)
        t_plan += time.perf_counter() - t0
        ws = torch.empty(plan.workspace_bytes() + 256, dtype=torch.uint8, device=dev)
        off = (-ws.data_ptr()) % 256
        ws = ws[off:off + plan.workspace_bytes()]
        fdc.fdc_plan_upload(plan, ws)
        plans.append(plan), wss.append(ws)
    x = torch.randn(B, d, generator=gt, device=dev).to(bf)
    q = torch.randn(B, H, dh, generator=gt, device=dev).to(bf)
    tb = torch.arange(B, dtype=torch.int32, device=dev)
    tp = torch.full((B,), S - 1, dtype=torch.int32, device=dev)
    RKmax = int(t["koff_r"][:, -1].max())
    RVmax = int(t["voff_r"][:, -1].max())
    q_lat = torch.empty(B * RKmax, dtype=torch.float32, device=dev)
    o_lat = torch.empty(B * RVmax, dtype=torch.float32, device=dev)
    y = torch.empty(B, d, dtype=bf, device=dev)
    scale = 1.0 / math.sqrt(dh)

    # replanning cost of a whole step's worth of layers, planned concurrently on the host cores (the
    # planner is pure host code and the binding releases the GIL): what a serving loop pays each time
    # a sequence crosses a granule boundary, i.e. once per `granule` decode steps
    from concurrent.futures import ThreadPoolExecutor
    n_thr = min(16, os.cpu_count() or 1, L)
    replan_runs = []
    with ThreadPoolExecutor(n_thr) as ex:
        for _ in range(5):      # the first pass also starts the pool's threads; the median is reported, all are listed
            t0 = time.perf_counter()
            fresh = list(ex.map(lambda l: fdc.fdc_plan_decode(lay, l, [S] * B, pp), range(L)))
            replan_runs.append((time.perf_counter() - t0) * 1e3)
            del fresh       # the old plans are released outside the timed interval
    replan_ms = float(np.median(replan_runs))

    tabs = [p.export() for p in plans]
    dec_bytes = [decode_bytes(tabs[l], ranks[l], ranks[l], [S] * B, int(t["koff_r"][l, -1]),
                              int(t["voff_r"][l, -1]), B) for l in range(L)]
    # algorithmic bytes of the other calls of a step: weights streamed once, activations in/out
    other_bytes = []
    for l in range(L):
        RK, RV = int(t["koff_r"][l, -1]), int(t["voff_r"][l, -1])
        proj = (RK + RV) * d * 2 + B * d * 2 + B * (RK + RV) * 2
        absq = RK * dh * 2 + B * H * dh * 2 + B * RK * 4
        apply_ = d * RV * 2 + B * RV * 4 + B * d * 2
        merge = sum(int(n) * (int(ranks[l][u % H]) + 2) * 4 for u, n in enumerate(np.diff(tabs[l]["unit_item_ptr"])) if n > 1)
        other_bytes.append(proj + absq + apply_ + merge)
    step_bytes = sum(dec_bytes) + sum(other_bytes)

    # HIP events around the tile kernel cost the stream about 5 us each time (the next kernel waits for
    # the event's timestamp), so a step times every fourth layer, rotating: each layer is timed in every
    # fourth step of the timed region and the instrumentation stays near 1% of a step.
    ev_stride = 4 if steps >= 4 else 1
    ev = HipEvents(2 * L * steps)
    timed = []   # (step, layer) of every event pair, in recording order

    def step(si=None):
        for l in range(L):
            # K'/V' of the new tokens and the absorbed queries: one launch at decode batch
            fdc.fdc_project_and_absorb_query(lay, l, x, tb, tp, A_cat_t[l], kc[l], vc[l], q, Bk[l], q_lat, fdc.FDC_F32)
            if si is not None and (l + si) % ev_stride == 0:
                i = 2 * len(timed)
                timed.append((si, l))
                fdc.fdc_profile_decode_events(ev.ev[i], ev.ev[i + 1])
            fdc.fdc_latent_attn_decode(lay, plans[l], q_lat, kc[l], vc[l], scale, o_lat, wss[l])
            fdc.fdc_absorb_output(lay, l, fdc.FDC_APPLY, None, None, Mt[l], o_lat, fdc.FDC_F32, B, y, fdc.FDC_BF16)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for si in range(steps):
        step(si)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps

    by_layer = [[] for _ in range(L)]
    for i, (_, l) in enumerate(timed):
        by_layer[l].append(ev.ms(2 * i, 2 * i + 1))
    ev.destroy()
    assert all(by_layer), "every layer is timed at least once"
    per_layer_ms = np.array([np.mean(v) for v in by_layer])
    avg_kernel_ms = float(per_layer_ms.mean())
    avg_bytes = float(np.mean(dec_bytes))
    achieved = avg_bytes / (avg_kernel_ms * 1e-3) / 1e9
    layer_gbps = np.array(dec_bytes) / (per_layer_ms * 1e-3) / 1e9
    imb = [float(tb_["worker_load"].max() / tb_["worker_load"].mean()) for tb_ in tabs]

    # decode attention call alone (tile kernel + merge), all layers back to back
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    reps = max(2, steps // 2)
    for _ in range(reps):
        for l in range(L):
            fdc.fdc_latent_attn_decode(lay, plans[l], q_lat, kc[l], vc[l], scale, o_lat, wss[l])
    torch.cuda.synchronize()
    attn_us_per_layer = (time.perf_counter() - t0) * 1e6 / (reps * L)

    # the other calls of a step on layer 0, each alone, 30 calls back to back (weight streams at decode
    # batch). A call costs the host about 10 us through ctypes, so these figures are upper bounds of the
    # kernels' durations; the kernel trace under profiles/ has the durations themselves.
    def timed_us(fn, n=30):
        fn()
        torch.cuda.synchronize()
        s_, e_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s_.record()
        for _ in range(n):
            fn()
        e_.record()
        torch.cuda.synchronize()
        return s_.elapsed_time(e_) * 1e3 / n
    RK0, RV0 = int(t["koff_r"][0, -1]), int(t["voff_r"][0, -1])
    small = {}
    us = timed_us(lambda: fdc.fdc_project_latent_kv(lay, 0, x, tb, tp, A_cat_t[0], kc[0], vc[0]))
    small["project_latent_kv"] = {"us": us, "weight_GBps": (RK0 + RV0) * d * 2 / us / 1e3}
    us = timed_us(lambda: fdc.fdc_absorb_query(lay, 0, q, Bk[0], q_lat, fdc.FDC_F32))
    small["absorb_query"] = {"us": us, "weight_GBps": RK0 * dh * 2 / us / 1e3}
    us = timed_us(lambda: fdc.fdc_project_and_absorb_query(lay, 0, x, tb, tp, A_cat_t[0], kc[0], vc[0], q, Bk[0], q_lat, fdc.FDC_F32))
    small["project_and_absorb_query"] = {"us": us, "weight_GBps": ((RK0 + RV0) * d + RK0 * dh) * 2 / us / 1e3}
    us = timed_us(lambda: fdc.fdc_absorb_output(lay, 0, fdc.FDC_APPLY, None, None, Mt[0], o_lat, fdc.FDC_F32, B, y, fdc.FDC_BF16))
    small["absorb_output_apply"] = {"us": us, "weight_GBps": d * RV0 * 2 / us / 1e3}

    # HBM bytes per launch of the tile kernel from the committed rocprofv3 counter summary (FETCH_SIZE and
    # WRITE_SIZE, each scaled by a plain copy of known size); null when that summary is for another workload
    traffic = None
    try:
        with open(os.path.join(ROOT, "profiles", "decode_tiles_traffic.json")) as fh:
            tj = json.load(fh)["decode_tiles_kernel"]
        if tj["workload"] == wl.name and wl.n_layers == gen.CONFIGS[wl.name].n_layers:
            traffic = tj["fetch_bytes_per_launch"] + tj["write_bytes_per_launch"]
    except (OSError, KeyError, ValueError):
        traffic = None

    result = {
        "ms_per_step": ms_per_step,
        "value": step_bytes / (ms_per_step * 1e-3) / 1e9,
        "roofline": {"bound": "hbm", "kernel": "decode_tiles_kernel", "achieved": achieved, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic,
                     "avg_launch_us": avg_kernel_ms * 1e3, "algorithmic_bytes_per_launch": avg_bytes,
                     "launches_timed": len(timed)},
        "decode_attn": {"us_per_layer_call": attn_us_per_layer,
                        "tile_kernel_us_per_layer": {"mean": float(per_layer_ms.mean() * 1e3),
                                                     "min": float(per_layer_ms.min() * 1e3),
                                                     "max": float(per_layer_ms.max() * 1e3)},
                        "tile_kernel_GBps_per_layer": {"min": float(layer_gbps.min()), "max": float(layer_gbps.max())},
                        "GBps_call": avg_bytes / (attn_us_per_layer * 1e-6) / 1e9,
                        "planner_imbalance_max_over_mean": {"mean": float(np.mean(imb)), "max": float(np.max(imb))},
                        "plan_host_ms_per_layer": t_plan * 1e3 / L,
                        "replan_all_layers_ms": replan_ms, "replan_all_layers_ms_runs": [round(v, 3) for v in replan_runs],
                        "replan_threads": n_thr,
                        "replan_amortised_fraction_of_step": replan_ms / pp.granule / ms_per_step,
                        "n_workers": W,
                        "tiles_per_layer": float(np.mean([tb_["n_items"] for tb_ in tabs])),
                        "by_layer": {"tile_kernel_GBps": [int(v) for v in layer_gbps],
                                     "tiles": [int(tb_["n_items"]) for tb_ in tabs],
                                     "max_tiles_of_a_unit": [int(np.diff(tb_["unit_item_ptr"]).max()) for tb_ in tabs]}},
        "decode_other_calls_layer0": small,
        "step_algorithmic_bytes": step_bytes,
    }
    state = dict(lay=lay, tables=t, kc=kc, vc=vc, ranks=ranks, q_lat=q_lat, scale=scale, B=B, S=S, H=H)
    return result, state


def cpu_baseline(state, budget_s=8.0):
    """The float64 oracle (as it stands) on the host cores, over (sequence, head) decode units of layer 0 of the
    same workload. The legs run in a child process that never touches the GPU (so it may fork workers): one
    thread; one single-threaded process per core over independent units (`value`); numpy's own threads on
    one unit at a time."""
    import subprocess
    ranks, S = state["ranks"], state["S"]
    spec = {"ranks": [int(r) for r in ranks[0]], "S": int(S), "scale": float(state["scale"]), "budget": budget_s}
    r = subprocess.run([sys.executable, os.path.abspath(__file__), "--oracle-legs", json.dumps(spec)],
                       capture_output=True, text=True, timeout=300)
    if r.returncode != 0:
        raise RuntimeError("oracle timing failed: " + r.stderr[-500:])
    return json.loads(r.stdout.strip().splitlines()[-1])


_LEG_DATA = []   # units of the oracle timing; forked workers inherit it, so only an index travels per unit


def _oracle_unit(i):
    from oracle import attention as oa
    qq, K, V, scale, nbytes = _LEG_DATA[i]
    oa.latent_attn_decode(qq, K, V, scale)
    return nbytes


def _one_blas_thread():
    from threadpoolctl import threadpool_limits
    threadpool_limits(limits=1)


def oracle_legs(spec):
    """Child-process part of cpu_baseline: no torch, no GPU."""
    import multiprocessing as mp
    from threadpoolctl import threadpool_info, threadpool_limits
    from workloads import generators as gen
    ranks, S, scale, budget = spec["ranks"], spec["S"], spec["scale"], spec["budget"]
    blas_threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    nproc = os.cpu_count() or 1
    cores = max(1, min(nproc, 16))          # the GPU machine gives one GPU's job 16 cores, whatever nproc says
    g = gen.make_rng(0)
    data = _LEG_DATA
    for h in g.integers(0, len(ranks), 32):
        r = ranks[int(h)]
        K = gen.round_to_bf16(gen.direct_latent(S, r, 32.0, g))
        V = gen.round_to_bf16(gen.direct_latent(S, r, 32.0, g))
        data.append((g.standard_normal(r), K, V, scale, S * 2 * r * 2))

    def leg(pool, budget_):
        done, n_units = 0, 0
        t0 = time.perf_counter()
        while time.perf_counter() - t0 < budget_:
            idx = range(len(data))
            done += sum(pool.map(_oracle_unit, idx, chunksize=1)) if pool else sum(_oracle_unit(i) for i in idx)
            n_units += len(data)
        dt = time.perf_counter() - t0
        return {"value": done / dt / 1e9, "unit": "GB/s", "us_per_unit": dt * 1e6 / n_units, "units": n_units, "seconds": dt}

    with threadpool_limits(limits=1):
        single = leg(None, budget * 0.4)
    with mp.get_context("fork").Pool(cores, initializer=_one_blas_thread) as pool:
        leg(pool, 0.5)                      # start the workers
        per_core = leg(pool, budget)
    blas = leg(None, budget * 0.4)
    return {"value": per_core["value"], "unit": "GB/s", "cores": cores, "kind": "oracle",
            "sample": f"{per_core['units']} (sequence, head) decode units of layer 0 (32 distinct, context {S}, bf16 bytes "
                      f"counted as for the GPU), {per_core['seconds']:.1f} s, one single-threaded process per core over "
                      "independent units",
            "us_per_unit": per_core["us_per_unit"], "nproc": nproc,
            "single_thread": {"value": single["value"], "unit": "GB/s", "us_per_unit": single["us_per_unit"],
                              "seconds": single["seconds"]},
            "numpy_threads_one_unit_at_a_time": {"value": blas["value"], "unit": "GB/s", "threads": int(blas_threads),
                                                 "us_per_unit": blas["us_per_unit"], "seconds": blas["seconds"]}}


# Vector-ALU cost of the softmax per score in the prefill kernel, from its instruction mix: per lane and 16 scores
# about 67 ordinary vector instructions (scale-and-subtract fma, running sum, maximum, packing to bf16, masks)
# and 17 v_exp_f32; measured issue cost with four waves per SIMD 2.4 and 8.5 cycles per wave instruction
# (the transcendental runs at quarter rate and does not overlap other vector work): 305 cycles per 1024 scores.
VALU_CYCLES_PER_SCORE = 305.0 / 1024.0
N_SIMD, SHADER_HZ = 256 * 4, 2.4e9


def valu_ceiling(n_scores, flops):
    """What the vector ALU alone allows: the time its softmax work takes on all SIMDs at the peak clock, and the
    TFLOP/s of the two products if nothing else took time. The lower of this and the MFMA peak bounds the kernel."""
    ms = n_scores * VALU_CYCLES_PER_SCORE / (N_SIMD * SHADER_HZ) * 1e3
    tf = flops / (ms * 1e-3) / 1e12
    return {"valu_only_ms": ms, "TFLOPs_if_valu_bound": tf, "binding_ceiling_TFLOPs": min(tf, MFMA_BF16_PEAK_TFLOPS),
            "bound": "valu/exp" if tf < MFMA_BF16_PEAK_TFLOPS else "mfma"}


def run_prefill_workload(fdc, gen, iters=20, warm=10):
    """Config 5: projection of 16384 tokens, causal latent attention, output absorption (bf16 MFMA)."""
    import torch
    dev = "cuda:0"
    wl = gen.CONFIGS["c5_prefill"]
    r = wl.ranks()[0]
    H, B, S, d, dh = wl.n_heads, wl.batch, wl.context, wl.d_model, wl.d_head
    lay = fdc.Layout(1, H, d, dh, [r], [r], B, S, fdc.FDC_BF16)
    t = lay.tables()
    RK, RV = int(t["koff_r"][0, -1]), int(t["voff_r"][0, -1])
    bf = torch.bfloat16
    gt = torch.Generator(device=dev).manual_seed(wl.seed)
    T = B * S
    x = torch.randn(T, d, generator=gt, device=dev).to(bf)
    A_cat_t = (torch.randn(RK + RV, d, generator=gt, device=dev) / math.sqrt(d)).to(bf)
    Bk = (torch.randn(RK, dh, generator=gt, device=dev) / math.sqrt(dh)).to(bf)
    Bv = (torch.randn(RV, dh, generator=gt, device=dev) / math.sqrt(dh)).to(bf)
    Wo_t = (torch.randn(d, H * dh, generator=gt, device=dev) / math.sqrt(H * dh)).to(bf)
    q = torch.randn(T, H, dh, generator=gt, device=dev).to(bf)
    kc = torch.zeros(int(t["k_bytes"][0]) // 2, dtype=bf, device=dev)
    vc = torch.zeros(int(t["v_bytes"][0]) // 2, dtype=bf, device=dev)
    tb = torch.arange(B, dtype=torch.int32, device=dev).repeat_interleave(S)
    tp = torch.arange(S, dtype=torch.int32, device=dev).repeat(B)
    q_lat = torch.empty(T, RK, dtype=bf, device=dev)
    o_lat = torch.empty(T, RV, dtype=bf, device=dev)
    Mt = torch.empty(d, RV, dtype=bf, device=dev)
    y = torch.empty(T, d, dtype=bf, device=dev)
    pp = fdc.fdc_plan_params_default()
    pp.n_workers, pp.cost_mode, pp.br_base, pp.br_cap, pp.softmax_cost = fdc.fdc_suggest_workers(1), 1, 512, 512, 150
    t0 = time.perf_counter()
    plan = fdc.fdc_plan_prefill(lay, 0, [S] * B, [S] * B, pp)
    plan_ms = (time.perf_counter() - t0) * 1e3
    ws = torch.empty(plan.workspace_bytes() + 256, dtype=torch.uint8, device=dev)
    off = (-ws.data_ptr()) % 256
    ws = ws[off:off + plan.workspace_bytes()]
    fdc.fdc_plan_upload(plan, ws)
    scale = 1.0 / math.sqrt(dh)
    calls = {
        "project_latent_kv": (lambda: fdc.fdc_project_latent_kv(lay, 0, x, tb, tp, A_cat_t, kc, vc), 2.0 * T * d * (RK + RV)),
        "absorb_query": (lambda: fdc.fdc_absorb_query(lay, 0, q, Bk, q_lat, fdc.FDC_BF16), 2.0 * T * dh * RK),
        "latent_attn_prefill": (lambda: fdc.fdc_latent_attn_prefill(lay, plan, q_lat, kc, vc, scale, True, o_lat, ws),
                                float(B * sum(int(rr) * 2 for rr in r) * 2 * (S * (S + 1) // 2))),
        "absorb_output_fold": (lambda: fdc.fdc_absorb_output(lay, 0, fdc.FDC_FOLD, Bv, Wo_t, Mt, None, 0, 0, None, 0), 2.0 * RV * dh * d),
        "absorb_output_apply": (lambda: fdc.fdc_absorb_output(lay, 0, fdc.FDC_APPLY, None, None, Mt, o_lat, fdc.FDC_BF16, T, y, fdc.FDC_BF16), 2.0 * T * RV * d),
    }
    # post-RoPE variant of the K / Q side (Section 5.1): RoPE + rotation truncated to r_h columns
    k_pre = torch.randn(T, H, dh, generator=gt, device=dev).to(bf)
    R_t = (torch.randn(RK, dh, generator=gt, device=dev) / math.sqrt(dh)).to(bf)
    ang = torch.arange(S, device=dev, dtype=torch.float32)[:, None] * \
        (10000.0 ** (-2.0 * torch.arange(dh // 2, device=dev, dtype=torch.float32) / dh))[None, :]
    cos_t, sin_t = torch.cos(ang).contiguous(), torch.sin(ang).contiguous()
    calls["rope_compress_keys"] = (lambda: fdc.fdc_rope_compress_keys(lay, 0, k_pre, tb, tp, cos_t, sin_t, R_t, kc),
                                   2.0 * T * dh * RK)
    calls["rope_absorb_query"] = (lambda: fdc.fdc_rope_absorb_query(lay, 0, q, tp, cos_t, sin_t, R_t, q_lat, fdc.FDC_BF16),
                                  2.0 * T * dh * RK)
    out = {"workload": "config 5: B=4, S=4096, d_model 4096, 32 heads, adaptive ranks", "plan_host_ms": plan_ms}
    total_ms = 0.0
    # every call: `warm` untimed calls (the shader clock settles over the first milliseconds of matrix work
    # after lighter kernels), then `iters` timed ones back to back
    for name, (fn, flops) in calls.items():
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s.record()
        for _ in range(iters):
            fn()
        e.record()
        torch.cuda.synchronize()
        ms = s.elapsed_time(e) / iters
        if not name.startswith("rope_"):
            total_ms += ms          # the five calls of the RoPE-free chain; the post-RoPE calls are alternatives
        out[name] = {"ms": ms, "TFLOPs": flops / (ms * 1e-3) / 1e12, "frac_of_bf16_mfma_peak": flops / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS}
        if name == "latent_attn_prefill":
            n_scores = float(B * H * (S * (S + 1) // 2))
            out[name]["softmax_valu_ceiling"] = valu_ceiling(n_scores, flops)
    out["total_ms"] = total_ms
    # attention alone by rank bucket: every head at the same rank (MFMA-bound when wide, exp-bound when narrow)
    buckets = {}
    del x, y, q, k_pre
    for rr in (16, 64, 128):
        ru = [rr] * H
        lay_u = fdc.Layout(1, H, d, dh, [ru], [ru], B, S, fdc.FDC_BF16)
        tu = lay_u.tables()
        kcu = torch.randn(int(tu["k_bytes"][0]) // 2, generator=gt, device=dev).to(bf)
        vcu = torch.randn(int(tu["v_bytes"][0]) // 2, generator=gt, device=dev).to(bf)
        qu = torch.randn(T, rr * H, generator=gt, device=dev).to(bf)
        ou = torch.empty(T, rr * H, dtype=bf, device=dev)
        plan_u = fdc.fdc_plan_prefill(lay_u, 0, [S] * B, [S] * B, pp)
        wsu = torch.empty(plan_u.workspace_bytes() + 256, dtype=torch.uint8, device=dev)
        offu = (-wsu.data_ptr()) % 256
        wsu = wsu[offu:offu + plan_u.workspace_bytes()]
        fdc.fdc_plan_upload(plan_u, wsu)
        fn = lambda: fdc.fdc_latent_attn_prefill(lay_u, plan_u, qu, kcu, vcu, scale, True, ou, wsu)
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s.record()
        for _ in range(iters):
            fn()
        e.record()
        torch.cuda.synchronize()
        ms = s.elapsed_time(e) / iters
        fl = float(B * H * rr * 2 * 2 * (S * (S + 1) // 2))
        buckets["rank_%d" % rr] = {"ms": ms, "TFLOPs": fl / (ms * 1e-3) / 1e12,
                                   "frac_of_bf16_mfma_peak": fl / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                                   "softmax_valu_ceiling": valu_ceiling(float(B * H * (S * (S + 1) // 2)), fl)}
    out["latent_attn_prefill_by_uniform_rank"] = buckets
    return out


def run_gqa_decode_workload(fdc, gen, iters=20):
    """Grouped-query decode attention (Section 5.1, GQA paragraph): 8 key/value heads shared by 4 query
    heads each (32 query heads), adaptive ranks, batch 64, context 8192, one layer."""
    import torch
    dev = "cuda:0"
    H, g, B, S, dh = 8, 4, 64, 8192, 128
    r = [int(x) for x in gen.adaptive_ranks(1, H, 11)[0]]
    lay = fdc.Layout(1, H, 4096, dh, [r], [r], B, S, fdc.FDC_BF16, q_per_kv=g)
    t = lay.tables()
    RK = int(t["koff_r"][0, -1])
    bf = torch.bfloat16
    gt = torch.Generator(device=dev).manual_seed(5)
    n = int(t["k_bytes"][0]) // 2
    kc = torch.randn(n, generator=gt, device=dev).to(bf)
    vc = torch.randn(n, generator=gt, device=dev).to(bf)
    q_lat = torch.randn(B, g * RK, generator=gt, device=dev)
    o_lat = torch.empty(B, g * RK, device=dev)
    pp = fdc.fdc_plan_params_default()
    pp.n_workers = fdc.fdc_suggest_workers(2)
    plan = fdc.fdc_plan_decode(lay, 0, [S] * B, pp)
    ws = torch.empty(plan.workspace_bytes() + 256, dtype=torch.uint8, device=dev)
    off = (-ws.data_ptr()) % 256
    ws = ws[off:off + plan.workspace_bytes()]
    fdc.fdc_plan_upload(plan, ws)
    fn = lambda: fdc.fdc_latent_attn_decode(lay, plan, q_lat, kc, vc, 1.0 / math.sqrt(dh), o_lat, ws)
    fn()
    torch.cuda.synchronize()
    ev = HipEvents(2)
    tile_us = []
    for _ in range(iters):
        fdc.fdc_profile_decode_events(ev.ev[0], ev.ev[1])
        fn()
        torch.cuda.synchronize()
        tile_us.append(ev.ms(0, 1) * 1e3)
    ev.destroy()
    s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    s.record()
    for _ in range(iters):
        fn()
    e.record()
    torch.cuda.synchronize()
    call_us = s.elapsed_time(e) / iters * 1e3
    cache_bytes = float(B * S * 2 * sum(r) * 2)    # every cached element once, whatever the group size
    tile = sum(tile_us) / len(tile_us)
    return {"workload": "8 kv heads x 4 query heads, adaptive ranks %s, batch 64, context 8192" % r,
            "n_workers": pp.n_workers, "tiles": int(plan.export()["n_items"]),
            "tile_kernel_us": tile, "tile_kernel_GBps": cache_bytes / tile / 1e3,
            "frac_of_hbm_peak": cache_bytes / tile / 1e3 / HBM_PEAK_GBPS,
            "call_us": call_us, "call_GBps": cache_bytes / call_us / 1e3}


def run_single_layer_decode(fdc, gen, name, copies=4, iters=24):
    """One decode-attention layer of a single-layer configuration (uniform rank 64 at batch 8 x 4096, whose cache is
    exactly the size of the last-level cache; or one 131072-token sequence cut into >= 256 chunks per head), timed
    over `copies` rotating copies of the cache so that no launch finds its bytes in the last-level cache."""
    import torch
    dev = "cuda:0"
    wl = gen.CONFIGS[name]
    ranks = wl.ranks()
    H, B, S, dh = wl.n_heads, wl.batch, wl.context, wl.d_head
    lay = fdc.Layout(1, H, wl.d_model, dh, ranks, ranks, B, S, fdc.FDC_BF16)
    t = lay.tables()
    RK, RV = int(t["koff_r"][0, -1]), int(t["voff_r"][0, -1])
    gt = torch.Generator(device=dev).manual_seed(wl.seed + 3)
    bf = torch.bfloat16
    kcs, vcs = [], []
    for _ in range(copies):
        k = torch.empty(int(t["k_bytes"][0]) // 2, dtype=bf, device=dev)
        v = torch.empty(int(t["v_bytes"][0]) // 2, dtype=bf, device=dev)
        fill_latent(k, lay, t["koff_r"][0], ranks[0], B, S, wl.decay, gt)
        fill_latent(v, lay, t["voff_r"][0], ranks[0], B, S, wl.decay, gt)
        kcs.append(k), vcs.append(v)
    q_lat = torch.randn(B, RK, generator=gt, device=dev)
    o_lat = torch.empty(B, RV, device=dev)
    pp = fdc.fdc_plan_params_default()
    pp.n_workers, pp.min_split = fdc.fdc_suggest_workers(0), wl.min_split
    plan = fdc.fdc_plan_decode(lay, 0, [S] * B, pp)
    ws = torch.empty(plan.workspace_bytes() + 256, dtype=torch.uint8, device=dev)
    off = (-ws.data_ptr()) % 256
    ws = ws[off:off + plan.workspace_bytes()]
    fdc.fdc_plan_upload(plan, ws)
    scale = 1.0 / math.sqrt(dh)
    fn = lambda i: fdc.fdc_latent_attn_decode(lay, plan, q_lat, kcs[i % copies], vcs[i % copies], scale, o_lat, ws)
    for i in range(2 * copies):
        fn(i)
    torch.cuda.synchronize()
    ev = HipEvents(2 * iters)
    for i in range(iters):
        fdc.fdc_profile_decode_events(ev.ev[2 * i], ev.ev[2 * i + 1])
        fn(i)
    torch.cuda.synchronize()
    tile_us = [ev.ms(2 * i, 2 * i + 1) * 1e3 for i in range(iters)]
    ev.destroy()
    s_, e_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    s_.record()
    for i in range(iters):
        fn(i)
    e_.record()
    torch.cuda.synchronize()
    call_us = s_.elapsed_time(e_) * 1e3 / iters
    tab = plan.export()
    nbytes = float(decode_bytes(tab, ranks[0], ranks[0], [S] * B, RK, RV, B))
    per_unit = np.diff(tab["unit_item_ptr"])
    merge_bytes = float(sum(int(n) * (int(ranks[0][u % H]) + 2) * 4 for u, n in enumerate(per_unit) if n > 1))
    tile = float(np.mean(tile_us))
    return {"workload": "%s: %d heads, batch %d, context %d, min_split %d, %d rotating cache copies of %.0f MB" %
                        (name, H, B, S, wl.min_split, copies, (kcs[0].numel() + vcs[0].numel()) * 2 / 1e6),
            "n_workers": pp.n_workers, "tiles": int(tab["n_items"]), "tiles_per_unit_min_max": [int(per_unit.min()), int(per_unit.max())],
            "algorithmic_bytes": nbytes,
            "tile_kernel_us": tile, "tile_kernel_us_min": float(np.min(tile_us)), "tile_kernel_GBps": nbytes / tile / 1e3,
            "tile_kernel_frac_of_hbm_peak": nbytes / tile / 1e3 / HBM_PEAK_GBPS,
            "call_us": call_us, "call_GBps": (nbytes + merge_bytes) / call_us / 1e3,
            "call_frac_of_hbm_peak": (nbytes + merge_bytes) / call_us / 1e3 / HBM_PEAK_GBPS,
            "merge_and_launch_us": call_us - tile}


def run_fp8_decode_workload(fdc, gen, wl, iters=12, fp4=False):
    """Decode attention of layer 0 of the decode workload with the cache stored as E4M3 codes
    (FDC_FP8 layout): the same tokens and ranks at half the cache bytes; or as E2M1 codes (FDC_FP4 layout,
    two codes per byte): a quarter of the bytes."""
    import torch
    dev = "cuda:0"
    ranks = wl.ranks()[:1]
    H, B, S, dh = wl.n_heads, wl.batch, wl.context, wl.d_head
    lay = fdc.Layout(1, H, wl.d_model, dh, ranks, ranks, B, S, fdc.FDC_FP4 if fp4 else fdc.FDC_FP8)
    t = lay.tables()
    RK = int(t["koff_r"][0, -1])
    gt = torch.Generator(device=dev).manual_seed(9)
    n = int(t["k_bytes"][0])
    copies = 4 if fp4 else 3   # rotate cache copies so that no launch finds its bytes in the last-level cache
    # random finite codes: any byte but the two NaN patterns (every byte is a pair of finite E2M1 codes)
    mk = (lambda: torch.randint(0, 256, (n,), generator=gt, device=dev, dtype=torch.uint8)) if fp4 else \
        (lambda: torch.randint(0, 0x7F, (n,), generator=gt, device=dev, dtype=torch.uint8) |
         (torch.randint(0, 2, (n,), generator=gt, device=dev, dtype=torch.uint8) << 7))
    kcs, vcs = [mk() for _ in range(copies)], [mk() for _ in range(copies)]
    q_lat = torch.randn(B, RK, generator=gt, device=dev) * 0.01
    o_lat = torch.empty(B, RK, device=dev)
    pp = fdc.fdc_plan_params_default()
    pp.n_workers, pp.min_split = fdc.fdc_suggest_workers(4 if fp4 else 3), wl.min_split
    plan = fdc.fdc_plan_decode(lay, 0, [S] * B, pp)
    ws = torch.empty(plan.workspace_bytes() + 256, dtype=torch.uint8, device=dev)
    off = (-ws.data_ptr()) % 256
    ws = ws[off:off + plan.workspace_bytes()]
    fdc.fdc_plan_upload(plan, ws)
    fn = lambda i: fdc.fdc_latent_attn_decode(lay, plan, q_lat, kcs[i % copies], vcs[i % copies], 1.0 / math.sqrt(dh), o_lat, ws)
    for i in range(copies):
        fn(i)
    torch.cuda.synchronize()
    ev = HipEvents(2 * iters)
    for i in range(iters):
        fdc.fdc_profile_decode_events(ev.ev[2 * i], ev.ev[2 * i + 1])
        fn(i)
    torch.cuda.synchronize()
    tile = float(np.mean([ev.ms(2 * i, 2 * i + 1) for i in range(iters)])) * 1e3
    ev.destroy()
    cache_bytes = float(B * S * 2 * int(np.sum(ranks[0]))) * (0.5 if fp4 else 1.0)    # one byte (half a byte) per cached element
    return {"workload": "layer 0 of %s with an %s" % (wl.name, "E2M1 cache (half a byte per element)" if fp4 else
                                                      "E4M3 cache (one byte per element)"),
            "n_workers": pp.n_workers, "tiles": int(plan.export()["n_items"]),
            "tile_kernel_us": tile, "tile_kernel_GBps": cache_bytes / tile / 1e3,
            "frac_of_hbm_peak": cache_bytes / tile / 1e3 / HBM_PEAK_GBPS,
            "cached_tokens_per_us": B * S / tile}


def run_device_planner(fdc, gen, wl, iters=5):
    """Re-planning every layer of the decode workload on the GPU (one workgroup per layer, one launch)
    beside the host planner on one core: what a re-plan costs once per `granule` decode steps."""
    import torch
    dev = "cuda:0"
    ranks = wl.ranks()
    L, H, B, S = wl.n_layers, wl.n_heads, wl.batch, wl.context
    lay = fdc.Layout(L, H, wl.d_model, wl.d_head, ranks, ranks, B, S, fdc.FDC_BF16)
    pp = fdc.fdc_plan_params_default()
    pp.n_workers, pp.min_split, pp.granule = fdc.fdc_suggest_workers(0), wl.min_split, wl.granule
    plans, wss = [], []
    for l in range(L):
        plan = fdc.fdc_plan_decode_device(lay, l, B, 0, pp)
        ws = torch.empty(plan.workspace_bytes() + 256, dtype=torch.uint8, device=dev)
        off = (-ws.data_ptr()) % 256
        ws = ws[off:off + plan.workspace_bytes()]
        fdc.fdc_plan_upload(plan, ws)
        plans.append(plan), wss.append(ws)
    seq = torch.full((B,), S, dtype=torch.int32, device=dev)
    per_launch = 32
    groups = [(plans[i:i + per_launch], wss[i:i + per_launch]) for i in range(0, L, per_launch)]
    run = lambda: [fdc.fdc_plan_decode_run(p, w, seq) for p, w in groups]
    run()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        run()
    e1.record()
    torch.cuda.synchronize()
    dev_ms = e0.elapsed_time(e1) / iters
    fdc.fdc_plan_download(plans[0], wss[0])
    t0 = time.perf_counter()
    host = [fdc.fdc_plan_decode(lay, l, [S] * B, pp) for l in range(L)]
    host_ms = (time.perf_counter() - t0) * 1e3
    same = all(np.array_equal(plans[0].export()[k], host[0].export()[k])
               for k in ("item_b", "item_h", "item_lo", "item_hi", "worker_ptr", "worker_items", "unit_item_ptr"))
    return {"workload": "%s: all %d layers re-planned" % (wl.name, L), "n_workers": pp.n_workers,
            "device_ms_all_layers": dev_ms, "host_one_core_ms_all_layers": host_ms,
            "tiles_layer0": int(plans[0].export()["n_items"]), "layer0_tables_equal_host": bool(same),
            "workspace_MB_per_layer": plans[0].workspace_bytes() / 1e6}


def run_serving_loop(fdc, gen, wl, steps=64):
    """A decode loop as a serving system runs it, with nothing on the host between steps: the lengths live in
    device memory and grow by one token per step, every layer appends its K'/V' rows at the sequence's end
    (fdc_project_and_absorb_query), attends at the actual lengths on a plan made for the lengths rounded up
    to the granule (fdc_latent_attn_decode_at), and all layers are re-planned on the GPU
    (fdc_plan_decode_run) whenever a sequence enters a new granule: once in the steps timed here (one granule's
    worth), which end at the workload's context."""
    import torch
    dev = "cuda:0"
    ranks = wl.ranks()
    L, H, B, S, d, dh = wl.n_layers, wl.n_heads, wl.batch, wl.context, wl.d_model, wl.d_head
    lay = fdc.Layout(L, H, d, dh, ranks, ranks, B, S, fdc.FDC_BF16)
    t = lay.tables()
    gt = torch.Generator(device=dev).manual_seed(wl.seed + 1)
    bf = torch.bfloat16
    pp = fdc.fdc_plan_params_default()
    pp.n_workers, pp.min_split, pp.granule = fdc.fdc_suggest_workers(0), wl.min_split, wl.granule
    G = pp.granule
    kc, vc, A_cat_t, Bk, Mt, plans, wss = [], [], [], [], [], [], []
    for l in range(L):
        RK, RV = int(t["koff_r"][l, -1]), int(t["voff_r"][l, -1])
        # cache contents: any finite values do (the kernels' speed does not depend on them); cheap to make
        kc.append((torch.randn(int(t["k_bytes"][l]) // 2, generator=gt, device=dev) * 0.3).to(bf))
        vc.append((torch.randn(int(t["v_bytes"][l]) // 2, generator=gt, device=dev) * 0.3).to(bf))
        A_cat_t.append((torch.randn(RK + RV, d, generator=gt, device=dev) / math.sqrt(d)).to(bf))
        Bk.append((torch.randn(RK, dh, generator=gt, device=dev) / math.sqrt(dh)).to(bf))
        Mt.append((torch.randn(d, RV, generator=gt, device=dev) / math.sqrt(RV)).to(bf))
        plan = fdc.fdc_plan_decode_device(lay, l, B, 0, pp)
        ws = torch.empty(plan.workspace_bytes() + 256, dtype=torch.uint8, device=dev)
        off = (-ws.data_ptr()) % 256
        ws = ws[off:off + plan.workspace_bytes()]
        fdc.fdc_plan_upload(plan, ws)
        plans.append(plan), wss.append(ws)
    x = torch.randn(B, d, generator=gt, device=dev).to(bf)
    q = torch.randn(B, H, dh, generator=gt, device=dev).to(bf)
    tb = torch.arange(B, dtype=torch.int32, device=dev)
    RKmax, RVmax = int(t["koff_r"][:, -1].max()), int(t["voff_r"][:, -1].max())
    q_lat = torch.empty(B * RKmax, dtype=torch.float32, device=dev)
    o_lat = torch.empty(B * RVmax, dtype=torch.float32, device=dev)
    y = torch.empty(B, d, dtype=bf, device=dev)
    scale = 1.0 / math.sqrt(dh)
    start = S - steps
    assert start % G == 0 and start > 0, "the loop starts on a granule boundary"
    pos = torch.full((B,), start, dtype=torch.int32, device=dev)       # tokens already cached = position of the new one
    lens = torch.empty_like(pos)                                       # tokens attended to in this step
    planned = torch.empty_like(pos)
    groups = [(plans[i:i + 32], wss[i:i + 32]) for i in range(0, L, 32)]

    def step(i):
        torch.add(pos, 1, out=lens)
        if i % G == 0:                                                 # the host knows the step count, not the lengths
            torch.div(lens + (G - 1), G, rounding_mode="floor", out=planned)
            planned.mul_(G)
            for p, w in groups:
                fdc.fdc_plan_decode_run(p, w, planned)
        for l in range(L):
            fdc.fdc_project_and_absorb_query(lay, l, x, tb, pos, A_cat_t[l], kc[l], vc[l], q, Bk[l], q_lat, fdc.FDC_F32)
            fdc.fdc_latent_attn_decode_at(lay, plans[l], lens, q_lat, kc[l], vc[l], scale, o_lat, wss[l])
            fdc.fdc_absorb_output(lay, l, fdc.FDC_APPLY, None, None, Mt[l], o_lat, fdc.FDC_F32, B, y, fdc.FDC_BF16)
        pos.add_(1)

    step(0)                     # warm-up (plans once, appends one token)
    pos.fill_(start)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    assert int(pos[0].item()) == S and bool(torch.isfinite(y.float()).all().item())
    return {"workload": "%s: %d steps from context %d to %d, appends and lengths on the device, one re-plan of all "
                        "%d layers by the GPU planner inside the timed steps" % (wl.name, steps, start, S, L),
            "ms_per_step": ms, "n_workers": pp.n_workers}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="c3_adaptive_decode",
                    choices=["c2_uniform_decode", "c3_adaptive_decode", "c4_long_decode"])
    ap.add_argument("--workers", type=int, default=0, help="decode workers (0 = resident wavefronts of the device)")
    ap.add_argument("--granule", type=int, default=0)
    ap.add_argument("--layers", type=int, default=0, help="use only the first N layers (own experiments)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (known HBM traffic) for scaling rocprofv3 counters")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-prefill", action="store_true")
    ap.add_argument("--no-gqa", action="store_true")
    ap.add_argument("--no-fp8", action="store_true")
    ap.add_argument("--no-device-planner", action="store_true")
    ap.add_argument("--no-serving-loop", action="store_true")
    ap.add_argument("--no-single-layer", action="store_true", help="skip the uniform-rank and long-context side objects")
    ap.add_argument("--only-single-layer", default=None, choices=["c2_uniform_decode", "c4_long_decode"],
                    help="run just this single-layer side measurement and print its object (for counter runs)")
    ap.add_argument("--oracle-legs", default=None, help=argparse.SUPPRESS)   # child process of cpu_baseline
    args = ap.parse_args()
    if args.oracle_legs:
        print(json.dumps(oracle_legs(json.loads(args.oracle_legs))))
        return
    if args.gpus != 1:
        print("bench.py: this build measures one GPU; --gpus N with N > 1 is not supported "
              "(no collective is part of this path)", file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    import paper_2408_04107_amd as fdc
    from workloads import generators as gen

    wl = gen.CONFIGS[args.workload]
    if args.layers:
        import copy
        wl = copy.copy(wl)
        wl._ranks = wl.ranks()[:args.layers].copy()
        wl.n_layers = args.layers
    if args.pmc_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0").fill_(3)
        dst = torch.empty_like(src)
        dst.copy_(src)          # one elementwise copy kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    if args.only_single_layer:
        print(json.dumps({"side": args.only_single_layer,
                          **run_single_layer_decode(fdc, gen, args.only_single_layer, iters=max(args.steps, 4))}))
        return
    res, state = run_decode_workload(fdc, gen, wl, args.steps, args.warmup, args)
    line = {
        "metric": "latent-KV decode step: achieved HBM GB/s (algorithmic bytes of the whole step / step time)",
        "value": res["value"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "layers": wl.n_layers, "heads": wl.n_heads, "d_head": wl.d_head,
                   "batch": wl.batch, "context": wl.context, "ranks": "adaptive 16..128, P(r)~1/r"
                   if wl.rank_seed is not None else "uniform 64", "kv_dtype": "bf16", "accumulate": "fp32",
                   "planner_granule": args.granule or wl.granule},
        "pct_of_hbm_peak": 100.0 * res["value"] / HBM_PEAK_GBPS,
        "roofline": res["roofline"], "decode_attn": res["decode_attn"],
        "decode_other_calls_layer0": res["decode_other_calls_layer0"],
        "step_algorithmic_bytes": res["step_algorithmic_bytes"],
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(state)
    del state
    torch.cuda.empty_cache()
    # side measurements of the other rows: a failure in one of them is reported in its place and does
    # not take the headline line with it
    def side(name, fn):
        try:
            torch.cuda.empty_cache()
            line[name] = fn()
        except Exception as exc:   # noqa: BLE001
            line[name] = {"error": f"{type(exc).__name__}: {exc}"}
            print(f"bench.py: {name} failed: {exc}", file=sys.stderr)
    if not args.no_single_layer:
        side("c2_uniform_decode", lambda: run_single_layer_decode(fdc, gen, "c2_uniform_decode"))
        side("c4_long_decode", lambda: run_single_layer_decode(fdc, gen, "c4_long_decode"))
    if not args.no_prefill:
        side("prefill", lambda: run_prefill_workload(fdc, gen))
    if not args.no_gqa:
        side("gqa_decode", lambda: run_gqa_decode_workload(fdc, gen))
    if not args.no_fp8:
        side("fp8_decode", lambda: run_fp8_decode_workload(fdc, gen, wl))
        side("fp4_decode", lambda: run_fp8_decode_workload(fdc, gen, wl, fp4=True))
    if not args.no_device_planner:
        side("device_planner", lambda: run_device_planner(fdc, gen, wl))
    if not args.no_serving_loop:
        side("serving_loop", lambda: run_serving_loop(fdc, gen, wl, steps=wl.granule))
    print(json.dumps(line))


if __name__ == "__main__":
    main()
