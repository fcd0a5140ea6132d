"""End-to-end bf16 chain parity at a scaled-down prefill configuration (one sequence of 512 tokens,
d_model 1024, 8 heads of width 128, adaptive ranks, factors from the oracle's truncated SVD):

  decode   x -> fdc_project_latent_kv -> fdc_absorb_query -> fdc_latent_attn_decode -> fold / apply -> y
  prefill  x -> fdc_project_latent_kv -> fdc_absorb_query -> fdc_latent_attn_prefill (causal) -> apply -> y

The oracle computes the same chain in float64 from the RAW inputs the library was given (the bf16
bits of x, A, B_k, B_v, W_o and q), with no rounding between the calls, so the error measured here is
the accumulated error of every bf16 store and bf16 matrix-core operand on the way: K'/V' rows in the
cache, q' (prefill), the softmax weights (prefill), o' (prefill store, decode operand), the folded
M and y itself.

Tolerance. One rounding to bf16 has relative error uniform in +-2^-9, rms 2^-9/sqrt(3) = 1.13e-3, and
independent roundings add in quadrature. Roundings of stored results (V', o', M, y) act on the output
directly: 4 of them give 2.3e-3. Roundings of score operands (K', and q' in prefill) act through
the softmax: a score error ds changes the output by about ds relative, and ds is about 1.13e-3 times
the size of the score's terms per rounding (the scores of this workload stay below 2): 1 to 1.5e-3.
Together about 3e-3 (observed: 3.2e-3 decode, 3.6e-3 prefill). The chain bar is the north-star
relative L2 of 5e-3 with max-abs 2e-2; a single query row may reach twice that.
"""
import math
import sys

import numpy as np
import pytest
import torch

import paper_2408_04107_amd as fdc
from oracle import attention as oa
from oracle.factors import truncated_svd_factors
from tests.gpu_util import Cache, assert_close, workspace_for
from workloads import generators as gen

pytestmark = pytest.mark.gpu

BF = torch.bfloat16
H, D, D_H, S = 8, 1024, 128, 512


def say(msg):
    print(f"[chain-parity] {msg}", flush=True)
    sys.stdout.flush()


def dev(a, dt):
    return torch.from_numpy(np.ascontiguousarray(a)).to(dt).cuda().contiguous()


def f64(t):
    return t.to(torch.float64).cpu().numpy()


def make_inputs(seed):
    g = gen.make_rng(seed)
    r = gen.adaptive_ranks(1, H, seed)[0].tolist()
    Wk = [gen.planted_weight(D, D_H, 32.0, g).W for _ in range(H)]
    Wv = [gen.planted_weight(D, D_H, 32.0, g).W for _ in range(H)]
    Wq = [g.standard_normal((D, D_H)) / math.sqrt(D) for _ in range(H)]
    Wo = g.standard_normal((H * D_H, D)) / math.sqrt(H * D_H)
    x = gen.hidden_states(S, D, g)
    Ak, Bk, Av, Bv = [], [], [], []
    for h in range(H):
        a, b, _ = truncated_svd_factors(Wk[h], r[h])
        Ak.append(a), Bk.append(b)
        a, b, _ = truncated_svd_factors(Wv[h], r[h])
        Av.append(a), Bv.append(b)
    t = dict(r=r)
    t["x"] = dev(x, BF)
    t["A_cat_t"] = dev(np.concatenate([a.T for a in Ak] + [a.T for a in Av], axis=0), BF)
    t["Bk"], t["Bv"] = dev(np.concatenate(Bk, axis=0), BF), dev(np.concatenate(Bv, axis=0), BF)
    t["Wo_t"] = dev(Wo.T, BF)
    # the model's own query projection is outside the library: q is an input, rounded once to bf16
    xq = f64(t["x"])
    t["q"] = dev(np.stack([xq @ Wq[h] for h in range(H)], axis=1), BF)       # [S, H, d_h]
    return t


def oracle_chain(t, rows):
    """float64 chain from the raw inputs for the query rows `rows` (causal: row i sees keys 0..i)."""
    r = t["r"]
    off = np.concatenate([[0], np.cumsum(r)])
    RK = int(off[-1])
    x64, A64 = f64(t["x"]), f64(t["A_cat_t"])
    K_lat = oa.project_latent_kv(x64, [A64[off[h]:off[h + 1]].T for h in range(H)])
    V_lat = oa.project_latent_kv(x64, [A64[RK + off[h]:RK + off[h + 1]].T for h in range(H)])
    ql = oa.absorb_query(f64(t["q"]), [f64(t["Bk"])[off[h]:off[h + 1]] for h in range(H)])
    scale = 1 / math.sqrt(D_H)
    ol = [np.stack([oa.latent_attn_decode(ql[h][i], K_lat[h][:i + 1], V_lat[h][:i + 1], scale) for i in rows])
          for h in range(H)]
    M = oa.fold_output([f64(t["Bv"])[off[h]:off[h + 1]] for h in range(H)], f64(t["Wo_t"]).T, D_H)
    smax = max(float(np.max(np.abs(scale * ql[h][rows] @ K_lat[h].T))) for h in range(H))
    return oa.apply_output(ol, M), np.concatenate(ol, axis=1), smax


def library_front(t):
    r = t["r"]
    lay = fdc.Layout(1, H, D, D_H, [r], [r], 1, S, fdc.FDC_BF16)
    cache = Cache(lay)
    tb = torch.zeros(S, dtype=torch.int32, device="cuda:0")
    tp = torch.arange(S, dtype=torch.int32, device="cuda:0")
    fdc.fdc_project_latent_kv(lay, 0, t["x"], tb, tp, t["A_cat_t"], cache.k, cache.v)
    Mt = torch.empty(D, cache.RV, dtype=BF, device="cuda:0")
    fdc.fdc_absorb_output(lay, 0, fdc.FDC_FOLD, t["Bv"], t["Wo_t"], Mt, None, 0, 0, None, 0)
    return lay, cache, Mt


@pytest.mark.parametrize("seed", [0, 1])
def test_decode_chain_bf16_scaled_prefill_config(seed):
    say(f"decode chain, seed {seed}")
    t = make_inputs(seed)
    say(f"  ranks {t['r']}")
    lay, cache, Mt = library_front(t)
    q_last = t["q"][S - 1:S].contiguous()
    q_lat = torch.empty(1, cache.RK, dtype=torch.float32, device="cuda:0")
    fdc.fdc_absorb_query(lay, 0, q_last, t["Bk"], q_lat, fdc.FDC_F32)
    pp = fdc.fdc_plan_params_default()
    pp.n_workers = 256
    plan = fdc.fdc_plan_decode(lay, 0, [S], pp)
    ws = workspace_for(plan)
    o_lat = torch.empty(1, cache.RV, dtype=torch.float32, device="cuda:0")
    fdc.fdc_latent_attn_decode(lay, plan, q_lat, cache.k, cache.v, 1 / math.sqrt(D_H), o_lat, ws)
    y = torch.empty(1, D, dtype=BF, device="cuda:0")
    fdc.fdc_absorb_output(lay, 0, fdc.FDC_APPLY, None, None, Mt, o_lat, fdc.FDC_F32, 1, y, fdc.FDC_BF16)
    torch.cuda.synchronize()
    y_ref, o_ref, smax = oracle_chain(t, [S - 1])
    ma, rl = assert_close(f64(o_lat), o_ref, "decode chain o'")
    say(f"  o' max_abs={ma:.2e} rel_l2={rl:.2e}  (largest |score| {smax:.2f})")
    ma, rl = assert_close(f64(y), y_ref, "decode chain y")
    say(f"  y  max_abs={ma:.2e} rel_l2={rl:.2e}")


@pytest.mark.parametrize("seed", [0, 1])
def test_prefill_chain_bf16_scaled_prefill_config(seed):
    say(f"prefill chain, seed {seed}")
    t = make_inputs(seed)
    lay, cache, Mt = library_front(t)
    q_lat = torch.empty(S, cache.RK, dtype=BF, device="cuda:0")
    fdc.fdc_absorb_query(lay, 0, t["q"], t["Bk"], q_lat, fdc.FDC_BF16)
    pp = fdc.fdc_plan_params_default()
    pp.n_workers, pp.cost_mode = 64, 1
    plan = fdc.fdc_plan_prefill(lay, 0, [S], [S], pp)
    ws = workspace_for(plan)
    o_lat = torch.empty(S, cache.RV, dtype=BF, device="cuda:0")
    fdc.fdc_latent_attn_prefill(lay, plan, q_lat, cache.k, cache.v, 1 / math.sqrt(D_H), True, o_lat, ws)
    y = torch.empty(S, D, dtype=BF, device="cuda:0")
    fdc.fdc_absorb_output(lay, 0, fdc.FDC_APPLY, None, None, Mt, o_lat, fdc.FDC_BF16, S, y, fdc.FDC_BF16)
    torch.cuda.synchronize()
    rows = list(range(S))
    y_ref, o_ref, smax = oracle_chain(t, rows)
    ma, rl = assert_close(f64(o_lat), o_ref, "prefill chain o'")
    say(f"  o' max_abs={ma:.2e} rel_l2={rl:.2e}  (largest |score| {smax:.2f})")
    ma, rl = assert_close(f64(y), y_ref, "prefill chain y")
    say(f"  y  max_abs={ma:.2e} rel_l2={rl:.2e}")
    # per-row bar as well: no single token may hide behind the others (first rows see few keys)
    err = np.linalg.norm(f64(y) - y_ref, axis=1) / np.linalg.norm(y_ref, axis=1)
    say(f"  worst row rel_l2={err.max():.2e} (row {int(err.argmax())})")
    assert err.max() <= 2 * 5e-3
