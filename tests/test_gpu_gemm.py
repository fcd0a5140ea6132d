"""GPU parity of the projection-type calls (fdc_project_latent_kv, fdc_absorb_query,
fdc_absorb_output) against the float64 oracle on identical stored inputs, and of the whole decode
chain at the config-1 shape in fp32.
"""
import math
import sys

import numpy as np
import pytest
import torch

import paper_2408_04107_amd as fdc
from oracle import attention as oa
from oracle.factors import truncated_svd_factors
from tests.gpu_util import Cache, assert_close, torch_dtype, workspace_for
from workloads import generators as gen

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[gemm-parity] {msg}", flush=True)
    sys.stdout.flush()


def dev(a: np.ndarray, dtype):
    return torch.from_numpy(np.ascontiguousarray(a)).to(dtype).cuda().contiguous()


def f64(t: torch.Tensor) -> np.ndarray:
    return t.to(torch.float64).cpu().numpy()


CASES = [
    # H, d_model, d_head, rk, rv, T
    (3, 64, 32, [16, 32, 16], [32, 16, 16], 5),
    (8, 512, 128, [16, 32, 48, 64, 80, 96, 112, 128], [128, 16, 48, 64, 32, 112, 96, 80], 300),
    (4, 1000, 64, [64, 16, 48, 32], [16, 64, 64, 48], 129),
    # few rows: the weight-streaming kernel (decode batches), 1 to 4 row tiles
    (8, 512, 128, [16, 32, 48, 64, 80, 96, 112, 128], [128, 16, 48, 64, 32, 112, 96, 80], 16),
    (4, 1000, 64, [64, 16, 48, 32], [16, 64, 64, 48], 64),
    (3, 264, 32, [16, 32, 16], [32, 16, 16], 33),
    (32, 4096, 128, [64] * 32, [64] * 32, 48),
    # at most 16 rows: the single-row-tile weight stream. K = 4096 (eight waves), K beyond one pass of
    # eight 512-wide chunks, a ragged last column tile of the output projection, and a wide V' (K = 4096 fp32 rows)
    (32, 4096, 128, [64] * 32, [64] * 32, 16),
    (4, 4616, 64, [64, 16, 48, 32], [16, 64, 64, 48], 9),
    (4, 1000, 64, [64, 16, 48, 32], [16, 64, 64, 48], 7),
    (32, 512, 128, [16] * 32, [128] * 32, 12),
]


@pytest.mark.parametrize("dtype", [fdc.FDC_BF16, fdc.FDC_F32])
@pytest.mark.parametrize("case", range(len(CASES)))
def test_project_latent_kv(case, dtype):
    H, d, d_h, rk, rv, T = CASES[case]
    say(f"project case {case} dtype {dtype}: H={H} d={d} T={T}")
    B, S = 3, 200
    lay = fdc.Layout(1, H, d, d_h, [rk], [rv], B, S, dtype)
    cache = Cache(lay)
    td = torch_dtype(dtype)
    g = gen.make_rng(case)
    x = dev(gen.hidden_states(T, d, g), td)
    A_cat_t = dev(g.standard_normal((cache.RK + cache.RV, d)) / math.sqrt(d), td)
    # distinct (sequence, position) slots, in random order
    slots = g.permutation(B * S)[:T]
    tb, tp = dev(slots // S, torch.int32), dev(slots % S, torch.int32)
    fdc.fdc_project_latent_kv(lay, 0, x, tb, tp, A_cat_t, cache.k, cache.v)
    torch.cuda.synchronize()
    x64, A64 = f64(x), f64(A_cat_t)
    kr, vr = cache.t["koff_r"][0], cache.t["voff_r"][0]
    K_ref = oa.project_latent_kv(x64, [A64[kr[h]:kr[h + 1]].T for h in range(H)])
    V_ref = oa.project_latent_kv(x64, [A64[cache.RK + vr[h]:cache.RK + vr[h + 1]].T for h in range(H)])
    got, ref = [], []
    for h in range(H):
        for side, R in (("k", K_ref), ("v", V_ref)):
            for b in range(B):
                u = f64(cache.unit(side, b, h))
                rows = np.nonzero(slots // S == b)[0]
                got.append(u[slots[rows] % S].ravel()), ref.append(R[h][rows].ravel())
                # untouched positions stay zero
                mask = np.ones(S, bool)
                mask[slots[rows] % S] = False
                assert not u[mask].any()
    tol = 5e-6 if dtype == fdc.FDC_F32 else 5e-3
    ma, rl = assert_close(np.concatenate(got), np.concatenate(ref), "latent rows", rel_l2_tol=tol)
    say(f"  max_abs={ma:.2e} rel_l2={rl:.2e}")


@pytest.mark.parametrize("dtype,q_lat_dtype", [(fdc.FDC_BF16, fdc.FDC_F32), (fdc.FDC_BF16, fdc.FDC_BF16),
                                               (fdc.FDC_F32, fdc.FDC_F32)])
@pytest.mark.parametrize("case", range(len(CASES)))
def test_absorb_query(case, dtype, q_lat_dtype):
    H, d, d_h, rk, rv, T = CASES[case]
    say(f"absorb_query case {case} dtype {dtype}->{q_lat_dtype}")
    lay = fdc.Layout(1, H, d, d_h, [rk], [rv], 1, 8, dtype)
    td = torch_dtype(dtype)
    g = gen.make_rng(10 + case)
    RK = sum(rk)
    q = dev(g.standard_normal((T, H, d_h)), td)
    Bk = dev(g.standard_normal((RK, d_h)) / math.sqrt(d_h), td)
    q_lat = torch.full((T, RK), float("nan"), dtype=torch_dtype(q_lat_dtype), device="cuda:0")
    fdc.fdc_absorb_query(lay, 0, q, Bk, q_lat, q_lat_dtype)
    torch.cuda.synchronize()
    off = np.concatenate([[0], np.cumsum(rk)])
    ref = oa.absorb_query(f64(q), [f64(Bk)[off[h]:off[h + 1]] for h in range(H)])
    tol = 5e-6 if q_lat_dtype == fdc.FDC_F32 else 5e-3
    ma, rl = assert_close(f64(q_lat), np.concatenate(ref, axis=1), "q_lat", rel_l2_tol=tol)
    say(f"  max_abs={ma:.2e} rel_l2={rl:.2e}")


@pytest.mark.parametrize("q_per_kv", [1, 4])
@pytest.mark.parametrize("q_lat_dtype", [fdc.FDC_F32, fdc.FDC_BF16])
@pytest.mark.parametrize("case", range(len(CASES)))
def test_project_and_absorb_query_equals_the_two_calls(case, q_lat_dtype, q_per_kv):
    """The one-launch form (T <= 16) and its two-call fallback (T > 16) write exactly what
    fdc_project_latent_kv and fdc_absorb_query write; those two are checked against the oracle above."""
    H, d, d_h, rk, rv, T = CASES[case]
    if H * q_per_kv > 128:
        pytest.skip("more query heads than the library supports")
    say(f"project_and_absorb_query case {case}: H={H}x{q_per_kv} d={d} T={T} q_lat {q_lat_dtype}")
    B, S = 3, 200
    lay = fdc.Layout(1, H, d, d_h, [rk], [rv], B, S, fdc.FDC_BF16, q_per_kv=q_per_kv)
    two, one = Cache(lay), Cache(lay)
    g = gen.make_rng(200 + case)
    x = dev(gen.hidden_states(T, d, g), torch.bfloat16)
    A_cat_t = dev(g.standard_normal((two.RK + two.RV, d)) / math.sqrt(d), torch.bfloat16)
    q = dev(g.standard_normal((T, H * q_per_kv, d_h)), torch.bfloat16)
    Bk = dev(g.standard_normal((two.RK, d_h)) / math.sqrt(d_h), torch.bfloat16)
    slots = g.permutation(B * S)[:T]
    tb, tp = dev(slots // S, torch.int32), dev(slots % S, torch.int32)
    qd = torch_dtype(q_lat_dtype)
    q_two = torch.full((T, q_per_kv * two.RK), float("nan"), dtype=qd, device="cuda:0")
    q_one = torch.full((T, q_per_kv * two.RK), float("nan"), dtype=qd, device="cuda:0")
    fdc.fdc_project_latent_kv(lay, 0, x, tb, tp, A_cat_t, two.k, two.v)
    fdc.fdc_absorb_query(lay, 0, q, Bk, q_two, q_lat_dtype)
    fdc.fdc_project_and_absorb_query(lay, 0, x, tb, tp, A_cat_t, one.k, one.v, q, Bk, q_one, q_lat_dtype)
    torch.cuda.synchronize()
    assert not torch.isnan(q_one.float()).any()
    assert torch.equal(one.k, two.k) and torch.equal(one.v, two.v)
    assert torch.equal(q_one, q_two)
    assert one.k.float().abs().sum() > 0 and one.v.float().abs().sum() > 0


@pytest.mark.parametrize("dtype,io", [(fdc.FDC_BF16, (fdc.FDC_F32, fdc.FDC_F32)), (fdc.FDC_BF16, (fdc.FDC_BF16, fdc.FDC_BF16)),
                                      (fdc.FDC_BF16, (fdc.FDC_F32, fdc.FDC_BF16)), (fdc.FDC_F32, (fdc.FDC_F32, fdc.FDC_F32))])
@pytest.mark.parametrize("case", range(len(CASES)))
def test_absorb_output_fold_and_apply(case, dtype, io):
    H, d, d_h, rk, rv, T = CASES[case]
    say(f"absorb_output case {case} dtype {dtype} io {io}")
    lay = fdc.Layout(1, H, d, d_h, [rk], [rv], 1, 8, dtype)
    td = torch_dtype(dtype)
    g = gen.make_rng(20 + case)
    RV = sum(rv)
    Bv = dev(g.standard_normal((RV, d_h)) / math.sqrt(d_h), td)
    Wo_t = dev(g.standard_normal((d, H * d_h)) / math.sqrt(H * d_h), td)
    Mt = torch.full((d, RV), float("nan"), dtype=td, device="cuda:0")
    fdc.fdc_absorb_output(lay, 0, fdc.FDC_FOLD, Bv, Wo_t, Mt, None, 0, 0, None, 0)
    torch.cuda.synchronize()
    off = np.concatenate([[0], np.cumsum(rv)])
    M_ref = oa.fold_output([f64(Bv)[off[h]:off[h + 1]] for h in range(H)], f64(Wo_t).T, d_h)
    tol = 5e-6 if dtype == fdc.FDC_F32 else 5e-3
    ma, rl = assert_close(f64(Mt).T, np.concatenate(M_ref, axis=0), "folded M", rel_l2_tol=tol)
    say(f"  fold  max_abs={ma:.2e} rel_l2={rl:.2e}")

    o_dt, y_dt = io
    o_lat = dev(g.standard_normal((T, RV)), torch_dtype(o_dt))
    y = torch.full((T, d), float("nan"), dtype=torch_dtype(y_dt), device="cuda:0")
    fdc.fdc_absorb_output(lay, 0, fdc.FDC_APPLY, None, None, Mt, o_lat, o_dt, T, y, y_dt)
    torch.cuda.synchronize()
    # apply is checked on the stored Mt (the oracle of this call), heads = column blocks of o_lat
    M_stored = f64(Mt).T
    o64 = f64(o_lat)                     # as passed: fp32 activations become bf16 MFMA operands inside the call
    y_ref = oa.apply_output([o64[:, off[h]:off[h + 1]] for h in range(H)],
                            [M_stored[off[h]:off[h + 1]] for h in range(H)])
    # bf16 layouts: operands (and a bf16 y) carry 2^-9 roundings, the spec bar; an fp32 layout is exact to fp32
    tol = 5e-6 if (dtype == fdc.FDC_F32) else 5e-3
    ma, rl = assert_close(f64(y), y_ref, "y", rel_l2_tol=tol)
    say(f"  apply max_abs={ma:.2e} rel_l2={rl:.2e}")


def test_zero_tokens_is_a_no_op():
    lay = fdc.Layout(1, 2, 64, 32, [[16, 32]], [[16, 16]], 1, 8, fdc.FDC_BF16)
    cache = Cache(lay)
    e = torch.empty(0, 64, dtype=torch.bfloat16, device="cuda:0")
    i = torch.empty(0, dtype=torch.int32, device="cuda:0")
    A = torch.zeros(80, 64, dtype=torch.bfloat16, device="cuda:0")
    fdc.fdc_project_latent_kv(lay, 0, e, i, i, A, cache.k, cache.v)
    torch.cuda.synchronize()


def test_full_chain_config1_fp32():
    """x -> latent cache -> absorbed query -> decode attention -> absorbed output, all in the library,
    against the oracle chain on the same fp32 inputs; the factors come from the oracle's SVD."""
    wl = gen.CONFIGS["c1_tiny_decode_f32"]
    say(f"full chain, config 1: {wl}")
    H, d, d_h, S = wl.n_heads, wl.d_model, wl.d_head, wl.context
    r = wl.ranks()[0].tolist()
    g = gen.make_rng(wl.seed)
    Wk = [gen.planted_weight(d, d_h, wl.decay, g).W for _ in range(H)]
    Wv = [gen.planted_weight(d, d_h, wl.decay, g).W for _ in range(H)]
    Wq = [g.standard_normal((d, d_h)) / math.sqrt(d) for _ in range(H)]
    Wo = g.standard_normal((H * d_h, d)) / math.sqrt(H * d_h)
    x = gen.hidden_states(S, d, g)
    Ak, Bk, Av, Bv = [], [], [], []
    for h in range(H):
        a, b, _ = truncated_svd_factors(Wk[h], r[h])
        Ak.append(a), Bk.append(b)
        a, b, _ = truncated_svd_factors(Wv[h], r[h])
        Av.append(a), Bv.append(b)
    f32 = torch.float32
    x_d = dev(x, f32)
    A_cat_t = dev(np.concatenate([a.T for a in Ak] + [a.T for a in Av], axis=0), f32)
    Bk_d, Bv_d = dev(np.concatenate(Bk, axis=0), f32), dev(np.concatenate(Bv, axis=0), f32)
    Wo_t = dev(Wo.T, f32)
    q = np.stack([x[-1:] @ Wq[h] for h in range(H)], axis=1)          # the last token's query, [1, H, d_h]
    q_d = dev(q, f32)

    lay = fdc.Layout(1, H, d, d_h, [r], [r], 1, S, fdc.FDC_F32)
    cache = Cache(lay)
    tb = torch.zeros(S, dtype=torch.int32, device="cuda:0")
    tp = torch.arange(S, dtype=torch.int32, device="cuda:0")
    fdc.fdc_project_latent_kv(lay, 0, x_d, tb, tp, A_cat_t, cache.k, cache.v)
    q_lat = torch.empty(1, cache.RK, dtype=f32, device="cuda:0")
    fdc.fdc_absorb_query(lay, 0, q_d, Bk_d, q_lat, fdc.FDC_F32)
    pp = fdc.fdc_plan_params_default()
    pp.n_workers = 64
    plan = fdc.fdc_plan_decode(lay, 0, [S], pp)
    ws = workspace_for(plan)
    o_lat = torch.empty(1, cache.RV, dtype=f32, device="cuda:0")
    fdc.fdc_latent_attn_decode(lay, plan, q_lat, cache.k, cache.v, 1 / math.sqrt(d_h), o_lat, ws)
    Mt = torch.empty(d, cache.RV, dtype=f32, device="cuda:0")
    fdc.fdc_absorb_output(lay, 0, fdc.FDC_FOLD, Bv_d, Wo_t, Mt, None, 0, 0, None, 0)
    y = torch.empty(1, d, dtype=f32, device="cuda:0")
    fdc.fdc_absorb_output(lay, 0, fdc.FDC_APPLY, None, None, Mt, o_lat, fdc.FDC_F32, 1, y, fdc.FDC_F32)
    torch.cuda.synchronize()

    # oracle chain on the fp32-rounded inputs the library saw
    x64, A64 = f64(x_d), f64(A_cat_t)
    RK = cache.RK
    off = np.concatenate([[0], np.cumsum(r)])
    K_lat = oa.project_latent_kv(x64, [A64[off[h]:off[h + 1]].T for h in range(H)])
    V_lat = oa.project_latent_kv(x64, [A64[RK + off[h]:RK + off[h + 1]].T for h in range(H)])
    ql = oa.absorb_query(f64(q_d), [f64(Bk_d)[off[h]:off[h + 1]] for h in range(H)])
    ol = [oa.latent_attn_decode(ql[h][0], K_lat[h], V_lat[h], 1 / math.sqrt(d_h))[None] for h in range(H)]
    M = oa.fold_output([f64(Bv_d)[off[h]:off[h + 1]] for h in range(H)], f64(Wo_t).T, d_h)
    y_ref = oa.apply_output(ol, M)
    ma, rl = assert_close(f64(y), y_ref, "chain output y", rel_l2_tol=1e-4)
    say(f"  chain max_abs={ma:.2e} rel_l2={rl:.2e}")
    ma, rl = assert_close(f64(o_lat), np.concatenate(ol, axis=1), "chain o_lat", rel_l2_tol=1e-4)
    say(f"  o_lat max_abs={ma:.2e} rel_l2={rl:.2e}")


def test_config5_size_projection_and_apply_sampled_rows():
    """The prefill-size products in the shape bench.py times (16384 tokens, d_model 4096, adaptive
    ranks: N = 3360 with a ragged last column tile, K = 1680 with a k tail): 256 sampled token rows,
    all columns, against the float64 oracle."""
    wl = gen.CONFIGS["c5_prefill"]
    r = wl.ranks()[0].tolist()
    H, B, S, d, d_h = wl.n_heads, wl.batch, wl.context, wl.d_model, wl.d_head
    T = B * S
    say(f"config 5 size projections: T={T} d={d} RK+RV={2 * sum(r)}")
    lay = fdc.Layout(1, H, d, d_h, [r], [r], B, S, fdc.FDC_BF16)
    cache = Cache(lay)
    bf = torch.bfloat16
    gt = torch.Generator(device="cuda:0").manual_seed(3)
    x = torch.randn(T, d, generator=gt, device="cuda:0").to(bf)
    A_cat_t = (torch.randn(cache.RK + cache.RV, d, generator=gt, device="cuda:0") / math.sqrt(d)).to(bf)
    tb = torch.arange(B, dtype=torch.int32, device="cuda:0").repeat_interleave(S)
    tp = torch.arange(S, dtype=torch.int32, device="cuda:0").repeat(B)
    fdc.fdc_project_latent_kv(lay, 0, x, tb, tp, A_cat_t, cache.k, cache.v)
    o_lat = torch.randn(T, cache.RV, generator=gt, device="cuda:0").to(bf)
    Mt = (torch.randn(d, cache.RV, generator=gt, device="cuda:0") / math.sqrt(cache.RV)).to(bf)
    y = torch.full((T, d), float("nan"), dtype=bf, device="cuda:0")
    fdc.fdc_absorb_output(lay, 0, fdc.FDC_APPLY, None, None, Mt, o_lat, fdc.FDC_BF16, T, y, fdc.FDC_BF16)
    torch.cuda.synchronize()
    g = gen.make_rng(5)
    rows = np.unique(np.concatenate([[0, 1, 255, 256, 257, S - 1, S, T - 257, T - 256, T - 1], g.integers(0, T, 246)]))
    rows_t = torch.from_numpy(rows).cuda()
    x64, A64 = f64(x[rows_t]), f64(A_cat_t)
    kr, vr = cache.t["koff_r"][0], cache.t["voff_r"][0]
    got, ref = [], []
    for h in range(H):
        Kh = oa.project_latent_kv(x64, [A64[kr[h]:kr[h + 1]].T])[0]
        Vh = oa.project_latent_kv(x64, [A64[cache.RK + vr[h]:cache.RK + vr[h + 1]].T])[0]
        for b in range(B):
            sel = np.nonzero(rows // S == b)[0]
            pos = torch.from_numpy(rows[sel] % S).cuda()
            got.append(f64(cache.unit("k", b, h)[pos]).ravel()), ref.append(Kh[sel].ravel())
            got.append(f64(cache.unit("v", b, h)[pos]).ravel()), ref.append(Vh[sel].ravel())
    ma, rl = assert_close(np.concatenate(got), np.concatenate(ref), "config 5 latent rows")
    say(f"  project max_abs={ma:.2e} rel_l2={rl:.2e}")
    y_ref = f64(o_lat[rows_t]) @ f64(Mt).T
    ma, rl = assert_close(f64(y[rows_t]), y_ref, "config 5 y rows")
    say(f"  apply max_abs={ma:.2e} rel_l2={rl:.2e}")
    assert torch.isfinite(y.float()).all().item()


def test_project_and_absorb_query_with_values_only():
    """k_cache = NULL (post-RoPE path: only V' comes from the projection): same V' rows and queries as the two calls."""
    H, d, d_h, rk, rv, T = 4, 1000, 64, [64, 16, 48, 32], [16, 64, 64, 48], 11
    B, S = 2, 50
    lay = fdc.Layout(1, H, d, d_h, [rk], [rv], B, S, fdc.FDC_BF16)
    two, one = Cache(lay), Cache(lay)
    g = gen.make_rng(321)
    x = dev(gen.hidden_states(T, d, g), torch.bfloat16)
    A_v_t = dev(g.standard_normal((two.RV, d)) / math.sqrt(d), torch.bfloat16)
    q = dev(g.standard_normal((T, H, d_h)), torch.bfloat16)
    Bk = dev(g.standard_normal((two.RK, d_h)) / math.sqrt(d_h), torch.bfloat16)
    slots = g.permutation(B * S)[:T]
    tb, tp = dev(slots // S, torch.int32), dev(slots % S, torch.int32)
    q_two = torch.full((T, two.RK), float("nan"), dtype=torch.float32, device="cuda:0")
    q_one = torch.full_like(q_two, float("nan"))
    fdc.fdc_project_latent_kv(lay, 0, x, tb, tp, A_v_t, None, two.v)
    fdc.fdc_absorb_query(lay, 0, q, Bk, q_two, fdc.FDC_F32)
    fdc.fdc_project_and_absorb_query(lay, 0, x, tb, tp, A_v_t, None, one.v, q, Bk, q_one, fdc.FDC_F32)
    torch.cuda.synchronize()
    assert torch.equal(one.v, two.v) and one.v.float().abs().sum() > 0
    assert not one.k.any() and torch.equal(q_one, q_two)
