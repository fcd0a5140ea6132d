"""The cache writers take their destination (sequence, position) per row from device memory, which no
host check can see. Rows whose indices lie outside the cache must be skipped (nothing stored, every
other row written exactly as without them) and reported in the caller's status word.

Each case runs the writer twice: once with a few poisoned rows, once with only the good rows, into
caches that sit between guard bands. Both caches and both guard bands must be bit-identical."""
import math
import sys

import numpy as np
import pytest
import torch

import paper_2408_04107_amd as fdc
from oracle import rope as orp
from workloads import generators as gen

pytestmark = pytest.mark.gpu
BF = torch.bfloat16
GUARD = 1 << 16     # elements on either side of a cache buffer
FAULT_BATCH, FAULT_POS = 1, 2


def say(msg):
    print(f"[writer-faults] {msg}", flush=True)
    sys.stdout.flush()


class GuardedCache:
    def __init__(self, lay, dtype):
        t = lay.tables()
        es = {torch.bfloat16: 2, torch.float32: 4, torch.uint8: 1}[dtype]
        self.nk, self.nv = int(t["k_bytes"][0]) // es, int(t["v_bytes"][0]) // es
        fill = 77 if dtype == torch.uint8 else 3.0
        self.kbuf = torch.full((self.nk + 2 * GUARD,), fill, dtype=dtype, device="cuda:0")
        self.vbuf = torch.full((self.nv + 2 * GUARD,), fill, dtype=dtype, device="cuda:0")
        self.k = self.kbuf[GUARD:GUARD + self.nk]
        self.v = self.vbuf[GUARD:GUARD + self.nv]
        self.k.zero_(), self.v.zero_()

    def same_as(self, other):
        return torch.equal(self.kbuf, other.kbuf) and torch.equal(self.vbuf, other.vbuf)


def poisoned_indices(T, B, S, rng, bad_rows):
    """Distinct (sequence, position) slots for the good rows; bad rows get out-of-range values."""
    slots = rng.permutation(B * S)[:T]
    tb, tp = (slots // S).astype(np.int32), (slots % S).astype(np.int32)
    want = 0
    for i, r in enumerate(bad_rows):
        kind = i % 4
        if kind == 0:
            tb[r], want = -1, want | FAULT_BATCH
        elif kind == 1:
            tb[r], want = B, want | FAULT_BATCH                # one past the last sequence: just behind the buffer
        elif kind == 2:
            tp[r], want = S, want | FAULT_POS
        else:
            tp[r], want = -7, want | FAULT_POS
    return tb, tp, want


@pytest.mark.parametrize("T,dtype", [(5, fdc.FDC_BF16), (16, fdc.FDC_FP8), (40, fdc.FDC_BF16), (64, fdc.FDC_FP8),
                                     (300, fdc.FDC_BF16), (700, fdc.FDC_FP8), (33, fdc.FDC_F32)])
def test_projection_skips_and_flags_rows_outside_the_cache(T, dtype):
    say(f"projection T={T} layout dtype {dtype}")
    H, d, d_h, B, S = 3, 256, 64, 3, 400
    rk, rv = [16, 64, 32], [48, 16, 64]
    lay = fdc.Layout(1, H, d, d_h, [rk], [rv], B, S, dtype)
    act = torch.float32 if dtype == fdc.FDC_F32 else BF
    cdt = {fdc.FDC_BF16: BF, fdc.FDC_FP8: torch.uint8, fdc.FDC_F32: torch.float32}[dtype]
    rng = gen.make_rng(T)
    x = torch.from_numpy(gen.hidden_states(T, d, rng).astype(np.float32)).to(act).cuda()
    A = torch.from_numpy((rng.standard_normal((sum(rk) + sum(rv), d)) / math.sqrt(d)).astype(np.float32)).to(act).cuda()
    bad = sorted(rng.choice(T, size=min(4, T - 1), replace=False).tolist())
    tb, tp, want = poisoned_indices(T, B, S, rng, bad)
    good = np.array([i for i in range(T) if i not in bad])
    say(f"  bad rows {bad}: tok_batch {tb[bad].tolist()} tok_pos {tp[bad].tolist()}")
    with_bad, only_good, silent = GuardedCache(lay, cdt), GuardedCache(lay, cdt), GuardedCache(lay, cdt)
    status = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    dv = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    fdc.fdc_project_latent_kv(lay, 0, x, dv(tb), dv(tp), A, with_bad.k, with_bad.v, status=status)
    fdc.fdc_project_latent_kv(lay, 0, x, dv(tb), dv(tp), A, silent.k, silent.v)          # no status word: still skipped
    clean = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    xg = x[torch.from_numpy(good).cuda()].contiguous()
    fdc.fdc_project_latent_kv(lay, 0, xg, dv(tb[good]), dv(tp[good]), A, only_good.k, only_good.v, status=clean)
    torch.cuda.synchronize()
    assert int(status.item()) == want and int(clean.item()) == 0
    # T and T - 4 rows fall into the same row-count class of kernels here, and a row's sum does not depend on the
    # other rows, so the stored bits agree
    assert with_bad.same_as(only_good), "a skipped row changed the cache or a guard band"
    assert silent.same_as(only_good)
    assert with_bad.k.count_nonzero() > 0


def test_project_and_absorb_query_one_launch_flags_too():
    H, d, d_h, B, S, T = 4, 512, 128, 4, 64, 9
    rk, rv = [16, 128, 48, 64], [32, 16, 128, 64]
    lay = fdc.Layout(1, H, d, d_h, [rk], [rv], B, S, fdc.FDC_BF16)
    rng = gen.make_rng(9)
    x = torch.from_numpy(gen.hidden_states(T, d, rng).astype(np.float32)).to(BF).cuda()
    A = torch.from_numpy((rng.standard_normal((sum(rk) + sum(rv), d)) / math.sqrt(d)).astype(np.float32)).to(BF).cuda()
    q = torch.from_numpy(rng.standard_normal((T, H, d_h)).astype(np.float32)).to(BF).cuda()
    Bk = torch.from_numpy((rng.standard_normal((sum(rk), d_h)) / math.sqrt(d_h)).astype(np.float32)).to(BF).cuda()
    tb, tp, want = poisoned_indices(T, B, S, rng, [2, 7])
    good = np.array([i for i in range(T) if i not in (2, 7)])
    dv = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    with_bad, only_good = GuardedCache(lay, BF), GuardedCache(lay, BF)
    status = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    ql = torch.full((T, sum(rk)), float("nan"), dtype=torch.float32, device="cuda:0")
    ql2 = torch.full((T, sum(rk)), float("nan"), dtype=torch.float32, device="cuda:0")
    fdc.fdc_project_and_absorb_query(lay, 0, x, dv(tb), dv(tp), A, with_bad.k, with_bad.v, q, Bk, ql, fdc.FDC_F32,
                                     status=status)
    fdc.fdc_project_latent_kv(lay, 0, x[torch.from_numpy(good).cuda()].contiguous(), dv(tb[good]), dv(tp[good]), A,
                              only_good.k, only_good.v)
    fdc.fdc_absorb_query(lay, 0, q, Bk, ql2, fdc.FDC_F32)
    torch.cuda.synchronize()
    assert int(status.item()) == want
    assert with_bad.same_as(only_good)
    assert torch.equal(ql, ql2)          # queries do not depend on the cache indices: all rows are computed


@pytest.mark.parametrize("dtype", [fdc.FDC_BF16, fdc.FDC_FP8])
def test_post_rope_writers_skip_and_flag(dtype):
    say(f"post-RoPE writers, layout dtype {dtype}")
    H, d_h, B, S, T, n_pos = 3, 64, 2, 300, 200, 256     # positions 256..299 exist in the cache but have no angle
    rk = [16, 64, 48]
    lay = fdc.Layout(1, H, 256, d_h, [rk], [rk], B, S, dtype)
    cdt = BF if dtype == fdc.FDC_BF16 else torch.uint8
    rng = gen.make_rng(11)
    k = torch.from_numpy(rng.standard_normal((T, H, d_h)).astype(np.float32)).to(BF).cuda()
    R_t = torch.from_numpy(np.ascontiguousarray(np.concatenate([gen.random_orthonormal(d_h, d_h, rng)[:, :r].T for r in rk]),
                                                dtype=np.float32)).to(BF).cuda().contiguous()
    cos, sin = orp.rope_tables(n_pos, d_h)
    cs = torch.from_numpy(np.ascontiguousarray(cos, dtype=np.float32)).cuda().contiguous()
    sn = torch.from_numpy(np.ascontiguousarray(sin, dtype=np.float32)).cuda().contiguous()
    slots = rng.permutation(B * n_pos)[:T]
    tb, tp = (slots // n_pos).astype(np.int32), (slots % n_pos).astype(np.int32)
    bad = [3, 64, 65, 150, 199]
    tb[3] = B + 5                    # sequence out of range
    tp[64] = n_pos                   # inside the cache, but no angle
    tp[65] = S + 100                 # outside both
    tp[150] = -1
    tb[199] = -2
    good = np.array([i for i in range(T) if i not in bad])
    dv = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    with_bad, only_good = GuardedCache(lay, cdt), GuardedCache(lay, cdt)
    status = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    fdc.fdc_rope_compress_keys(lay, 0, k, dv(tb), dv(tp), cs, sn, R_t, with_bad.k, status=status)
    fdc.fdc_rope_compress_keys(lay, 0, k[torch.from_numpy(good).cuda()].contiguous(), dv(tb[good]), dv(tp[good]), cs, sn,
                               R_t, only_good.k)
    torch.cuda.synchronize()
    assert int(status.item()) == FAULT_BATCH | FAULT_POS
    assert with_bad.same_as(only_good) and with_bad.k.count_nonzero() > 0
    # queries: a position without an angle leaves the row of q_lat untouched and is flagged
    q = torch.from_numpy(rng.standard_normal((T, H, d_h)).astype(np.float32)).to(BF).cuda()
    pos = rng.integers(0, n_pos, T).astype(np.int32)
    pos_bad = pos.copy()
    pos_bad[[0, 77]] = [n_pos + 3, -1]
    ql = torch.full((T, sum(rk)), -5.0, dtype=torch.float32, device="cuda:0")
    ref = torch.full((T, sum(rk)), -5.0, dtype=torch.float32, device="cuda:0")
    status.zero_()
    fdc.fdc_rope_absorb_query(lay, 0, q, dv(pos_bad), cs, sn, R_t, ql, fdc.FDC_F32, status=status)
    fdc.fdc_rope_absorb_query(lay, 0, q, dv(pos), cs, sn, R_t, ref, fdc.FDC_F32)
    torch.cuda.synchronize()
    assert int(status.item()) == FAULT_POS
    keep = np.ones(T, bool)
    keep[[0, 77]] = False
    keep_t = torch.from_numpy(keep).cuda()
    assert torch.equal(ql[keep_t], ref[keep_t])
    assert bool((ql[~keep_t] == -5.0).all())
