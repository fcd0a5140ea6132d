"""A decode layer captured into a HIP graph: re-plan on the device, projection + query absorption,
decode attention at the actual lengths, output projection. No call of the library allocates,
synchronises or clears memory with a memset, so the sequence must be capturable; every replay is
compared bit for bit with the same calls made eagerly on a second copy of the cache, with eager
work and synchronisations between the replays.
"""
import math
import sys

import numpy as np
import pytest
import torch

import paper_2408_04107_amd as fdc
from tests.gpu_util import workspace_for

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[graph] {msg}", flush=True)
    sys.stdout.flush()


@pytest.mark.parametrize("g,dtype", [(1, fdc.FDC_BF16), (4, fdc.FDC_FP8)])
def test_decode_layer_in_a_hip_graph(g, dtype):
    dev = "cuda:0"
    rk, rv = [16, 32, 48, 64, 80, 96, 112, 128], [128, 16, 48, 64, 32, 112, 96, 80]
    H, B, S_max, d, dh, G = len(rk), 6, 1536, 512, 128, 64
    say(f"g={g} dtype={dtype}")
    lay = fdc.Layout(1, H, d, dh, [rk], [rv], B, S_max, dtype, q_per_kv=g)
    t = lay.tables()
    RK, RV = int(t["koff_r"][0, -1]), int(t["voff_r"][0, -1])
    gt = torch.Generator(device=dev).manual_seed(21)
    bf = torch.bfloat16
    es = 2 if dtype == fdc.FDC_BF16 else 1
    nk, nv = int(t["k_bytes"][0]) // es, int(t["v_bytes"][0]) // es
    if dtype == fdc.FDC_BF16:
        k0 = (torch.randn(nk, generator=gt, device=dev) * 0.5).to(bf)
        v0 = (torch.randn(nv, generator=gt, device=dev) * 0.5).to(bf)
    else:   # small-magnitude E4M3 codes of either sign
        mk = lambda n: torch.randint(0, 0x40, (n,), generator=gt, device=dev, dtype=torch.uint8) | \
            (torch.randint(0, 2, (n,), generator=gt, device=dev, dtype=torch.uint8) << 7)
        k0, v0 = mk(nk), mk(nv)
    A_cat = (torch.randn(RK + RV, d, generator=gt, device=dev) / math.sqrt(d)).to(bf)
    Bk = (torch.randn(RK, dh, generator=gt, device=dev) / math.sqrt(dh)).to(bf)
    Mt = (torch.randn(d, g * RV, generator=gt, device=dev) / math.sqrt(RV)).to(bf)
    scale = 1.0 / math.sqrt(dh)
    pp = fdc.fdc_plan_params_default()
    pp.n_workers, pp.granule = 192, G
    plan = fdc.fdc_plan_decode_device(lay, 0, B, 0, pp)
    ws = workspace_for(plan)
    tb = torch.arange(B, dtype=torch.int32, device=dev)

    class Bufs:
        def __init__(self):
            self.k, self.v = k0.clone(), v0.clone()
            self.x = torch.zeros(B, d, dtype=bf, device=dev)
            self.q = torch.zeros(B, H * g, dh, dtype=bf, device=dev)
            self.lens = torch.zeros(B, dtype=torch.int32, device=dev)      # lengths including the new token
            self.planned = torch.zeros(B, dtype=torch.int32, device=dev)   # rounded up to the granule
            self.pos = torch.zeros(B, dtype=torch.int32, device=dev)
            self.q_lat = torch.zeros(B * g * RK, dtype=torch.float32, device=dev)
            self.o_lat = torch.zeros(B * g * RV, dtype=torch.float32, device=dev)
            self.y = torch.zeros(B, d, dtype=bf, device=dev)

        def set(self, lens, seed):
            gi = torch.Generator(device=dev).manual_seed(seed)
            self.x.copy_(torch.randn(B, d, generator=gi, device=dev).to(bf))
            self.q.copy_(torch.randn(B, H * g, dh, generator=gi, device=dev).to(bf))
            l = torch.tensor(lens, dtype=torch.int32, device=dev)
            self.lens.copy_(l)
            self.planned.copy_((l + (G - 1)) // G * G)
            self.pos.copy_(l - 1)

        def layer(self):
            fdc.fdc_plan_decode_run([plan], [ws], self.planned)
            fdc.fdc_project_and_absorb_query(lay, 0, self.x, tb, self.pos, A_cat, self.k, self.v, self.q, Bk,
                                             self.q_lat, fdc.FDC_F32)
            fdc.fdc_latent_attn_decode_at(lay, plan, self.lens, self.q_lat, self.k, self.v, scale, self.o_lat, ws)
            fdc.fdc_absorb_output(lay, 0, fdc.FDC_APPLY, None, None, Mt, self.o_lat, fdc.FDC_F32, B, self.y, fdc.FDC_BF16)

    eager, graphed = Bufs(), Bufs()
    lens0 = [1000, 1, 64, 65, 1500, 700]
    eager.set(lens0, 0), graphed.set(lens0, 0)
    graphed.layer()               # warm-up outside the capture (first-call set-up of the kernels)
    graphed.k.copy_(k0), graphed.v.copy_(v0)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        graphed.layer()
    graphed.k.copy_(k0), graphed.v.copy_(v0)   # capture itself runs nothing, but keep the state explicit
    for r, lens in enumerate([lens0, [l + 1 for l in lens0], [1536, 2, 128, 129, 1, 701], [64] * B]):
        say(f"replay {r}: lens={lens}")
        eager.set(lens, 100 + r), graphed.set(lens, 100 + r)
        eager.layer()
        graph.replay()
        torch.cuda.synchronize()
        junk = torch.randn(1 << 20, device=dev).sum().item()   # eager work and a host sync between replays
        assert math.isfinite(junk)
        assert torch.equal(eager.y.view(torch.int16), graphed.y.view(torch.int16)), f"replay {r}: y differs"
        assert torch.equal(eager.o_lat, graphed.o_lat), f"replay {r}: o_lat differs"
        kk = lambda b: b.view(torch.int16) if dtype == fdc.FDC_BF16 else b
        assert torch.equal(kk(eager.k), kk(graphed.k)) and torch.equal(kk(eager.v), kk(graphed.v)), f"replay {r}: cache differs"
        assert np.all(np.isfinite(graphed.y.float().cpu().numpy()))
