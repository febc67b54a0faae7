"""A whole step (fused forward calls + fused backward) captured in a HIP graph
replays to the same bits as eager launches: the library allocates nothing,
synchronises nothing and clears memory with kernels, so a caller may capture
it.  Replays are interleaved with eager work and new inputs, and every replay
is checked.
"""
import pytest
import torch

import synth_inputs as si
from gpu_harness import GpuLayer, desc_for

pytestmark = pytest.mark.gpu

OUTS = ("H_res", "H_pre", "H_post", "h", "x_out", "g_x", "g_y", "g_W", "g_b", "g_alpha")


@pytest.mark.parametrize("wl", [
    si.Workload("graph_n4", n=4, C=512, T=1000),
    si.Workload("graph_n5", n=5, C=128, T=300),
    si.Workload("graph_sk", n=4, C=256, T=257, res_mode="sk"),
    si.Workload("graph_f32", n=3, C=40, T=50, io="f32"),
    si.Workload("graph_n8_k64", n=8, C=64, T=150, res_mode="subset", n_perm=64),
], ids=lambda w: w.name)
def test_captured_step_replays_bitwise(wl):
    print(f"case {wl}", flush=True)
    inp = si.make_inputs(wl, seed=0, device="cuda")
    L = GpuLayer(desc_for(wl, perm=inp.get("perm")), inp)
    L.step()                                   # warm up outside the capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        L.step()
    for rep in range(3):
        fresh = si.make_inputs(wl, seed=10 + rep, device="cuda")
        for k, v in fresh.items():             # new values in the captured buffers
            inp[k].copy_(v)
        L.step()                               # eager
        torch.cuda.synchronize()
        want = {k: getattr(L, k).clone() for k in OUTS}
        for k in OUTS:                         # poison, so that a replay that does nothing is seen
            getattr(L, k).fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        for k in OUTS:
            assert torch.equal(getattr(L, k), want[k]), (rep, k)
