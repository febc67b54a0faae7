"""mhcl_profile_next_call arms ONE library call of this host thread: whatever that call is,
the arming is gone afterwards, so a later call never records the events."""
import ctypes

import pytest
import torch

import paper_2601_05732_amd as mhcl
import synth_inputs as si
from bench import HipEvents
from gpu_harness import GpuLayer, desc_for

pytestmark = pytest.mark.gpu

STAGE_POST = 3


def _recorded(ev):
    try:
        ev.elapsed_ms(0, 1)
        return True
    except RuntimeError:
        return False


def test_any_call_clears_a_pending_arming():
    wl = si.Workload("arm", n=4, C=256, T=300, io="bf16")
    inp = si.make_inputs(wl, seed=0, device="cuda")
    L = GpuLayer(desc_for(wl), inp)
    L.forward_fused()
    lib = mhcl.lib()
    lib.mhcl_profile_next_call.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    calls = {
        "mhcl_post_bwd": lambda: mhcl.mhcl_post_bwd(L.d, inp["x"], inp["y"], L.H_res, L.H_post, inp["g_xout"],
                                                    L.g_x, L.g_y, L.g_H_res, L.g_H_post),
        "mhcl_pre_bwd": lambda: mhcl.mhcl_pre_bwd(L.d, inp["x"], L.H_pre, inp["g_h"], L.g_x, L.g_H_pre),
        "mhcl_pre": lambda: mhcl.mhcl_pre(L.d, inp["x"], L.H_pre, L.h),
        "mhcl_bwd_fused": L.backward_fused,
    }
    for name, other in calls.items():
        ev = HipEvents(2)
        assert lib.mhcl_profile_next_call(STAGE_POST, ev.ev[0], ev.ev[1]) == 0
        other()                                   # has no POST stage: records nothing, disarms
        mhcl.mhcl_post(L.d, inp["x"], inp["y"], L.H_res, L.H_post, L.x_out)
        torch.cuda.synchronize()
        assert not _recorded(ev), f"{name} left the bracket armed"
        ev.close()
    ev = HipEvents(2)                             # and an armed call does record
    assert lib.mhcl_profile_next_call(STAGE_POST, ev.ev[0], ev.ev[1]) == 0
    mhcl.mhcl_post(L.d, inp["x"], inp["y"], L.H_res, L.H_post, L.x_out)
    torch.cuda.synchronize()
    assert _recorded(ev)
    ev.close()
