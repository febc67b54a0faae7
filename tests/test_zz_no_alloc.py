"""The allocation-free forward entry point (mhcl_fwd_coeffs_pre_static, scratch in a static
device array) against mhcl_fwd_coeffs_pre with a caller workspace: at these shapes both run the
same kernels (the projection, the coefficient stage, the pre-aggregate), so every output must
agree bit for bit; two calls in a row, the second on a smaller input, so that
what the first left in the shared array is shown not to leak into the second.  Also against
the oracle, at the tolerances of the parity tests.
"""
import numpy as np
import pytest
import torch

import paper_2601_05732_amd as mhcl
import synth_inputs as si
from gpu_harness import desc_for, oracle_reference, rel_err, to_np64

pytestmark = pytest.mark.gpu


def _run_both(wl, seed):
    inp = si.make_inputs(wl, seed=seed, device="cuda:0")
    d = desc_for(wl)
    dev, f, io = inp["x"].device, torch.float32, d.torch_dtype
    T, n, C = d.T, d.n, d.C
    mk = lambda: (torch.full((T, n, n), float("nan"), device=dev, dtype=f),
                  torch.full((T, n), float("nan"), device=dev, dtype=f),
                  torch.full((T, n), float("nan"), device=dev, dtype=f),
                  torch.full((T, C), float("nan"), device=dev, dtype=io))
    ref = mk()
    ws = mhcl.binding.new_workspace(d, mhcl.OP_FWD_COEFFS_PRE, dev)
    mhcl.mhcl_fwd_coeffs_pre(d, inp["x"], inp["W"], inp["b"], inp["alpha"], *ref, ws)
    got = mk()
    before = torch.cuda.memory_allocated()
    mhcl.mhcl_fwd_coeffs_pre_static(d, inp["x"], inp["W"], inp["b"], inp["alpha"], *got)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    return inp, ref, got


def _same_bits(a, b):
    return torch.equal(a.view(torch.uint8), b.view(torch.uint8))


def test_static_scratch_matches_workspace_call_twice_second_smaller():
    big = si.Workload("static_big", n=4, C=1024, T=4133, io="bf16")       # MFMA path, ragged tail
    small = si.Workload("static_small", n=4, C=1024, T=517, io="bf16")    # fewer tokens: K split differs
    for wl, seed in ((big, 11), (small, 12)):
        inp, ref, got = _run_both(wl, seed)
        for name, a, b in zip(("H_res", "H_pre", "H_post", "h"), ref, got):
            assert _same_bits(a, b), f"{wl.name}: {name} differs from the workspace call"
        o = oracle_reference(inp, wl, backward=False)
        for name, t, tol in zip(("H_res", "H_pre", "H_post", "h"), got, (1e-5, 1e-5, 1e-5, 2e-2)):
            e = rel_err(to_np64(t), o[name])
            assert e <= tol, f"{wl.name}: {name} vs oracle {e:.3e} > {tol}"


def test_static_scratch_other_forms_and_plain_path():
    cases = [si.Workload("static_f32", n=3, C=40, T=300, io="f32"),                       # plain ALU kernels
             si.Workload("static_sk", n=4, C=256, T=1000, io="bf16", res_mode="sk"),
             si.Workload("static_n5", n=5, C=128, T=70, io="bf16")]
    for k, wl in enumerate(cases):
        _, ref, got = _run_both(wl, 20 + k)
        for name, a, b in zip(("H_res", "H_pre", "H_post", "h"), ref, got):
            assert _same_bits(a, b), f"{wl.name}: {name} differs from the workspace call"


def test_static_scratch_rejects_shapes_beyond_the_array():
    wl = si.Workload("static_too_big", n=4, C=64, T=200000, io="bf16")
    d = desc_for(wl)
    assert mhcl.workspace_bytes(d, mhcl.OP_FWD_COEFFS_PRE) > mhcl.STATIC_SCRATCH_BYTES
    import ctypes
    # null tensors would be INVALID_ARG; use real (tiny) pointers so that the size check is what answers
    t = torch.zeros(64, device="cuda:0")
    p = ctypes.c_void_p(t.data_ptr())
    rc = mhcl.lib().mhcl_fwd_coeffs_pre_static(ctypes.byref(d.c), p, p, p, p, p, p, p, p, None)
    assert rc == 3   # MHCL_ERR_WORKSPACE, nothing enqueued
    torch.cuda.synchronize()


def test_static_scratch_call_under_graph_capture():
    """The callers it is for: captured in a HIP graph (after one eager call, which looks up the
    array's address), every replay gives the bits of the eager call, with new inputs and eager
    work between the replays."""
    wl = si.Workload("static_graph", n=4, C=512, T=1500, io="bf16")
    inp = si.make_inputs(wl, seed=31, device="cuda:0")
    d = desc_for(wl)
    dev, f = inp["x"].device, torch.float32
    T, n, C = d.T, d.n, d.C
    outs = (torch.empty(T, n, n, device=dev, dtype=f), torch.empty(T, n, device=dev, dtype=f),
            torch.empty(T, n, device=dev, dtype=f), torch.empty(T, C, device=dev, dtype=d.torch_dtype))
    call = lambda: mhcl.mhcl_fwd_coeffs_pre_static(d, inp["x"], inp["W"], inp["b"], inp["alpha"], *outs)
    call()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        call()
    for rep in range(3):
        fresh = si.make_inputs(wl, seed=40 + rep, device="cuda:0")
        for k in ("x", "W", "b"):
            inp[k].copy_(fresh[k])
        call()
        torch.cuda.synchronize()
        want = [t.clone() for t in outs]
        for t in outs:
            t.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        for name, a, b in zip(("H_res", "H_pre", "H_post", "h"), want, outs):
            assert _same_bits(a, b), (rep, name)


def test_static_scratch_empty_input_and_bad_arguments():
    import ctypes
    d0 = desc_for(si.Workload("static_empty", n=4, C=64, T=0, io="bf16"))
    assert mhcl.lib().mhcl_fwd_coeffs_pre_static(ctypes.byref(d0.c), *([None] * 9)) == 0    # T = 0: nothing to do
    d = desc_for(si.Workload("static_bad", n=4, C=64, T=8, io="bf16"))
    t = torch.zeros(4096, device="cuda:0")
    p = ctypes.c_void_p(t.data_ptr())
    assert mhcl.lib().mhcl_fwd_coeffs_pre_static(ctypes.byref(d.c), None, p, p, p, p, p, p, p, None) == 1   # null x
    odd = ctypes.c_void_p(t.data_ptr() + 4)
    assert mhcl.lib().mhcl_fwd_coeffs_pre_static(ctypes.byref(d.c), odd, p, p, p, p, p, p, p, None) == 1    # misaligned
    torch.cuda.synchronize()
