"""The single-read forward behind mhcl_fwd_coeffs_pre (Sec. 3.2 Eqs. (4)-(5), Sec. 2 Eq. (1)): at
shapes where it applies the call must run that kernel (no pre-aggregate stage of its own), match
the oracle on every token, agree with the separable calls, and repeat bit for bit on a reused
workspace (its exchange rings start from zero in every call)."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2601_05732_amd as mhcl
import synth_inputs as si
from bench import HipEvents
from gpu_harness import (GpuLayer, TOL_BF16_COEF, TOL_BF16_OUT, desc_for, oracle_reference, rel_err,
                         to_np64)

pytestmark = pytest.mark.gpu

STAGE_FWD_PRE = 2

# (the smallest token counts at which the kernel is used: 32 groups of 16 tokens per cluster,
#  256 / (C / 256) clusters; ragged tails on purpose)
CASES = [
    si.Workload("once_n4_c4096", n=4, C=4096, T=8192 + 7, io="bf16", backward=False),
    si.Workload("once_n4_c2048_sk", n=4, C=2048, T=16384, io="bf16", res_mode="sk", backward=False),
    si.Workload("once_n3_c1024", n=3, C=1024, T=32768 + 33, io="bf16", backward=False),
    si.Workload("once_n2_c1024", n=2, C=1024, T=32768 + 1, io="bf16", backward=False),
    si.Workload("once_n4_c2048_k12", n=4, C=2048, T=16384 + 17, io="bf16", res_mode="subset", n_perm=12,
                backward=False),
    # part counts that divide neither 16 nor 256: 12 (21 clusters), 20 (12), 5 (51); and 32
    si.Workload("once_n4_c3072", n=4, C=3072, T=10752 + 5, io="bf16", backward=False),
    si.Workload("once_n4_c5120", n=4, C=5120, T=6144 + 11, io="bf16", backward=False),
    si.Workload("once_n3_c1280", n=3, C=1280, T=26112 + 3, io="bf16", backward=False),
    si.Workload("once_n4_c8192", n=4, C=8192, T=4096 + 9, io="bf16", backward=False),
]


def _pre_stage_recorded(L):
    """True if the next mhcl_fwd_coeffs_pre runs a pre-aggregate kernel of its own."""
    lib = mhcl.lib()
    lib.mhcl_profile_next_call.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    ev = HipEvents(2)
    assert lib.mhcl_profile_next_call(STAGE_FWD_PRE, ev.ev[0], ev.ev[1]) == 0
    L.forward_fused()
    torch.cuda.synchronize()
    try:
        ev.elapsed_ms(0, 1)
        return True
    except RuntimeError:
        return False
    finally:
        ev.close()


@pytest.mark.parametrize("wl", CASES, ids=lambda w: w.name)
def test_single_read_forward_matches_oracle_and_separable_calls(wl):
    inp = si.make_inputs(wl, seed=3, device="cuda")
    d = desc_for(wl, perm=inp.get("perm"))
    assert mhcl.workspace_bytes(d, mhcl.OP_FWD_COEFFS_PRE) > mhcl.workspace_bytes(d, mhcl.OP_COEFFS), \
        "the shape is meant to take the single-read kernel (it needs one slice per 256 columns)"
    L = GpuLayer(d, inp)
    L.ws.fill_(0xA5)     # whatever a workspace holds must not matter
    assert not _pre_stage_recorded(L), "mhcl_fwd_coeffs_pre ran the two-kernel path"
    got = {k: getattr(L, k).clone() for k in ("H_res", "H_pre", "H_post", "h", "x_out")}
    # every token against the oracle
    ref = oracle_reference(inp, wl, backward=False)
    for k in ("H_res", "H_pre", "H_post"):
        err = rel_err(to_np64(got[k]), ref[k].reshape(got[k].shape))
        assert err <= TOL_BF16_COEF, (k, err)
    for k in ("h", "x_out"):
        err = rel_err(to_np64(got[k]), ref[k].reshape(got[k].shape))
        assert err <= TOL_BF16_OUT, (k, err)
    if wl.res_mode != "sk":   # (20 Sinkhorn-Knopp iterations only approach these sums)
        rs = to_np64(got["H_res"]).sum(-1)
        cs = to_np64(got["H_res"]).sum(-2)
        assert np.abs(rs - 1).max() <= 1e-6 and np.abs(cs - 1).max() <= 1e-6
    # h was made with the H_pre the call returns: the kernel adds the parts' sums in the order
    # the coefficient stage adds the slices, and mixes like mhcl_pre
    h2 = torch.empty_like(got["h"])
    mhcl.mhcl_pre(d, inp["x"], got["H_pre"], h2)
    torch.cuda.synchronize()
    assert torch.equal(h2, got["h"]), "h is not H_pre x of the returned H_pre, bit for bit"
    # a second call on the same workspace: the same bits
    L.forward_fused()
    torch.cuda.synchronize()
    for k, v in got.items():
        assert torch.equal(getattr(L, k), v), f"{k} differs between two calls"
    # the separable calls split the projection's fp32 sum over n C terms differently: the
    # coefficients agree to a few fp32 roundings of the logits, h to one bf16 step
    L.forward_separable()
    torch.cuda.synchronize()
    for k in ("H_res", "H_pre", "H_post"):
        err = rel_err(to_np64(getattr(L, k)), to_np64(got[k]))
        assert err <= 2e-5, (k, err)
    dh = (L.h.float() - got["h"].float()).abs()
    err = float((dh / got["h"].float().abs().clamp_min(1e-3)).max())
    assert err <= 2 ** -7, err


def test_environment_switch_keeps_the_two_kernel_path(monkeypatch):
    wl = si.Workload("once_off", n=4, C=2048, T=16384, io="bf16", backward=False)
    inp = si.make_inputs(wl, seed=2, device="cuda")
    d = desc_for(wl)
    on = mhcl.workspace_bytes(d, mhcl.OP_FWD_COEFFS_PRE)
    monkeypatch.setenv("MHCL_FWD_ONCE", "0")
    assert mhcl.workspace_bytes(d, mhcl.OP_FWD_COEFFS_PRE) == mhcl.workspace_bytes(d, mhcl.OP_COEFFS) < on
    L = GpuLayer(d, inp)
    assert _pre_stage_recorded(L)
    monkeypatch.delenv("MHCL_FWD_ONCE")
    L = GpuLayer(d, inp)
    assert not _pre_stage_recorded(L)


def test_shapes_outside_keep_the_two_kernel_path():
    for wl in (si.Workload("small_t", n=4, C=4096, T=8192 - 16, io="bf16"),
               si.Workload("odd_c", n=4, C=4096 + 64, T=8192, io="bf16"),
               si.Workload("wide_c", n=2, C=16384, T=4096, io="bf16"),
               si.Workload("n5", n=5, C=1024, T=16384, io="bf16")):
        inp = si.make_inputs(wl, seed=0, device="cuda")
        L = GpuLayer(desc_for(wl), inp)
        assert _pre_stage_recorded(L), wl.name


def _guarded(nbytes, guard=1 << 16):
    buf = torch.full((nbytes + 2 * guard + 256,), 0xA5, dtype=torch.uint8, device="cuda")
    off = guard + ((-(buf.data_ptr() + guard)) % 256)
    return buf, buf[off:off + nbytes], off


def test_single_read_forward_stays_inside_its_buffers():
    """Outputs and a workspace of exactly mhcl_workspace_bytes between guard regions."""
    wl = si.Workload("once_guard", n=4, C=2048, T=16384 + 5, io="bf16", backward=False)
    inp = si.make_inputs(wl, seed=5, device="cuda")
    d = desc_for(wl)
    L = GpuLayer(d, inp)
    guards = []
    for k in ("H_res", "H_pre", "H_post", "h"):
        t = getattr(L, k)
        nb = t.numel() * t.element_size()
        buf, view, off = _guarded(nb)
        setattr(L, k, view.view(t.dtype).view(t.shape))
        guards.append((k, buf, off, nb))
    nb = mhcl.workspace_bytes(d, mhcl.OP_FWD_COEFFS_PRE)
    buf, L.ws, off = _guarded(nb)
    guards.append(("ws", buf, off, nb))
    mhcl.mhcl_fwd_coeffs_pre(d, inp["x"], inp["W"], inp["b"], inp["alpha"], L.H_res, L.H_pre, L.H_post,
                             L.h, L.ws)
    torch.cuda.synchronize()
    for k, buf, off, nb in guards:
        assert bool((buf[:off] == 0xA5).all()) and bool((buf[off + nb:] == 0xA5).all()), k
    assert bool(torch.isfinite(L.h.float()).all())


def test_single_read_forward_in_a_graph_and_on_two_streams():
    """The kernel is an ordinary launch: it can be captured, and two calls on two streams (own
    outputs and workspaces) may overlap: each has 256 blocks that want a compute unit of their
    own, so they share the device cluster by cluster; both must come out bit for bit."""
    wl = si.Workload("once_graph", n=4, C=4096, T=8192 + 3, io="bf16", backward=False)
    inp = si.make_inputs(wl, seed=6, device="cuda")
    d = desc_for(wl)
    A, B = GpuLayer(d, inp), GpuLayer(d, inp)
    names = ("H_res", "H_pre", "H_post", "h")
    call = lambda L: mhcl.mhcl_fwd_coeffs_pre(d, inp["x"], inp["W"], inp["b"], inp["alpha"], L.H_res,
                                              L.H_pre, L.H_post, L.h, L.ws)
    call(A)
    torch.cuda.synchronize()
    want = {k: getattr(A, k).clone() for k in names}
    # captured and replayed, with eager calls in between
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        call(A)
    for rep in range(3):
        for k in names:
            getattr(A, k).fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        for k in names:
            assert torch.equal(getattr(A, k), want[k]), ("replay", rep, k)
        call(B)
        torch.cuda.synchronize()
    # two streams at once, several rounds
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    for rep in range(4):
        for L in (A, B):
            for k in names:
                getattr(L, k).fill_(float("nan"))
        torch.cuda.synchronize()
        with torch.cuda.stream(s1):
            call(A)
        with torch.cuda.stream(s2):
            call(B)
        torch.cuda.synchronize()
        for L in (A, B):
            for k in names:
                assert torch.equal(getattr(L, k), want[k]), ("two streams", rep, k)


def test_single_read_forward_seeded_shapes_against_the_separable_calls():
    """Seeded shapes and forms around the smallest token counts the kernel takes (every ragged
    tail 1..15 of the last 16-token group at least once over the cases): coefficients against
    mhcl_coeffs, h against mhcl_pre of the returned H_pre bit for bit."""
    import random
    rng = random.Random(17)
    for case in range(18):
        C = rng.choice([1024, 2048, 4096, 1536, 2560, 6144, 7168])
        mode = rng.choice(["lite", "lite", "sk", "subset"])
        n = rng.choice([2, 3, 4])
        K = 0
        if mode == "subset":
            K = rng.randint(1, min(32 - 2 * n, [0, 1, 2, 6, 24][n]))
        T = 32 * 16 * (256 // (C // 256)) + rng.randint(0, 300) * 16 + (case % 15 + 1)
        wl = si.Workload(f"once_fuzz{case}", n=n, C=C, T=T, io="bf16", res_mode=mode, n_perm=K,
                         backward=False)
        print(f"case {wl}", flush=True)
        inp = si.make_inputs(wl, seed=100 + case, device="cuda")
        d = desc_for(wl, perm=inp.get("perm"))
        L = GpuLayer(d, inp)
        assert not _pre_stage_recorded(L), wl
        got = {k: getattr(L, k).clone() for k in ("H_res", "H_pre", "H_post", "h")}
        assert all(bool(torch.isfinite(v.float()).all()) for v in got.values()), wl
        h2 = torch.empty_like(got["h"])
        mhcl.mhcl_pre(d, inp["x"], got["H_pre"], h2)
        mhcl.mhcl_coeffs(d, inp["x"], inp["W"], inp["b"], inp["alpha"], L.H_res, L.H_pre, L.H_post, L.ws)
        torch.cuda.synchronize()
        assert torch.equal(h2, got["h"]), wl
        for k in ("H_res", "H_pre", "H_post"):
            err = rel_err(to_np64(getattr(L, k)), to_np64(got[k]))
            assert err <= 2e-5, (wl, k, err)
        del L, inp, got, h2
        torch.cuda.empty_cache()


def test_autograd_stack_with_and_without_the_single_read_forward(monkeypatch):
    """Two bf16 layers through the torch.autograd front end at a shape the kernel takes: output
    and every gradient agree with the same stack run on the two-kernel forward (the two differ
    in how the projection's fp32 sum is split, nothing else)."""
    from paper_2601_05732_amd.autograd import HyperConnectionStack
    n, C, T, L = 4, 1024, 32768 + 5, 2
    f = lambda h: torch.tanh(h.float()).to(h.dtype)

    def run():
        torch.manual_seed(0)
        g = torch.Generator(device="cuda").manual_seed(4)
        x0 = (torch.randn(T, C, device="cuda", generator=g)).bfloat16().requires_grad_(True)
        G = torch.randn(T, C, device="cuda", generator=g).bfloat16()
        stack = HyperConnectionStack(n, C, [f] * L, "lite")   # (streams take the dtype of x0)
        for l, m in enumerate(stack.layers):
            gg = torch.Generator(device="cuda").manual_seed(50 + l)
            with torch.no_grad():
                m.W.copy_(0.02 * torch.randn(m.W.shape, device="cuda", generator=gg))
                m.b.copy_(0.1 * torch.randn(m.b.shape, device="cuda", generator=gg))
                m.alpha.fill_(1.0)
        out = stack(x0)
        (out.float() * G.float()).sum().backward()
        torch.cuda.synchronize()
        return [out.detach().float(), x0.grad.float()] + [p.grad.float() for m in stack.layers
                                                          for p in (m.W, m.b, m.alpha)]
    got = run()
    monkeypatch.setenv("MHCL_FWD_ONCE", "0")
    ref = run()
    names = ["out", "g_x0"] + [f"{p}{l}" for l in range(L) for p in ("g_W", "g_b", "g_alpha")]
    for k, a, b in zip(names, got, ref):
        tol = 2e-2 if k in ("out", "g_x0") else 2e-3
        err = rel_err(to_np64(a), to_np64(b))
        assert err <= tol, (k, err)
