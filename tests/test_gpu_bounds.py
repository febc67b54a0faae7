"""No call writes outside what it was given: every workspace is exactly as large as
mhcl_workspace_bytes says and, like every output tensor, sits between two 64 KiB
guard regions filled with a pattern that must survive.  Seeded random shapes and
forms, all entry points of the hot path."""
import math
import random

import pytest
import torch

import paper_2601_05732_amd as mhcl
import synth_inputs as si
from gpu_harness import GpuLayer, desc_for

pytestmark = pytest.mark.gpu

GUARD = 1 << 16
OUTS = ("H_res", "H_pre", "H_post", "h", "x_out", "g_x", "g_y", "g_W", "g_b", "g_alpha",
        "g_H_res", "g_H_pre", "g_H_post")


def _guarded(nbytes):
    buf = torch.full((nbytes + 2 * GUARD + 256,), 0xA5, dtype=torch.uint8, device="cuda")
    off = GUARD + ((-(buf.data_ptr() + GUARD)) % 256)
    return buf, buf[off:off + nbytes], off


def _intact(buf, off, nbytes):
    return bool((buf[:off] == 0xA5).all()) and bool((buf[off + nbytes:] == 0xA5).all())


@pytest.mark.parametrize("seed", [0, 1])
def test_guard_regions_survive(seed):
    rng = random.Random(seed)
    broken = []
    for case in range(40):
        mode = rng.choice(["lite", "lite", "sk", "subset", "subset"])
        io = rng.choice(["bf16", "bf16", "bf16", "f32"])
        if mode == "subset":
            n = rng.randint(1, 8)
            K = rng.randint(1, min(128, math.factorial(n)))
        else:
            n, K = rng.randint(1, 5), 0
        C = rng.choice([64, 128, 192, 256, 512, 1024, 40, 72, 8, 2048])
        T = rng.choice([1, 15, 17, 31, 33, 63, 65, 100, 127, 129, 255, 257, 513, 1000, 2049,
                        16385, 20000, 32641])
        if n * C * T > 6e7:
            T = max(1, int(6e7 / (n * C)))
        wl = si.Workload(name=f"guard{case}", n=n, C=C, T=T, io=io, res_mode=mode, n_perm=K)
        print(f"case {wl}", flush=True)
        i = si.make_inputs(wl, seed=700 + case, device="cuda")
        d = desc_for(wl, perm=i.get("perm"))
        L = GpuLayer(d, i)
        guards = []
        for k in OUTS:
            t = getattr(L, k)
            nb = t.numel() * t.element_size()
            buf, view, off = _guarded(nb)
            setattr(L, k, view.view(t.dtype).view(t.shape))
            guards.append((k, buf, off, nb))
        L.forward_separable()
        L.forward_fused()
        L.backward_fused()
        L.backward_separable()
        calls = [
            (mhcl.OP_COEFFS, lambda ws: mhcl.mhcl_coeffs(d, i["x"], i["W"], i["b"], i["alpha"], L.H_res, L.H_pre,
                                                         L.H_post, ws)),
            (mhcl.OP_FWD_COEFFS_PRE, lambda ws: mhcl.mhcl_fwd_coeffs_pre(d, i["x"], i["W"], i["b"], i["alpha"],
                                                                         L.H_res, L.H_pre, L.H_post, L.h, ws)),
            (mhcl.OP_BWD_FUSED, lambda ws: mhcl.mhcl_bwd_fused(d, i["x"], i["y"], i["W"], i["b"], i["alpha"],
                                                               i["g_xout"], i["g_h"], L.g_x, L.g_y, L.g_W, L.g_b,
                                                               L.g_alpha, ws)),
            (mhcl.OP_COEFFS_BWD, lambda ws: mhcl.mhcl_coeffs_bwd(d, i["x"], i["W"], i["b"], i["alpha"], L.g_H_res,
                                                                 L.g_H_pre, L.g_H_post, L.g_x, L.g_W, L.g_b,
                                                                 L.g_alpha, ws)),
        ]
        for op, fn in calls:
            nb = mhcl.workspace_bytes(d, op)
            buf, ws, off = _guarded(nb)
            fn(ws)
            torch.cuda.synchronize()
            if not _intact(buf, off, nb):
                broken.append(f"{wl}: workspace of op {op} ({nb} bytes)")
        for k, buf, off, nb in guards:
            if not _intact(buf, off, nb):
                broken.append(f"{wl}: around {k}")
        del L, i
    assert not broken, "\n".join(broken)
