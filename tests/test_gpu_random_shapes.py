"""GPU parity on seeded random shapes and forms: stream counts 1-8, widths that take
the MFMA path (multiples of 64) and widths that do not, token counts around the tile
sizes, both stream types, the permutation, Sinkhorn-Knopp and subset forms.  Every
token and every output is compared with the oracle; tolerances as in
test_gpu_parity.py."""
import math
import random

import pytest
import torch

import synth_inputs as si
from gpu_harness import (GpuLayer, desc_for, oracle_reference, rel_err, to_np64,
                         TOL_BF16_OUT, TOL_BF16_COEF, TOL_BF16_PARAM)

pytestmark = pytest.mark.gpu

WIDTHS = [64, 128, 192, 256, 320, 512, 1024, 40, 72, 8, 96]
TOKENS = [1, 7, 15, 16, 17, 63, 64, 65, 100, 127, 129, 200, 255, 257, 300, 511, 513, 700]


def _draw(rng, case):
    mode = rng.choice(["lite", "lite", "sk", "subset", "subset"])
    io = rng.choice(["bf16", "bf16", "bf16", "f32"])
    if mode == "subset":
        n = rng.randint(1, 8)
        K = rng.randint(1, min(128, math.factorial(n)))
    else:
        n, K = rng.randint(1, 5), 0
    C, T = rng.choice(WIDTHS), rng.choice(TOKENS)
    if n * C > 8192:
        C = 64
    iters = rng.choice([20, 20, 3, 1]) if mode == "sk" else 20
    return si.Workload(name=f"random{case}", n=n, C=C, T=T, io=io, res_mode=mode, n_perm=K, sk_iters=iters)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_random_shapes_against_the_oracle(seed):
    rng = random.Random(seed)
    failures = []
    for case in range(40):
        wl = _draw(rng, case)
        print(f"case {wl}", flush=True)
        inp = si.make_inputs(wl, seed=1000 * seed + case, device="cuda")
        L = GpuLayer(desc_for(wl, perm=inp.get("perm")), inp)
        L.forward_fused()
        L.backward_fused()
        torch.cuda.synchronize()
        ref = oracle_reference(inp, wl)
        out, coef, par = (1e-5, 1e-5, 1e-5) if wl.io == "f32" else (TOL_BF16_OUT, TOL_BF16_COEF, TOL_BF16_PARAM)
        for name, tol in [("H_res", coef), ("H_pre", coef), ("H_post", coef), ("h", out), ("x_out", out),
                          ("g_x", out), ("g_y", out), ("g_W", par), ("g_b", par), ("g_alpha", par)]:
            e = rel_err(to_np64(getattr(L, name)), ref[name])
            if not e <= tol:
                failures.append(f"{wl.name} {wl}: {name} {e:.3e} > {tol}")
        if case % 4 == 0:      # the separable calls (other kernels) on the same input
            L.forward_separable()
            L.backward_separable()
            torch.cuda.synchronize()
            for name, tol in [("H_res", coef), ("h", out), ("x_out", out), ("g_x", out), ("g_y", out),
                              ("g_W", par), ("g_b", par), ("g_alpha", par)]:
                e = rel_err(to_np64(getattr(L, name)), ref[name])
                if not e <= tol:
                    failures.append(f"{wl.name} {wl}: separable {name} {e:.3e} > {tol}")
    assert not failures, "\n".join(failures)


def test_random_shapes_with_many_tokens():
    """The same with 16k to 65k tokens (narrow streams, so that the oracle still redoes
    every token): token counts around the points where launch shapes change, and counts
    that the token-chunk grids of the backward do not divide."""
    rng = random.Random(0)
    failures = []
    for case in range(10):
        mode = rng.choice(["lite", "sk", "subset"])
        if mode == "subset":
            n = rng.randint(2, 8)
            K = rng.randint(1, min(96, math.factorial(n)))
        else:
            n, K = rng.randint(1, 5), 0
        C = rng.choice([64, 128, 192, 256])
        T = rng.choice([32639, 32640, 32641, 32768, 40000, 50001, 65539, 16383, 16385, 20000])
        wl = si.Workload(name=f"many{case}", n=n, C=C, T=T, io="bf16", res_mode=mode, n_perm=K)
        print(f"case {wl}", flush=True)
        inp = si.make_inputs(wl, seed=77 + case, device="cuda")
        L = GpuLayer(desc_for(wl, perm=inp.get("perm")), inp)
        L.forward_fused()
        L.backward_fused()
        torch.cuda.synchronize()
        ref = oracle_reference(inp, wl)
        for name, tol in [("H_res", TOL_BF16_COEF), ("H_pre", TOL_BF16_COEF), ("H_post", TOL_BF16_COEF),
                          ("h", 2e-2), ("x_out", 2e-2), ("g_x", 2e-2), ("g_y", 2e-2),
                          ("g_W", TOL_BF16_PARAM), ("g_b", TOL_BF16_PARAM), ("g_alpha", TOL_BF16_PARAM)]:
            e = rel_err(to_np64(getattr(L, name)), ref[name])
            if not e <= tol:
                failures.append(f"{wl}: {name} {e:.3e} > {tol}")
        del L, inp, ref
    assert not failures, "\n".join(failures)


def test_random_shapes_with_16_byte_aligned_tensors():
    """The C ABI asks for 16-byte alignment only: every stream tensor, inputs and outputs,
    starts an odd multiple of 16 bytes past a 1 KiB boundary."""
    from paper_2601_05732_amd.layer import empty_stream, place_stream
    rng = random.Random(5)
    failures = []
    for case in range(30):
        wl = _draw(rng, case)
        print(f"case {wl}", flush=True)
        inp = si.make_inputs(wl, seed=300 + case, device="cuda")
        phase = lambda: 16 * rng.choice([1, 3, 5, 7, 9, 13, 21, 33, 47, 63])
        for k in ("x", "y", "g_xout", "g_h"):
            inp[k] = place_stream(inp[k], phase())
        L = GpuLayer(desc_for(wl, perm=inp.get("perm")), inp)
        for k in ("h", "x_out", "g_x", "g_y"):
            t = getattr(L, k)
            setattr(L, k, empty_stream(t.shape, t.dtype, t.device, phase()))
        L.forward_fused()
        L.backward_fused()
        torch.cuda.synchronize()
        ref = oracle_reference(inp, wl)
        out, coef, par = (1e-5, 1e-5, 1e-5) if wl.io == "f32" else (TOL_BF16_OUT, TOL_BF16_COEF, TOL_BF16_PARAM)
        for name, tol in [("H_res", coef), ("H_pre", coef), ("H_post", coef), ("h", out), ("x_out", out),
                          ("g_x", out), ("g_y", out), ("g_W", par), ("g_b", par), ("g_alpha", par)]:
            e = rel_err(to_np64(getattr(L, name)), ref[name])
            if not e <= tol:
                failures.append(f"{wl}: {name} {e:.3e} > {tol}")
    assert not failures, "\n".join(failures)
