"""Helpers of the GPU parity tests: the error metric and the oracle's results
for the same input bits.  Nothing here computes any part of the method.
"""
from __future__ import annotations

import numpy as np
import torch

import synth_inputs as si
from paper_2601_05732_amd.layer import GpuLayer, desc_for  # noqa: F401


# Tolerances of the GPU parity tests, metric rel_err() below, per tensor.
#  * f32 streams: 1e-5 on every output (the stated bound for fp32 paths).
#  * bf16 streams, bf16 outputs: 2e-2 (the stated bound).
#  * bf16 streams, fp32 coefficients H_res, H_pre, H_post: the MFMA projection carries W as two
#    bf16 parts, |dW| <= 2^-18 |W| per entry, x is exact.  With independent roundings the logit
#    error has standard deviation 2^-18 / sqrt(3) * std(z): 5.6e-6 at std(z) = 2.56 (n = 4,
#    C = 4096, W ~ N(0, 0.02^2)); a softmax weight moves by that fraction of itself, so the
#    largest error over the 10^6 entries of a 32k-token workload is about 4.5 sigma = 2.5e-5.
#    Gate: 5e-5.  (Measured: 1.3e-5 over 70 tokens, 3e-6 typical.)
#  * bf16 streams, fp32 parameter gradients: vr = r alpha g_z enters the g_W MFMAs as two bf16
#    parts (2^-18 per term, random signs: the relative error of a sum over tokens stays at that
#    level), g_z itself comes from fp32 sums of exact bf16 products over C.  Measured <= 3.5e-5;
#    gate 2e-4.
TOL_F32 = 1e-5
TOL_BF16_OUT = 2e-2
TOL_BF16_COEF = 5e-5
TOL_BF16_PARAM = 2e-4


def to_np64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu", torch.float64).numpy()


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max_e |got_e - ref_e| / max(|ref_e|, rms(ref))."""
    if ref.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(ref * ref)))
    den = np.maximum(np.abs(ref), max(rms, 1e-300))
    return float(np.max(np.abs(got - ref) / den))


def oracle_reference(inp: dict, wl: si.Workload, tokens=None, backward=True):
    """Oracle results for `tokens` (index array; None = all) from the same
    input bits.  Sums over tokens (g_W, g_b, g_alpha) cover only `tokens`."""
    import oracle
    sel = (lambda t: t) if tokens is None else (lambda t: t[torch.as_tensor(tokens, device=t.device)])
    x, y = to_np64(sel(inp["x"])), to_np64(sel(inp["y"]))
    W, b, al = to_np64(inp["W"]), to_np64(inp["b"]), to_np64(inp["alpha"])
    sigma = inp["perm"].cpu().numpy().astype(np.int32) if wl.res_mode == "subset" else None
    if not backward:
        return oracle.forward(x, W, b, al, y, eps=wl.eps, res_mode=wl.res_mode, iters=wl.sk_iters,
                              sigma=sigma)
    return oracle.backward(x, W, b, al, y, to_np64(sel(inp["g_xout"])), to_np64(sel(inp["g_h"])),
                           eps=wl.eps, res_mode=wl.res_mode, iters=wl.sk_iters, sigma=sigma)
