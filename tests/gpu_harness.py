"""Helpers of the GPU parity tests: the error metric and the oracle's results
for the same input bits.  Nothing here computes any part of the method.
"""
from __future__ import annotations

import numpy as np
import torch

import synth_inputs as si
from paper_2601_05732_amd.layer import GpuLayer, desc_for  # noqa: F401


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
