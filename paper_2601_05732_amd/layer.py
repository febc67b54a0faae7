"""Buffers of one hyper-connection layer on the GPU and the library calls that
fill them: a convenience over :mod:`paper_2601_05732_amd.binding` used by the
tests, the smoke check and the benchmark.  It computes nothing itself.
"""
from __future__ import annotations

import torch

from . import binding as mhcl


def desc_for(wl, T=None, perm=None) -> mhcl.Desc:
    """Descriptor for a workload record (fields n, C, T, io, res_mode, sk_iters, eps);
    `perm` is the int8 GPU tensor [K, n] of the permutation-subset form."""
    mode = {"lite": mhcl.RES_LITE, "sk": mhcl.RES_SK, "subset": mhcl.RES_SUBSET}[wl.res_mode]
    if (mode == mhcl.RES_SUBSET) != (perm is not None):
        raise ValueError("perm goes with res_mode 'subset', and only with it")
    return mhcl.Desc(wl.n, wl.C, wl.T if T is None else T,
                     mhcl.BF16 if wl.io == "bf16" else mhcl.F32, mode, wl.sk_iters, wl.eps, perm)


# Start of a stream tensor relative to a 1 KiB boundary, by role.  Pass 2 of the fused
# backward keeps each block on one 256-byte column window of x, g_xout and g_x; when the
# three tensors are equally aligned all its loads and stores share address bits 8-12, and
# the kernel runs about 5 % slower than with the tensors 256 bytes out of step (measured;
# steps of 1 KiB and more change nothing, the other kernels do not care).
PHASE_X, PHASE_G_XOUT, PHASE_G_X = 0, 256, 512


def empty_stream(shape, dtype, device, phase: int = 0) -> torch.Tensor:
    """Uninitialised contiguous tensor whose first byte lies `phase` bytes (a multiple of
    16, below 1024) past a 1 KiB boundary: a view into a buffer 1 KiB larger than needed."""
    if phase % 16 or not 0 <= phase < 1024:
        raise ValueError("phase must be a multiple of 16 in [0, 1024)")
    numel = 1
    for v in shape:
        numel *= int(v)
    esize = torch.empty((), dtype=dtype).element_size()
    buf = torch.empty(numel * esize + 1024, dtype=torch.uint8, device=device)
    off = (phase - buf.data_ptr()) % 1024
    return buf[off:off + numel * esize].view(dtype).view(*shape)


def place_stream(t: torch.Tensor, phase: int) -> torch.Tensor:
    """Copy of `t` at the given phase (see `empty_stream`)."""
    out = empty_stream(t.shape, t.dtype, t.device, phase)
    out.copy_(t)
    return out


class GpuLayer:
    """Buffers of one layer on the GPU plus the calls that fill them."""

    def __init__(self, d: mhcl.Desc, inp: dict):
        self.d, self.inp = d, inp
        dev, f, io = inp["x"].device, torch.float32, d.torch_dtype
        T, n, C, M = d.T, d.n, d.C, d.M
        e = lambda *s, dt=f: torch.empty(s, device=dev, dtype=dt)
        self.H_res, self.H_pre, self.H_post = e(T, n, n), e(T, n), e(T, n)
        self.h, self.x_out = e(T, C, dt=io), empty_stream((T, n, C), io, dev, PHASE_X)
        self.g_x, self.g_y = empty_stream((T, n, C), io, dev, PHASE_G_X), e(T, C, dt=io)
        self.g_W, self.g_b, self.g_alpha = e(n * C, M), e(M), e(3)
        self.g_H_res, self.g_H_pre, self.g_H_post = e(T, n, n), e(T, n), e(T, n)
        nb = max(mhcl.workspace_bytes(d, op) for op in
                 (mhcl.OP_COEFFS, mhcl.OP_COEFFS_BWD, mhcl.OP_FWD_COEFFS_PRE, mhcl.OP_BWD_FUSED))
        self.ws = torch.empty(nb, device=dev, dtype=torch.uint8)

    # forward, separable calls
    def forward_separable(self):
        i, d = self.inp, self.d
        mhcl.mhcl_coeffs(d, i["x"], i["W"], i["b"], i["alpha"], self.H_res, self.H_pre,
                         self.H_post, self.ws)
        mhcl.mhcl_pre(d, i["x"], self.H_pre, self.h)
        mhcl.mhcl_post(d, i["x"], i["y"], self.H_res, self.H_post, self.x_out)

    # forward, fused calls (what the benchmark times)
    def forward_fused(self):
        i, d = self.inp, self.d
        mhcl.mhcl_fwd_coeffs_pre(d, i["x"], i["W"], i["b"], i["alpha"], self.H_res, self.H_pre,
                                 self.H_post, self.h, self.ws)
        mhcl.mhcl_post(d, i["x"], i["y"], self.H_res, self.H_post, self.x_out)

    def backward_separable(self):
        i, d = self.inp, self.d
        mhcl.mhcl_post_bwd(d, i["x"], i["y"], self.H_res, self.H_post, i["g_xout"], self.g_x,
                           self.g_y, self.g_H_res, self.g_H_post)
        mhcl.mhcl_pre_bwd(d, i["x"], self.H_pre, i["g_h"], self.g_x, self.g_H_pre)
        mhcl.mhcl_coeffs_bwd(d, i["x"], i["W"], i["b"], i["alpha"], self.g_H_res, self.g_H_pre,
                             self.g_H_post, self.g_x, self.g_W, self.g_b, self.g_alpha, self.ws)

    def backward_fused(self):
        i, d = self.inp, self.d
        mhcl.mhcl_bwd_fused(d, i["x"], i["y"], i["W"], i["b"], i["alpha"], i["g_xout"], i["g_h"],
                            self.g_x, self.g_y, self.g_W, self.g_b, self.g_alpha, self.ws)

    def step(self):
        """One pass of the whole hot path: forward (two calls around the
        caller's f) and the fused backward."""
        self.forward_fused()
        self.backward_fused()
