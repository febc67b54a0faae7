"""`torch.autograd` front end of the hyper-connection layer (paper Sec. 2 Eq. 1,
Sec. 3.2) and a stack of such layers around caller-supplied layer functions.

Every tensor operation of the layer runs in ``libmhcl.so``; this module only
wires the library calls into autograd's graph.  One layer is

    h     = H_pre x                  (mhcl_fwd_coeffs_pre: coefficients + h)
    y     = f(h)                     (the caller's function, ordinary autograd)
    x_out = H_res x + H_post^T y     (mhcl_post)

and its backward, once the gradient on x_out has arrived, is

    g_y                    = sum_i H_post[i] g_xout[i]   (the pre-aggregate kernel run on g_xout)
    g_h                    = backward of f               (autograd)
    g_x, g_W, g_b, g_alpha = mhcl_bwd_fused(x, y, g_xout, g_h)

The two graph nodes of a layer share a small link object: the node of the post
update hands g_xout and y over to the node of the coefficients, whose backward
runs the fused kernel and returns the whole g_x.  Autograd runs the post node
first because h reaches x_out only through y.

Initialisation follows Sec. 4 ("Initialization"): W = 0, alpha = 0.01,
b_res = -8 except 0 for the identity permutation (or the diagonal in the
Sinkhorn-Knopp form), b_pre = b_post = -1 except +1 for one stream.

The paper does not define how the n streams are created at the network's input
and merged at its output; :class:`HyperConnectionStack` replicates the input
into every stream and sums the streams at the end (a choice, not the paper's).
"""
from __future__ import annotations

import math

import torch

from . import binding as mhcl
from .layer import PHASE_G_X, PHASE_G_XOUT, PHASE_X, empty_stream


class _Link:
    """What the post node leaves for the coefficient node of the same layer."""
    __slots__ = ("y", "g_xout", "H_pre", "ws", "g_x_phase", "perm")

    def __init__(self, g_x_phase=PHASE_G_X, perm=None):
        self.y = self.g_xout = self.H_pre = self.ws = None
        self.g_x_phase = g_x_phase
        self.perm = perm      # int8 [K, n] table of the permutation-subset form, else None


def _desc(x, res_mode, sk_iters, eps, perm=None):
    T, n, C = x.shape
    io = {torch.bfloat16: mhcl.BF16, torch.float32: mhcl.F32}[x.dtype]
    return mhcl.Desc(n, C, T, io, res_mode, sk_iters, eps, perm)


class _CoeffsPre(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, W, b, alpha, link, res_mode, sk_iters, eps):
        d = _desc(x, res_mode, sk_iters, eps, link.perm)
        T, n, C = x.shape
        f = torch.float32
        H_res = torch.empty(T, n, n, device=x.device, dtype=f)
        H_pre = torch.empty(T, n, device=x.device, dtype=f)
        H_post = torch.empty(T, n, device=x.device, dtype=f)
        h = torch.empty(T, C, device=x.device, dtype=x.dtype)
        ws = mhcl.new_workspace(d, mhcl.OP_FWD_COEFFS_PRE, x.device)
        mhcl.mhcl_fwd_coeffs_pre(d, x, W, b, alpha, H_res, H_pre, H_post, h, ws)
        ctx.save_for_backward(x, W, b, alpha)
        ctx.link, ctx.d = link, d
        link.H_pre = H_pre
        ctx.mark_non_differentiable(H_pre)
        return h, H_res, H_post, H_pre

    @staticmethod
    def backward(ctx, g_h, _g_H_res, _g_H_post, _g_H_pre):
        x, W, b, alpha = ctx.saved_tensors
        d, link = ctx.d, ctx.link
        T, n, C = x.shape
        if link.y is None:
            raise RuntimeError("hyper-connection backward: the post update of this layer was never run")
        g_xout = link.g_xout if link.g_xout is not None else torch.zeros_like(x)
        g_h = torch.zeros(T, C, device=x.device, dtype=x.dtype) if g_h is None else g_h.contiguous()
        f = torch.float32
        g_x = empty_stream(x.shape, x.dtype, x.device, link.g_x_phase)
        g_W, g_b = torch.empty_like(W, dtype=f), torch.empty_like(b, dtype=f)
        g_alpha = torch.empty(3, device=x.device, dtype=f)
        ws = mhcl.new_workspace(d, mhcl.OP_BWD_FUSED, x.device)
        # g_y went out through the post node already: not asked for again
        mhcl.mhcl_bwd_fused(d, x, link.y, W, b, alpha, g_xout, g_h, g_x, None, g_W, g_b, g_alpha, ws)
        link.y = link.g_xout = None
        return g_x, g_W, g_b, g_alpha, None, None, None, None


class _Post(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, y, H_res, H_post, link, res_mode, sk_iters, eps):
        d = _desc(x, res_mode, sk_iters, eps, link.perm)
        y = y.contiguous()
        x_out = empty_stream(x.shape, x.dtype, x.device, PHASE_X)
        mhcl.mhcl_post(d, x, y, H_res, H_post, x_out)
        ctx.save_for_backward(H_res, H_post)
        ctx.link, ctx.d = link, d
        link.y = y
        return x_out

    @staticmethod
    def backward(ctx, g_xout):
        H_res, H_post = ctx.saved_tensors
        d, link = ctx.d, ctx.link
        g_xout = g_xout.contiguous()
        link.g_xout = g_xout
        g_y = torch.empty(d.T, d.C, device=g_xout.device, dtype=g_xout.dtype)
        mhcl.mhcl_pre(d, g_xout, H_post, g_y)            # g_y = sum_i H_post[i] g_xout[i]
        # x and the coefficients get their gradients from the coefficient node
        # (fused kernel); zeros here only keep that node in the graph.
        return None, g_y, torch.zeros_like(H_res), torch.zeros_like(H_post), None, None, None, None


def init_params(n: int, C: int, res_mode: int = mhcl.RES_LITE, one_index: int = 0, device="cuda",
                n_perm: int = 0):
    """W, b, alpha at the paper's initialisation (Sec. 4, "Initialization").  For a permutation
    subset (``n_perm`` rows) the identity is expected as the table's first row."""
    R = {mhcl.RES_LITE: math.factorial(n), mhcl.RES_SK: n * n, mhcl.RES_SUBSET: n_perm}[res_mode]
    b = torch.full((R + 2 * n,), -1.0, dtype=torch.float32)
    b[:R] = -8.0
    if res_mode in (mhcl.RES_LITE, mhcl.RES_SUBSET):
        b[0] = 0.0                         # the identity: first in lexicographic order / first row of the table
    else:
        b[:R:n + 1] = 0.0                  # the diagonal
    b[R + one_index] = 1.0
    b[R + n + one_index] = 1.0
    W = torch.zeros(n * C, R + 2 * n, dtype=torch.float32)
    alpha = torch.full((3,), 0.01, dtype=torch.float32)
    return W.to(device), b.to(device), alpha.to(device)


class HyperConnection(torch.nn.Module):
    """One layer: ``x_out = H_res x + H_post^T f(H_pre x)`` on ``x [T, n, C]``."""

    def __init__(self, n: int, C: int, res_mode: str = "lite", sk_iters: int = 20, eps: float = 1e-6,
                 one_index: int = 0, device="cuda", layer_index: int = 0, perm=None):
        """res_mode: "lite" (all n! permutations), "sk" (Sinkhorn-Knopp) or "subset" (Sec. 5: only
        the K permutations in ``perm``, an int8 tensor [K, n] with the identity as its first row,
        n up to 8)."""
        super().__init__()
        self.n, self.C = n, C
        if (res_mode == "subset") != (perm is not None):
            raise ValueError("perm goes with res_mode 'subset', and only with it")
        # g_x of this layer is g_xout of the one below: alternate the two gradient phases
        # so that x, g_xout and g_x of a layer all differ (see layer.empty_stream)
        self.g_x_phase = PHASE_G_X if layer_index % 2 == 0 else PHASE_G_XOUT
        self.res_mode = {"lite": mhcl.RES_LITE, "sk": mhcl.RES_SK, "subset": mhcl.RES_SUBSET}[res_mode]
        self.sk_iters, self.eps = sk_iters, eps
        if perm is not None:
            self.register_buffer("perm", perm.to(device=device, dtype=torch.int8).contiguous())
        else:
            self.perm = None
        W, b, alpha = init_params(n, C, self.res_mode, one_index, device,
                                  n_perm=0 if perm is None else int(perm.shape[0]))
        self.W, self.b, self.alpha = (torch.nn.Parameter(t) for t in (W, b, alpha))

    def forward(self, x: torch.Tensor, f):
        if x.dim() != 3 or x.shape[1] != self.n or x.shape[2] != self.C:
            raise ValueError(f"x must be [T, {self.n}, {self.C}], got {tuple(x.shape)}")
        x = x.contiguous()
        link = _Link(self.g_x_phase, self.perm)
        cfg = (self.res_mode, self.sk_iters, self.eps)
        h, H_res, H_post, _ = _CoeffsPre.apply(x, self.W, self.b, self.alpha, link, *cfg)
        y = f(h)
        return _Post.apply(x, y, H_res, H_post, link, *cfg)


class HyperConnectionStack(torch.nn.Module):
    """``len(fs)`` layers around the callables ``fs``.  Input ``[T, C]`` is
    copied into the n streams, the output is the sum of the streams: the paper
    leaves both ends open, this is one choice."""

    def __init__(self, n: int, C: int, fs, res_mode: str = "lite", device="cuda", **kw):
        super().__init__()
        self.n = n
        self.fs = list(fs)
        self.mods = torch.nn.ModuleList([f for f in self.fs if isinstance(f, torch.nn.Module)])
        self.layers = torch.nn.ModuleList(
            [HyperConnection(n, C, res_mode, one_index=l % n, device=device, layer_index=l, **kw)
             for l in range(len(self.fs))])

    def forward(self, x0: torch.Tensor):
        x = x0.unsqueeze(1).expand(-1, self.n, -1).contiguous()
        for layer, f in zip(self.layers, self.fs):
            x = layer(x, f)
        return x.sum(dim=1)
