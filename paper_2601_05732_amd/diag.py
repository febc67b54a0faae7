"""Doubly-stochasticity diagnostics on the GPU (paper Sec. 3.1 and Sec. 4.3).

For a stack of L synthetic layers this collects, per token, the residual
matrices H_res of every layer (permutation form or 20-step Sinkhorn-Knopp),
the relative range log(1/nu) of the Sinkhorn-Knopp input (Eq. 3), the column
sums and l1 errors of each matrix ("per-matrix" in Fig. 2) and of the product
over the layers ("prod").  All arithmetic runs in ``libmhcl.so``
(``mhcl_coeffs``, ``mhcl_logits``, ``mhcl_ds_chain``); this module only
allocates, draws inputs and summarises.

The paper takes these statistics from trained models; those weights are not
available, so each layer gets its own seeded Gaussian x, W, b and the spread
of the residual logits is swept through alpha_res instead.

The package draws no inputs itself: ``layer_stack`` takes them, or a callable
that draws layer l's; the command line below uses the repository's seeded
generator (``synth_inputs`` at the repository root).

Run ``python -m paper_2601_05732_amd.diag`` for a table.
"""
from __future__ import annotations

import argparse

import torch

from . import binding as mhcl
from .layer import desc_for


def layer_stack(wl, L: int, inputs, device: str = "cuda"):
    """H [L,T,n,n], z [L,T,M], log_inv_nu [L,T] for L layers.  ``wl`` is a workload
    record (fields n, C, T, M, io, res_mode, sk_iters, eps); ``inputs`` is a list of L
    dicts with the GPU tensors x, W, b, alpha of each layer, or a callable ``l -> dict``."""
    d = desc_for(wl)
    f = torch.float32
    H = torch.empty(L, wl.T, wl.n, wl.n, device=device, dtype=f)
    z = torch.empty(L, wl.T, wl.M, device=device, dtype=f)
    spread = torch.empty(L, wl.T, device=device, dtype=f)
    # the library wants 16-byte aligned pointers, which a slice H[l] need not be:
    # each call writes its own buffers, copied into the stack afterwards
    Hl = torch.empty(wl.T, wl.n, wl.n, device=device, dtype=f)
    zl = torch.empty(wl.T, wl.M, device=device, dtype=f)
    sl = torch.empty(wl.T, device=device, dtype=f)
    Hp = torch.empty(wl.T, wl.n, device=device, dtype=f)
    Hq = torch.empty(wl.T, wl.n, device=device, dtype=f)
    ws = mhcl.new_workspace(d, mhcl.OP_COEFFS, device)
    for l in range(L):
        inp = inputs(l) if callable(inputs) else inputs[l]
        mhcl.mhcl_coeffs(d, inp["x"], inp["W"], inp["b"], inp["alpha"], Hl, Hp, Hq, ws)
        mhcl.mhcl_logits(d, inp["x"], inp["W"], inp["b"], inp["alpha"], zl, sl, ws)
        H[l].copy_(Hl)
        z[l].copy_(zl)
        spread[l].copy_(sl)
    return H, z, spread


def chain(H: torch.Tensor) -> dict:
    """Runs mhcl_ds_chain on H [L,T,n,n]; returns its five outputs."""
    L, T, n, _ = H.shape
    e = lambda *s: torch.empty(s, device=H.device, dtype=torch.float32)
    out = dict(colsum=e(L, T, n), l1=e(L, T), prod=e(T, n, n), prod_colsum=e(L, T, n), prod_l1=e(L, T))
    mhcl.mhcl_ds_chain(n, L, T, H, out["colsum"], out["l1"], out["prod"], out["prod_colsum"],
                       out["prod_l1"])
    return out


def _q(t: torch.Tensor, qs=(0.5, 0.99, 1.0)):
    t = t.flatten().double()
    return [float(torch.quantile(t, q)) if q < 1.0 else float(t.max()) for q in qs]


def report(draw, layers=(6, 24), alphas=(1.0, 4.0, 8.0, 16.0), device="cuda"):
    """Prints, for each alpha_res and depth, quantiles of log(1/nu), of the
    per-matrix column-sum deviation and l1 error, and of the same for the
    product over the layers, for Sinkhorn-Knopp (20) and the permutation form.
    ``draw(mode, alpha_res)`` returns (workload record, callable l -> inputs of layer l)."""
    rows = []
    for a in alphas:
        for mode in ("sk", "lite"):
            wl, inputs = draw(mode, a)
            Lmax = max(layers)
            H, _, spread = layer_stack(wl, Lmax, inputs, device=device)
            out = chain(H)
            for L in layers:
                dev1 = (out["colsum"][:L] - 1).abs()
                devp = (out["prod_colsum"][L - 1] - 1).abs()
                rows.append((a, mode, L, _q(spread[:L]), float((spread[:L] > 30).double().mean()),
                             _q(dev1), _q(out["l1"][:L]), _q(devp), _q(out["prod_l1"][L - 1])))
    torch.cuda.synchronize()
    hdr = ("alpha_res mode  L | log(1/nu) p50/p99/max  frac>30 | per-matrix |colsum-1| p50/p99/max | "
           "l1 p50/p99/max | prod |colsum-1| p50/p99/max | prod l1 p50/p99/max")
    print(hdr)
    f3 = lambda v: "/".join(f"{x:.3g}" for x in v)
    for a, mode, L, sp, fr, d1, l1, dp, lp in rows:
        print(f"{a:8.1f} {mode:5s} {L:2d} | {f3(sp):>22s}  {fr:6.3f} | {f3(d1):>26s} | {f3(l1):>22s} | "
              f"{f3(dp):>26s} | {f3(lp):>22s}")
    return rows


if __name__ == "__main__":
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--n", type=int, default=4)
    ap.add_argument("--C", type=int, default=512)
    ap.add_argument("--T", type=int, default=16384)
    args = ap.parse_args()
    import os
    import sys
    sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    import synth_inputs as si      # the repository's seeded input generator (command line only)

    def _draw(mode, a):
        wl = si.Workload(f"diag_{mode}", n=args.n, C=args.C, T=args.T, res_mode=mode,
                         alpha=(a, 1.0, 1.0), backward=False)
        return wl, (lambda l: si.make_inputs(wl, seed=100 + l, device="cuda"))

    report(_draw)
