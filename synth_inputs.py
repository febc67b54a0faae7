"""Seeded synthetic inputs for the mHC-lite hyper-connection path.

This module only draws random tensors of the shapes and distributions used
by the workloads; it contains none of the method's arithmetic and is the one
piece of code that both the CPU oracle's tests and the HIP path's tests use,
so that both sides see identical input bits.

The paper trains on activations of a language model (Sec. 4, App. A); those
need datasets and weights that are not available, so i.i.d. Gaussian streams
of the same shapes stand in for them:

    x   ~ N(0, 1)        [T, n, C]   residual streams (Eq. 1)
    W   ~ N(0, 0.02^2)   [n*C, M]    fused projection, columns [res | pre | post]
    b   ~ N(0, b_std^2)  [M]
    y   ~ N(0, 1)        [T, C]      stand-in for the layer output f(H_pre x)
    g_xout ~ N(0, 1)     [T, n, C]   upstream gradient on x_{l+1}
    g_h    ~ N(0, 1)     [T, C]      upstream gradient on H_pre x

M = n! + 2n for the permutation parameterisation (Sec. 3.2) and n^2 + 2n for
the Sinkhorn-Knopp one (Eq. 2).  alpha = (1, 1, 1) unless the caller asks for
the paper's initialisation (Sec. 4, "Initialization").
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np
import torch


@dataclass(frozen=True)
class Workload:
    name: str
    n: int
    C: int
    T: int
    io: str = "bf16"          # "bf16" | "f32": dtype of every stream tensor
    b_std: float = 0.1
    res_mode: str = "lite"    # "lite" | "sk" | "subset"
    sk_iters: int = 20
    eps: float = 1e-6
    alpha: tuple = (1.0, 1.0, 1.0)
    backward: bool = True
    n_perm: int = 0           # "subset": number of permutations kept

    @property
    def M(self) -> int:
        if self.res_mode == "lite":
            return math.factorial(self.n) + 2 * self.n
        if self.res_mode == "subset":
            return self.n_perm + 2 * self.n
        return self.n * self.n + 2 * self.n

    @property
    def nC(self) -> int:
        return self.n * self.C


# The five stated workloads: a tiny all-fp32 case and four bf16 cases.
WORKLOADS = {
    "tiny_f32": Workload("tiny_f32", n=4, C=64, T=256, io="f32", b_std=0.0),
    "n4_c2048_fwd": Workload("n4_c2048_fwd", n=4, C=2048, T=32768, backward=False),
    "n4_c4096": Workload("n4_c4096", n=4, C=4096, T=32768),
    "n3_c1024": Workload("n3_c1024", n=3, C=1024, T=65536),
    "n5_c2560": Workload("n5_c2560", n=5, C=2560, T=16384),
    "n4_c4096_sk": Workload("n4_c4096_sk", n=4, C=4096, T=32768, res_mode="sk"),
    # The paper's own hidden sizes (App. A, scale-specific hyperparameters: S / M / L)
    # at its per-GPU micro-batch of 16 sequences x 1024 tokens (App. A, shared
    # hyperparameters), n = 4 (Sec. 4).
    "paper_s_c512": Workload("paper_s_c512", n=4, C=512, T=16384),
    "paper_m_c768": Workload("paper_m_c768", n=4, C=768, T=16384),
    "paper_l_c1024": Workload("paper_l_c1024", n=4, C=1024, T=16384),
    # Larger n with a subset of the permutations (Sec. 5): 8 streams, 64 of the 8! matrices.
    "n8_c1024_k64": Workload("n8_c1024_k64", n=8, C=1024, T=16384, res_mode="subset", n_perm=64),
}


def _stream_dtype(io: str) -> torch.dtype:
    return {"bf16": torch.bfloat16, "f32": torch.float32}[io]


def _randn(shape, gen, device, dtype, std=1.0, chunk_rows=4096):
    """N(0, std^2) drawn in fp32 and rounded (nearest-even) to `dtype`.

    Large tensors are drawn in row chunks so that the fp32 staging buffer
    stays small next to the result.
    """
    out = torch.empty(shape, device=device, dtype=dtype)
    if out.numel() == 0:
        return out
    flat = out.view(shape[0], -1)
    for r0 in range(0, shape[0], chunk_rows):
        r1 = min(shape[0], r0 + chunk_rows)
        blk = torch.randn((r1 - r0, flat.shape[1]), generator=gen, device=device,
                          dtype=torch.float32)
        if std != 1.0:
            blk.mul_(std)
        flat[r0:r1].copy_(blk)
    return out


def subset_permutations(n: int, K: int, seed: int = 0) -> np.ndarray:
    """K distinct permutations of 0..n-1, the identity first, the rest drawn
    uniformly (Sec. 5: "sampling a subset of permutation matrices"), int8 [K, n]."""
    assert 1 <= K <= math.factorial(n)
    rng = np.random.default_rng(seed)
    rows = [tuple(range(n))]
    seen = set(rows)
    while len(rows) < K:
        p = tuple(rng.permutation(n).tolist())
        if p not in seen:
            seen.add(p)
            rows.append(p)
    return np.array(rows, dtype=np.int8)


def make_inputs(wl: Workload, seed: int = 0, device: str = "cpu") -> dict:
    """Draw x, W, b, alpha, y, g_xout, g_h for `wl`, in that order, from one
    generator seeded with `seed` on `device`.

    The same (seed, device) always yields the same bits; a test hands those
    bits to both implementations (copying to the host where needed).
    """
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    sd = _stream_dtype(wl.io)
    n, C, T, M = wl.n, wl.C, wl.T, wl.M
    d = {}
    d["x"] = _randn((T, n, C), gen, device, sd)
    d["W"] = _randn((n * C, M), gen, device, torch.float32, std=0.02)
    if wl.b_std > 0:
        d["b"] = _randn((M,), gen, device, torch.float32, std=wl.b_std)
    else:
        d["b"] = torch.zeros((M,), device=device, dtype=torch.float32)
    d["alpha"] = torch.tensor(wl.alpha, device=device, dtype=torch.float32)
    d["y"] = _randn((T, C), gen, device, sd)
    if wl.backward:
        d["g_xout"] = _randn((T, n, C), gen, device, sd)
        d["g_h"] = _randn((T, C), gen, device, sd)
    if wl.res_mode == "subset":
        d["perm"] = torch.from_numpy(subset_permutations(n, wl.n_perm, seed)).to(device)
    return d


def paper_init_params(n: int, C: int, res_mode: str = "lite", one_index: int = 0):
    """Parameters at the paper's initialisation (Sec. 4, "Initialization"):
    W = 0, alpha = 0.01, b_pre = b_post = -1 except one entry (+1), b_res = -8
    except the identity permutation (lite) or the diagonal (SK), which are 0.

    Returns numpy float32 arrays (W, b, alpha) in the fused column order
    [res | pre | post].  For "lite" the identity is permutation index 0 in
    lexicographic order.
    """
    if res_mode == "lite":
        R = math.factorial(n)
        b_res = np.full(R, -8.0, dtype=np.float32)
        b_res[0] = 0.0
    else:
        R = n * n
        b_res = np.full(R, -8.0, dtype=np.float32)
        b_res[:: n + 1] = 0.0
    b_gate = np.full(n, -1.0, dtype=np.float32)
    b_gate[one_index] = 1.0
    b = np.concatenate([b_res, b_gate, b_gate]).astype(np.float32)
    W = np.zeros((n * C, R + 2 * n), dtype=np.float32)
    alpha = np.full(3, 0.01, dtype=np.float32)
    return W, b, alpha


def small_case(n: int, C: int, T: int, seed: int = 0, res_mode: str = "lite",
               w_std: float = 0.3, b_std: float = 0.3):
    """Tiny fp64 numpy inputs for oracle-only checks (finite differences,
    brute force).  Larger W/b spreads than the workloads so that softmax and
    the gates are far from both uniform and saturated.
    """
    rng = np.random.default_rng(seed)
    R = math.factorial(n) if res_mode == "lite" else n * n
    M = R + 2 * n
    return {
        "x": rng.standard_normal((T, n, C)),
        "W": w_std * rng.standard_normal((n * C, M)),
        "b": b_std * rng.standard_normal(M),
        "alpha": 0.5 + rng.random(3),
        "y": rng.standard_normal((T, C)),
        "g_xout": rng.standard_normal((T, n, C)),
        "g_h": rng.standard_normal((T, C)),
    }
