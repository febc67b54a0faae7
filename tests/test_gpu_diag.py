"""GPU parity of the diagnostics entry points (mhcl_logits, mhcl_ds_chain)
against the fp64 oracle, through the C ABI, plus the paper's 3x3
Sinkhorn-Knopp example run on the GPU.

mhcl_ds_chain is fp32: its inputs (H from the GPU coefficients) go to the
oracle bit for bit, so the difference is the rounding of at most L n x n
products, each a sum of n terms: bound L * n * 2^-24 relative to the product's
size (1.2e-5 at L = 24, n = 4); the tests allow 2e-5.  Column sums and l1
errors of single matrices are sums of n terms: 1e-6.

mhcl_logits: 1e-5 for f32 streams.  With bf16 streams the projection runs on
the matrix cores with W carried as two bf16 numbers (16 significant bits), a
relative error of up to 2^-17 = 7.6e-6 per product; the logits are not squashed
by a softmax or a logistic function as H is, so the worst of a few thousand
logits reaches about 1e-5 of the logits' rms; 3e-5 is allowed there.
"""
import dataclasses
import math
import os

import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
import paper_2601_05732_amd as mhcl
from paper_2601_05732_amd import diag
from gpu_harness import desc_for, rel_err, to_np64

pytestmark = pytest.mark.gpu


def _wl(name, **kw):
    base = dict(n=4, C=64, T=100, io="bf16", backward=False)
    base.update(kw)
    return si.Workload(name, **base)


LOGIT_CASES = [
    _wl("lite_n4", C=256, T=333),
    _wl("sk_n4", C=256, T=129, res_mode="sk", alpha=(6.0, 1.0, 1.0)),
    _wl("lite_n5", n=5, C=128, T=150),
    _wl("sk_n3_f32", n=3, C=40, T=19, io="f32", res_mode="sk"),
    _wl("sk_n5", n=5, C=64, T=70, res_mode="sk", alpha=(10.0, 0.5, 2.0)),
    _wl("lite_c4096", C=4096, T=70),
]


@pytest.mark.parametrize("wl", LOGIT_CASES, ids=lambda w: w.name)
def test_logits_and_relative_range_match_oracle(wl):
    print(f"case {wl}", flush=True)
    inp = si.make_inputs(wl, seed=3, device="cuda")
    d = desc_for(wl)
    z = torch.empty(wl.T, wl.M, device="cuda")
    spread = torch.empty(wl.T, device="cuda")
    ws = mhcl.binding.new_workspace(d, mhcl.OP_COEFFS)
    mhcl.mhcl_logits(d, inp["x"], inp["W"], inp["b"], inp["alpha"], z, spread, ws)
    torch.cuda.synchronize()
    ref = oracle.logits(to_np64(inp["x"]), to_np64(inp["W"]), to_np64(inp["b"]), to_np64(inp["alpha"]),
                        eps=wl.eps, res_mode=wl.res_mode)
    tol = 1e-5 if wl.io == "f32" else 3e-5
    assert rel_err(to_np64(z), ref) <= tol
    if wl.res_mode == "sk":
        R = wl.n * wl.n
        nu = oracle.relative_range(np.exp(ref[:, :R]).reshape(wl.T, wl.n, wl.n))   # Eq. 3 on exp(mat(z_res))
        assert rel_err(to_np64(spread), np.log(1.0 / nu)) <= 2 * tol
    # either output alone
    z2 = torch.empty_like(z)
    s2 = torch.empty_like(spread)
    mhcl.mhcl_logits(d, inp["x"], inp["W"], inp["b"], inp["alpha"], z2, None, ws)
    mhcl.mhcl_logits(d, inp["x"], inp["W"], inp["b"], inp["alpha"], None, s2, ws)
    torch.cuda.synchronize()
    assert torch.equal(z2, z) and torch.equal(s2, spread)


def test_sk_worked_example_from_the_paper_on_the_gpu(golden_dir):
    """Sec. 1: the 3x3 matrix with alpha = 1e-13 after 20 iterations, fed in
    through the bias (W = 0, so the logits are log of the matrix)."""
    kv = {}
    for line in open(os.path.join(golden_dir, "sk_example_sec1.txt")):
        if "=" in line and not line.startswith("#"):
            k, v = line.split("=", 1)
            kv[k.strip()] = v.strip()
    al = float(kv["alpha"])
    X0 = np.array([[0.5, al, al], [0.5, al, al], [al, 1.0, 1.0]])
    n, C, T = 3, 64, 5
    wl = _wl("e1", n=n, C=C, T=T, res_mode="sk", sk_iters=int(kv["iters"]))
    inp = si.make_inputs(wl, seed=0, device="cuda")
    inp["W"].zero_()
    inp["b"].zero_()
    inp["b"][: n * n] = torch.tensor(np.log(X0).reshape(-1), dtype=torch.float32)
    H, z, spread = diag.layer_stack(wl, 24, [inp] * 24)
    out = diag.chain(H)
    torch.cuda.synchronize()
    Hn = to_np64(H)
    printed = np.array([float(v) for v in kv["out"].split()]).reshape(3, 3)
    half_ulp = np.array([[0.005, 0.0005, 0.0005]] * 2 + [[0.05, 0.05, 0.05]])
    assert np.all(np.abs(Hn[0, 0] - printed) <= half_ulp), Hn[0, 0]
    assert np.all(Hn == Hn[0, 0])                          # the same matrix at every token and layer
    assert rel_err(Hn[0, 0], oracle.sk(np.exp(to_np64(z)[0, 0, :9]).reshape(3, 3), 20)) <= 1e-5
    want = [float(v) for v in kv["colsums_from_printed_matrix"].split()]
    assert np.allclose(to_np64(out["colsum"])[0, 0], want, atol=0.006)
    assert abs(float(spread[0, 0]) - math.log(1 / al)) < 1e-4      # log(1/nu) = log(1e13) = 29.93
    ref = oracle.ds_chain(Hn)
    for k in out:
        assert rel_err(to_np64(out[k]), ref[k]) <= 2e-5, k
    # the deviation compounds with depth (Sec. 3.1): first column sum of the product grows
    pc = to_np64(out["prod_colsum"])[:, 0, 0]
    assert pc[23] > pc[5] > pc[0] > 1.8


CHAIN_CASES = [
    (_wl("sk_n4_illcond", T=1000, res_mode="sk", alpha=(16.0, 1.0, 1.0)), 24),
    (_wl("sk_n4_mild", T=333, res_mode="sk"), 6),
    (_wl("lite_n4", T=1000, alpha=(16.0, 1.0, 1.0)), 24),
    (_wl("sk_n3", n=3, T=129, res_mode="sk", alpha=(12.0, 1.0, 1.0)), 12),
    (_wl("sk_n5", n=5, T=200, res_mode="sk", alpha=(12.0, 1.0, 1.0)), 24),
    (_wl("lite_n5", n=5, T=77), 3),
    (_wl("sk_n1", n=1, T=5, res_mode="sk"), 2),
    (_wl("sk_n2_one_layer", n=2, T=64, res_mode="sk", alpha=(20.0, 1.0, 1.0)), 1),
]


@pytest.mark.parametrize("wl,L", CHAIN_CASES, ids=lambda v: v.name if isinstance(v, si.Workload) else str(v))
def test_chain_matches_oracle(wl, L):
    print(f"case {wl} L={L}", flush=True)
    H, _, _ = diag.layer_stack(wl, L, lambda l: si.make_inputs(wl, seed=40 + l, device="cuda"))
    out = diag.chain(H)
    torch.cuda.synchronize()
    ref = oracle.ds_chain(to_np64(H))
    assert rel_err(to_np64(out["colsum"]), ref["colsum"]) <= 1e-6
    assert np.abs(to_np64(out["l1"]) - ref["l1"]).max() <= 2e-6 * wl.n
    for k in ("prod", "prod_colsum"):
        assert rel_err(to_np64(out[k]), ref[k]) <= 2e-5, k
    scale = max(1.0, float(np.abs(ref["prod_colsum"]).max()))
    assert np.abs(to_np64(out["prod_l1"]) - ref["prod_l1"]).max() <= 2e-5 * 2 * wl.n * scale
    if wl.res_mode == "lite":     # exactly doubly stochastic at every depth (Theorem 3.1)
        # up to fp32 rounding: each factor's row and column sums are within 1e-6 of 1, those
        # deviations add up at most linearly over the L factors, plus n 2^-24 per product
        assert float(out["prod_l1"].max()) <= 2 * wl.n * L * (1e-6 + wl.n * 2.0 ** -24)
        assert float(out["l1"].max()) <= 2 * wl.n * 1e-6          # every row and column sum within 1e-6
    # only some outputs requested
    only = torch.empty_like(out["prod_colsum"])
    mhcl.mhcl_ds_chain(wl.n, L, wl.T, H, None, None, None, only, None)
    torch.cuda.synchronize()
    assert torch.equal(only, out["prod_colsum"])


def test_depth_statistics_at_the_paper_shape():
    """n = 4, C = 512, 16384 tokens, 24 layers with widely spread residual
    logits: the permutation form stays doubly stochastic through the product,
    20 Sinkhorn-Knopp steps do not (Sec. 3.1, Sec. 4.3); oracle on sampled tokens."""
    T, L = 16384, 24
    res = {}
    for mode in ("lite", "sk"):
        wl = si.Workload("depth_" + mode, n=4, C=512, T=T, res_mode=mode, alpha=(16.0, 1.0, 1.0),
                         backward=False)
        H, _, spread = diag.layer_stack(wl, L, lambda l: si.make_inputs(wl, seed=200 + l, device="cuda"))
        out = diag.chain(H)
        torch.cuda.synchronize()
        pick = torch.tensor([0, 1, 63, 64, 127, 128, 4095, 8191, 8192, T - 65, T - 2, T - 1], device="cuda")
        ref = oracle.ds_chain(to_np64(H[:, pick]))
        for k in ("colsum", "prod_colsum"):
            assert rel_err(to_np64(out[k][:, pick]), ref[k]) <= 2e-5, (mode, k)
        # l1 errors are differences from 1 (pure rounding noise when exact): absolute bounds
        scale = max(1.0, float(np.abs(ref["prod_colsum"]).max()))
        assert np.abs(to_np64(out["l1"][:, pick]) - ref["l1"]).max() <= 2e-6 * 4
        assert np.abs(to_np64(out["prod_l1"][:, pick]) - ref["prod_l1"]).max() <= 2e-5 * 8 * scale
        assert rel_err(to_np64(out["prod"][pick]), ref["prod"]) <= 2e-5
        res[mode] = (out, spread)
    lite, sk = res["lite"][0], res["sk"][0]
    assert float((lite["prod_colsum"] - 1).abs().max()) <= L * (1e-6 + 4 * 2.0 ** -24)   # linear in depth
    assert float((lite["colsum"] - 1).abs().max()) <= 1e-6
    # rows are normalised last, so row sums of every SK matrix and product stay 1 ...
    assert float((sk["prod"].sum(dim=2) - 1).abs().max()) <= 1e-4
    # ... while column sums drift, more so in the product than per matrix
    dev1 = float((sk["colsum"] - 1).abs().max())
    devp = float((sk["prod_colsum"][L - 1] - 1).abs().max())
    print(f"SK(20): max |colsum-1| per matrix {dev1:.3g}, product over {L} layers {devp:.3g}; "
          f"frac log(1/nu)>30: {float((res['sk'][1] > 30).float().mean()):.3f}", flush=True)
    assert dev1 > 1e-3 and devp > dev1
