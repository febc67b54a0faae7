"""GPU parity of the permutation-subset form (Sec. 5, larger n: K chosen
permutations from a run-time table, n up to 8) against the fp64 oracle,
through the C ABI; tolerances as in test_gpu_parity.py.
"""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
import paper_2601_05732_amd as mhcl
from gpu_harness import GpuLayer, desc_for, oracle_reference, rel_err, to_np64
from test_gpu_parity import _check_backward, _check_forward, _tols

pytestmark = pytest.mark.gpu


def _wl(name, **kw):
    base = dict(name=name, n=6, C=64, T=100, io="bf16", res_mode="subset", n_perm=12)
    base.update(kw)
    return si.Workload(**base)


CASES = [
    _wl("n6_k12"),
    _wl("n8_k32_f32", n=8, C=24, T=37, io="f32", n_perm=32),
    _wl("n8_k120", n=8, C=128, T=130, n_perm=120),          # 136 logits: nine MFMA logit tiles
    _wl("n7_k40", n=7, C=64, T=65, n_perm=40),              # 54 logits: 4 logit tiles
    _wl("n8_k64", n=8, C=64, T=150, n_perm=64),             # 80 logits: 5 tiles
    _wl("n8_k96", n=8, C=128, T=77, n_perm=96),             # 112 logits: 7 tiles
    _wl("n6_k100", n=6, C=192, T=129, n_perm=100),          # 112 logits, C not a power of two
    _wl("n4_k5", n=4, C=256, T=333, n_perm=5),
    _wl("n5_k1", n=5, C=64, T=20, n_perm=1),                # one permutation: H_res is that matrix
    _wl("n1", n=1, C=64, T=9, n_perm=1),
    _wl("n6_c4096", n=6, C=4096, T=40, n_perm=24),
]


@pytest.mark.parametrize("wl", CASES, ids=lambda w: w.name)
def test_subset_forward_and_backward_match_oracle(wl):
    print(f"case {wl}", flush=True)
    inp = si.make_inputs(wl, seed=1, device="cuda")
    ref = oracle_reference(inp, wl)
    L = GpuLayer(desc_for(wl, perm=inp["perm"]), inp)
    L.forward_separable()
    torch.cuda.synchronize()
    _check_forward(L, ref, wl)
    sep = {k: getattr(L, k).clone() for k in ("H_res", "H_pre", "H_post", "h", "x_out")}
    L.forward_fused()
    torch.cuda.synchronize()
    _check_forward(L, ref, wl)
    for k, v in sep.items():
        assert torch.equal(getattr(L, k), v), k
    L.backward_fused()
    torch.cuda.synchronize()
    _check_backward(L, ref, wl)
    fused_gx = to_np64(L.g_x)
    L.backward_separable()
    torch.cuda.synchronize()
    t_out = _tols(wl)[0]
    assert rel_err(to_np64(L.g_x), fused_gx) <= (t_out if wl.io == "f32" else 2 * t_out)
    _check_backward(L, ref, wl)      # the separable chain's g_x, g_y and parameter gradients
    if wl.n_perm == 1:
        sig = inp["perm"].cpu().numpy()[0]
        P = np.zeros((wl.n, wl.n)); P[np.arange(wl.n), sig] = 1
        assert np.array_equal(to_np64(L.H_res), np.broadcast_to(P, (wl.T, wl.n, wl.n)))


def test_all_permutations_in_order_reproduce_the_full_form():
    """K = n! rows in lexicographic order: the same matrices as the compile-time table."""
    n, C, T = 4, 256, 200
    full = si.Workload("full", n=n, C=C, T=T)
    sub = si.Workload("sub", n=n, C=C, T=T, res_mode="subset", n_perm=24)
    inp = si.make_inputs(full, seed=2, device="cuda")
    perm = torch.from_numpy(oracle.perm_table(n).astype(np.int8)).cuda()
    Lf = GpuLayer(desc_for(full), inp)
    Ls = GpuLayer(desc_for(sub, perm=perm), inp)
    for L in (Lf, Ls):
        L.forward_fused()
        L.backward_fused()
    torch.cuda.synchronize()
    for k in ("H_pre", "H_post"):
        assert torch.equal(getattr(Lf, k), getattr(Ls, k)), k
    assert rel_err(to_np64(Ls.H_res), to_np64(Lf.H_res)) <= 1e-6       # other summation order
    for k, tol in (("h", 0.0), ("x_out", 2e-2), ("g_x", 2e-2), ("g_y", 2e-2), ("g_W", 2e-4), ("g_b", 2e-4)):
        assert rel_err(to_np64(getattr(Ls, k)), to_np64(getattr(Lf, k))) <= tol, k


def test_subset_descriptor_validation():
    import ctypes
    perm = torch.zeros(4, 6, dtype=torch.int8, device="cuda")
    ok = mhcl.Desc(6, 64, 10, mhcl.BF16, mhcl.RES_SUBSET, perm=perm)
    assert mhcl.lib().mhcl_validate(ctypes.byref(ok.c)) == 0 and mhcl.logit_count(ok) == 4 + 12
    bad = mhcl.Desc(6, 64, 10, mhcl.BF16, mhcl.RES_SUBSET)                # no table
    assert mhcl.lib().mhcl_validate(ctypes.byref(bad.c)) == 1
    bad = mhcl.Desc(9, 64, 10, mhcl.BF16, mhcl.RES_SUBSET, perm=torch.zeros(4, 9, dtype=torch.int8, device="cuda"))
    assert mhcl.lib().mhcl_validate(ctypes.byref(bad.c)) == 1
    bad = mhcl.Desc(6, 64, 10, mhcl.BF16, mhcl.RES_SUBSET, perm=torch.zeros(129, 6, dtype=torch.int8, device="cuda"))
    assert mhcl.lib().mhcl_validate(ctypes.byref(bad.c)) == 1
    assert mhcl.lib().mhcl_validate(ctypes.byref(mhcl.Desc(6, 64, 10).c)) == 1     # n = 6 needs the subset form
