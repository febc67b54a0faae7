"""GPU parity: libmhcl (through its C ABI) against the fp64 oracle on the same
seeded input bits.

Tolerances (metric: max_e |got - ref| / max(|ref_e|, rms(ref)) per tensor), derived in
gpu_harness.py:
  * f32 streams: 1e-5 on every output;
  * bf16 streams: 2e-2 on bf16 outputs; fp32 coefficients 5e-5; parameter gradients 2e-4;
  * H_res rows and columns sum to 1 within 1e-6 (permutation form).
"""
import numpy as np
import pytest
import torch

import synth_inputs as si
from gpu_harness import (GpuLayer, desc_for, oracle_reference, rel_err, to_np64,
                         TOL_F32, TOL_BF16_OUT, TOL_BF16_COEF, TOL_BF16_PARAM)

pytestmark = pytest.mark.gpu



def _tols(wl):
    if wl.io == "f32":
        return TOL_F32, TOL_F32, TOL_F32
    return TOL_BF16_OUT, TOL_BF16_COEF, TOL_BF16_PARAM


def _check_forward(L, ref, wl, tokens=None):
    t_out, t_coef, _ = _tols(wl)
    sel = (lambda a: a) if tokens is None else (lambda a: a[tokens])
    for name, tol in [("H_res", t_coef), ("H_pre", t_coef), ("H_post", t_coef),
                      ("h", t_out), ("x_out", t_out)]:
        got = sel(to_np64(getattr(L, name)))
        e = rel_err(got, ref[name])
        assert e <= tol, f"{name}: {e:.3e} > {tol}"
    if wl.res_mode in ("lite", "subset"):
        H = to_np64(L.H_res)
        assert np.abs(H.sum(axis=1) - 1).max() <= 1e-6 and np.abs(H.sum(axis=2) - 1).max() <= 1e-6
        assert H.min() >= 0.0


def _check_backward(L, ref, wl, tokens=None, params=True):
    t_out, _, t_par = _tols(wl)
    sel = (lambda a: a) if tokens is None else (lambda a: a[tokens])
    for name in ("g_x", "g_y"):
        e = rel_err(sel(to_np64(getattr(L, name))), ref[name])
        assert e <= t_out, f"{name}: {e:.3e} > {t_out}"
    if params:
        for name in ("g_W", "g_b", "g_alpha"):
            e = rel_err(to_np64(getattr(L, name)), ref[name])
            assert e <= t_par, f"{name}: {e:.3e} > {t_par}"


def _small(name, **kw):
    base = dict(name=name, n=4, C=64, T=256, io="bf16")
    base.update(kw)
    return si.Workload(**base)


SMALL_CASES = [
    si.WORKLOADS["tiny_f32"],                                  # the stated all-fp32 case
    _small("f32_sk", io="f32", res_mode="sk"),
    _small("bf16_n4", C=256, T=333),                           # ragged T
    _small("bf16_n4_sk", C=256, T=129, res_mode="sk"),
    _small("bf16_n1", n=1, C=128, T=67),
    _small("bf16_n2", n=2, C=64, T=130),
    _small("bf16_n3", n=3, C=1024, T=77),
    _small("bf16_n5", n=5, C=96, T=45),
    _small("bf16_n5_sk", n=5, C=64, T=33, res_mode="sk"),
    _small("bf16_n5_c128", n=5, C=128, T=150),                 # 130 logits: nine MFMA logit tiles
    _small("bf16_n5_empty_chunks", n=5, C=64, T=2230),         # 70 token blocks over 64 g_W chunks: 29 stay empty
    _small("f32_n3", n=3, C=40, T=19, io="f32"),
    _small("bf16_c4096", C=4096, T=70),                        # full width, several tiles + tail
    _small("one_token", C=64, T=1),
    _small("f32_c4096", C=4096, T=300, io="f32"),              # f32 streams at full width: 1e-5 holds
                                                               # (the plain projection sums in fp64)
    _small("sk_3iters", C=64, T=40, res_mode="sk", sk_iters=3),
]


@pytest.mark.parametrize("wl", SMALL_CASES, ids=lambda w: w.name)
def test_forward_and_backward_match_oracle(wl):
    print(f"case {wl}", flush=True)
    inp = si.make_inputs(wl, seed=0, device="cuda")
    ref = oracle_reference(inp, wl)
    L = GpuLayer(desc_for(wl), inp)
    L.forward_separable()
    torch.cuda.synchronize()
    _check_forward(L, ref, wl)
    sep = {k: getattr(L, k).clone() for k in ("H_res", "H_pre", "H_post", "h", "x_out")}
    L.forward_fused()
    torch.cuda.synchronize()
    _check_forward(L, ref, wl)
    for k, v in sep.items():      # fused and separable forward agree
        assert rel_err(to_np64(getattr(L, k)), to_np64(v)) <= (1e-6 if k.startswith("H") else _tols(wl)[0])
    L.backward_fused()
    torch.cuda.synchronize()
    _check_backward(L, ref, wl)
    fused_gx = to_np64(L.g_x)
    L.backward_separable()
    torch.cuda.synchronize()
    # the separable chain (post_bwd, pre_bwd, coeffs_bwd) rounds g_x to the stream type three
    # times; it still meets the bound of a bf16 output, and so do its g_y and its parameter
    # gradients (other kernels than the fused call's)
    _check_backward(L, ref, wl)
    t_out = _tols(wl)[0]
    assert rel_err(to_np64(L.g_x), fused_gx) <= (t_out if wl.io == "f32" else 2 * t_out)
    for name, tol in [("g_H_res", _tols(wl)[2]), ("g_H_pre", _tols(wl)[2]), ("g_H_post", _tols(wl)[2])]:
        assert rel_err(to_np64(getattr(L, name)), ref[name]) <= tol, name


def test_paper_initialisation_case():
    # W = 0, alpha = 0.01, init biases (Sec. 4 "Initialization"): coefficients are
    # input independent and the block is almost an ordinary residual connection
    wl = _small("init", C=128, T=50, alpha=(0.01, 0.01, 0.01))
    inp = si.make_inputs(wl, seed=1, device="cuda")
    W, b, al = si.paper_init_params(wl.n, wl.C, "lite", one_index=1)
    inp["W"], inp["b"], inp["alpha"] = (torch.tensor(a, device="cuda") for a in (W, b, al))
    ref = oracle_reference(inp, wl)
    L = GpuLayer(desc_for(wl), inp)
    L.step()
    torch.cuda.synchronize()
    _check_forward(L, ref, wl)
    _check_backward(L, ref, wl, params=False)
    H = to_np64(L.H_res)
    assert abs(H[0, 0, 0] - 0.9940079055) < 1e-6 and abs(H[0, 0, 1] - 0.0019973648) < 1e-7
    # g_W is not identically zero here even though W is (alpha g_z x_hat'^T)
    for name in ("g_W", "g_b", "g_alpha"):
        assert rel_err(to_np64(getattr(L, name)), ref[name]) <= TOL_BF16_PARAM, name


@pytest.mark.parametrize("n,C", [(5, 128), (4, 256)])
def test_weights_of_large_magnitude(n, C):
    # |W| up to a few 1e6 (with alpha small, so that the logits stay ordinary): the n = 5 backward
    # carries W as ONE fp16 part, scaled by a power of two chosen from max |W|; without the
    # scale every entry above 65504 would become infinite in g_x
    s = 3.0e7
    wl = _small(f"bigw_n{n}", n=n, C=C, T=150, alpha=(1 / s, 1 / s, 1 / s))
    inp = si.make_inputs(wl, seed=5, device="cuda")
    inp["W"] = inp["W"] * s
    assert float(inp["W"].abs().max()) > 1e6
    ref = oracle_reference(inp, wl)
    L = GpuLayer(desc_for(wl), inp)
    L.step()
    torch.cuda.synchronize()
    _check_forward(L, ref, wl)
    _check_backward(L, ref, wl)
    assert torch.isfinite(L.g_x.float()).all()


def test_empty_input_is_a_no_op():
    wl = _small("empty", T=0)
    inp = si.make_inputs(wl, seed=0, device="cuda")
    L = GpuLayer(desc_for(wl), inp)
    L.g_W.fill_(7.0); L.g_b.fill_(7.0); L.g_alpha.fill_(7.0)
    L.forward_separable(); L.forward_fused(); L.backward_fused()
    torch.cuda.synchronize()
    assert float(L.g_W.abs().max()) == 0.0 and float(L.g_b.abs().max()) == 0.0
    assert float(L.g_alpha.abs().max()) == 0.0
    L.g_W.fill_(7.0)
    L.backward_separable()
    torch.cuda.synchronize()
    assert float(L.g_W.abs().max()) == 0.0


def test_zero_input_with_eps():
    # all-zero streams: x_hat' = 0, logits equal the bias
    wl = _small("zeros", C=64, T=9)
    inp = si.make_inputs(wl, seed=0, device="cuda")
    inp["x"].zero_()
    ref = oracle_reference(inp, wl)
    L = GpuLayer(desc_for(wl), inp)
    L.step()
    torch.cuda.synchronize()
    _check_forward(L, ref, wl)
    _check_backward(L, ref, wl)


def test_results_are_bitwise_reproducible():
    wl = _small("repro", C=512, T=300)
    inp = si.make_inputs(wl, seed=3, device="cuda")
    L = GpuLayer(desc_for(wl), inp)
    L.step(); torch.cuda.synchronize()
    first = {k: getattr(L, k).clone() for k in ("H_res", "h", "x_out", "g_x", "g_y", "g_W", "g_b", "g_alpha")}
    for _ in range(3):
        L.step(); torch.cuda.synchronize()
        for k, v in first.items():
            assert torch.equal(getattr(L, k), v), k


def test_stream_sum_conservation_full_width():
    # column sums of H_res are 1  =>  sum_i x_out[i] = sum_j x[j] + (sum_i H_post[i]) y
    wl = _small("conserve", C=4096, T=512)
    inp = si.make_inputs(wl, seed=4, device="cuda")
    L = GpuLayer(desc_for(wl), inp)
    L.forward_fused(); torch.cuda.synchronize()
    lhs = L.x_out.double().sum(dim=1)
    rhs = inp["x"].double().sum(dim=1) + L.H_post.double().sum(dim=1, keepdim=True) * inp["y"].double()
    # each of the n outputs is rounded to bf16 once: |err| <= n * 2^-9 * max|x_out|
    assert float((lhs - rhs).abs().max()) <= 4 * 2.0 ** -9 * float(L.x_out.abs().max())


def test_one_hot_weights_give_exact_permutation_matrices():
    # b_res = 0 at one permutation and -1e4 elsewhere, W = 0: H_res must be that
    # permutation matrix exactly (Theorem 3.1, vertices of the Birkhoff polytope)
    import itertools
    wl = _small("onehot", n=4, C=64, T=24)
    inp = si.make_inputs(wl, seed=2, device="cuda")
    inp["W"].zero_()
    perms = list(itertools.permutations(range(4)))
    L = GpuLayer(desc_for(wl), inp)
    for k in (0, 5, 17, 23):
        b = torch.zeros(32, device="cuda")
        b[:24] = -1e4
        b[k] = 0.0
        inp["b"] = b
        L.forward_fused()
        torch.cuda.synchronize()
        expect = torch.zeros(4, 4)
        for i, j in enumerate(perms[k]):
            expect[i, j] = 1.0
        assert torch.equal(L.H_res.cpu(), expect.expand(24, 4, 4)), k
        # x_out[i] = x[sigma_k(i)] + H_post[i] y: the residual part is a pure stream permutation
        ref = oracle_reference(inp, wl, backward=False)
        assert rel_err(to_np64(L.x_out), ref["x_out"]) <= TOL_BF16_OUT


def test_eps_zero_and_large_width():
    # eps = 0 (pure RMS) on non-zero input; C = 8192 exercises long rows (n*C = 16384 per token)
    wl = si.Workload("eps0", n=2, C=8192, T=100, io="bf16", eps=0.0)
    inp = si.make_inputs(wl, seed=5, device="cuda")
    ref = oracle_reference(inp, wl)
    L = GpuLayer(desc_for(wl), inp)
    L.step()
    torch.cuda.synchronize()
    _check_forward(L, ref, wl)
    _check_backward(L, ref, wl)


def test_saturated_gates_stay_finite():
    # very large |bias| on the gate logits: sigmoid saturates to 0 / 1 (2 for H_post) without NaN
    wl = _small("saturated", C=64, T=16)
    inp = si.make_inputs(wl, seed=6, device="cuda")
    b = inp["b"].clone()
    b[24:28] = torch.tensor([80.0, -80.0, 30.0, -30.0], device="cuda")
    b[28:32] = torch.tensor([-80.0, 80.0, -30.0, 30.0], device="cuda")
    inp["b"] = b
    ref = oracle_reference(inp, wl)
    L = GpuLayer(desc_for(wl), inp)
    L.step()
    torch.cuda.synchronize()
    for t in (L.H_pre, L.H_post, L.g_x.float(), L.g_W, L.g_b):
        assert torch.isfinite(t).all()
    _check_forward(L, ref, wl)
    _check_backward(L, ref, wl, params=False)
    for name in ("g_W", "g_b", "g_alpha"):
        assert rel_err(to_np64(getattr(L, name)), ref[name]) <= TOL_BF16_PARAM, name


@pytest.mark.parametrize("n,C", [(4, 256), (5, 128), (3, 64)])
def test_backward_scales_exactly_with_the_upstream_gradients(n, C):
    """Upstream gradients 2^-24 and 2^12 times as large (exact in bf16): every backward
    output scales by the same power of two, bit for bit, with no underflow or overflow
    on the way (the n = 5 pass 2 carries its per-token vector in fp16 with a scale)."""
    wl = _small(f"scale_n{n}", n=n, C=C, T=130)
    inp = si.make_inputs(wl, seed=4, device="cuda")
    L = GpuLayer(desc_for(wl), inp)
    L.backward_fused()
    torch.cuda.synchronize()
    base = {k: getattr(L, k).float().clone() for k in ("g_x", "g_y", "g_W", "g_b", "g_alpha")}
    for sc in (2.0 ** -24, 2.0 ** 12):
        scaled = dict(inp)
        scaled["g_xout"] = (inp["g_xout"].float() * sc).to(inp["g_xout"].dtype)
        scaled["g_h"] = (inp["g_h"].float() * sc).to(inp["g_h"].dtype)
        Ls = GpuLayer(desc_for(wl), scaled)
        Ls.backward_fused()
        torch.cuda.synchronize()
        for k, v in base.items():
            got = getattr(Ls, k).float() / sc
            assert torch.equal(got, v), (sc, k, float((got - v).abs().max()))


# Many tokens, narrow streams: the launch shapes that depend on the token count (128-token
# blocks of backward pass 1 from 32640 tokens on, one round of resident blocks in pass 2,
# the K split of the projection) with a ragged tail, for stream counts and forms the
# stated workloads do not cover at that length.  Narrow enough for the oracle to redo every token.
LONG_CASES = [
    _small("long_n1", n=1, C=64, T=32768 + 77),
    _small("long_n2_sk", n=2, C=128, T=32640 + 5, res_mode="sk"),
    _small("long_n3", n=3, C=192, T=33000),
    _small("long_n4", n=4, C=64, T=40000 - 1),
    _small("long_n5", n=5, C=64, T=32768 + 130),
    si.Workload(name="long_n6_k24", n=6, C=128, T=32768 + 65, io="bf16", res_mode="subset", n_perm=24),
    # wide backward with few logit tiles: 513 / 625 token blocks over 64 g_W chunks leave the
    # last chunks without tokens (their partial sums must still be written, as zeros)
    _small("long_n5_sk_empty_chunks", n=5, C=128, T=16385, res_mode="sk"),
    si.Workload(name="long_n8_k9_empty_chunks", n=8, C=128, T=20000, io="bf16", res_mode="subset", n_perm=9),
    si.Workload(name="long_n2_k2", n=2, C=256, T=50001, io="bf16", res_mode="subset", n_perm=2),
]


@pytest.mark.parametrize("wl", LONG_CASES, ids=lambda w: w.name)
def test_many_tokens_all_compared(wl):
    print(f"case {wl}", flush=True)
    inp = si.make_inputs(wl, seed=11, device="cuda")
    L = GpuLayer(desc_for(wl, perm=inp.get("perm")), inp)
    L.forward_fused()
    L.backward_fused()
    torch.cuda.synchronize()
    ref = oracle_reference(inp, wl)
    _check_forward(L, ref, wl)
    _check_backward(L, ref, wl)


@pytest.mark.parametrize("wl", [_small("nogy_n4", C=256, T=333), _small("nogy_n5", n=5, C=128, T=150),
                                _small("nogy_f32", n=3, C=40, T=19, io="f32"),
                                si.Workload(name="nogy_n8", n=8, C=64, T=150, io="bf16",
                                            res_mode="subset", n_perm=64),
                                si.Workload(name="nogy_n8_k120", n=8, C=128, T=130, io="bf16",
                                            res_mode="subset", n_perm=120)],
                         ids=lambda w: w.name)
def test_fused_backward_without_g_y(wl):
    """g_y is optional in mhcl_bwd_fused: without it every other output is bit for bit
    the same and the g_y buffer is left alone."""
    import paper_2601_05732_amd as mhcl
    print(f"case {wl}", flush=True)
    inp = si.make_inputs(wl, seed=5, device="cuda")
    L = GpuLayer(desc_for(wl, perm=inp.get("perm")), inp)
    L.backward_fused()
    torch.cuda.synchronize()
    want = {k: getattr(L, k).clone() for k in ("g_x", "g_W", "g_b", "g_alpha")}
    L.g_y.fill_(7.0)
    for k in want:
        getattr(L, k).zero_()
    i = L.inp
    mhcl.mhcl_bwd_fused(L.d, i["x"], i["y"], i["W"], i["b"], i["alpha"], i["g_xout"], i["g_h"],
                        L.g_x, None, L.g_W, L.g_b, L.g_alpha, L.ws)
    torch.cuda.synchronize()
    for k, v in want.items():
        assert torch.equal(getattr(L, k), v), k
    assert bool((L.g_y.float() == 7.0).all())


def test_two_streams_with_their_own_buffers_do_not_interfere():
    """The library keeps no global state: the same calls issued on two streams (default
    priority) with disjoint tensors and workspaces give the bits of sequential runs."""
    wls = [_small("streams_a", C=512, T=3000), _small("streams_b", n=5, C=128, T=2000)]
    layers, want = [], []
    for k, wl in enumerate(wls):
        inp = si.make_inputs(wl, seed=20 + k, device="cuda")
        L = GpuLayer(desc_for(wl), inp)
        L.step()
        torch.cuda.synchronize()
        want.append({nm: getattr(L, nm).clone() for nm in ("x_out", "g_x", "g_y", "g_W", "g_b", "g_alpha")})
        for nm in want[-1]:
            getattr(L, nm).zero_()
        layers.append(L)
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for rep in range(3):
        for L, s in zip(layers, streams):
            with torch.cuda.stream(s):
                L.step()
    torch.cuda.synchronize()
    for L, w in zip(layers, want):
        for nm, v in w.items():
            assert torch.equal(getattr(L, nm), v), nm
