"""GPU tests of the autograd front end: gradients of one layer and of a stack of
layers around an elementwise layer function, against the fp64 oracle chained
by hand (the chain rule through f is written out here, in numpy).

The ends of the stack (copy the input into n streams, sum the streams at the
output) are this package's choice, not the paper's: parity unpinned for them,
the test only checks the chain rule through them.
"""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from paper_2601_05732_amd.autograd import HyperConnection, HyperConnectionStack, init_params
from paper_2601_05732_amd import binding as mhcl
from gpu_harness import rel_err, to_np64

pytestmark = pytest.mark.gpu


def _f(h):               # the stand-in layer function, torch
    return 0.5 * torch.tanh(h)


def _f_np(h):
    return 0.5 * np.tanh(h)


def _df_np(h):
    return 0.5 * (1.0 - np.tanh(h) ** 2)


def _set_random_params(layer, seed, res_mode):
    wl = si.Workload("p", n=layer.n, C=layer.C, T=1, io="f32", res_mode=res_mode, backward=False)
    inp = si.make_inputs(wl, seed=seed, device="cuda")
    with torch.no_grad():
        layer.W.copy_(inp["W"] * 5)          # std 0.1: logits of order 1, gradients through every path
        layer.b.copy_(inp["b"])
        layer.alpha.copy_(torch.tensor([0.7, 1.2, 0.9], device="cuda"))


@pytest.mark.parametrize("res_mode,io,n,C,T", [
    ("lite", "f32", 4, 64, 50), ("sk", "f32", 3, 40, 21), ("lite", "bf16", 4, 256, 130),
    ("lite", "bf16", 5, 128, 70), ("sk", "bf16", 4, 64, 33)])
def test_single_layer_gradients(res_mode, io, n, C, T):
    print(f"case {res_mode} {io} n={n} C={C} T={T}", flush=True)
    dt = torch.float32 if io == "f32" else torch.bfloat16
    g = torch.Generator(device="cuda").manual_seed(5)
    x = torch.randn(T, n, C, device="cuda", generator=g).to(dt).requires_grad_(True)
    G = torch.randn(T, n, C, device="cuda", generator=g).to(dt)
    layer = HyperConnection(n, C, res_mode)
    _set_random_params(layer, 6, res_mode)
    seen = {}

    def f(h):        # the layer function is not the library's: its own bits go to the oracle
        y = _f(h)
        seen["h"], seen["y"] = h.detach(), y.detach()
        h.register_hook(lambda g: seen.__setitem__("g_h", g.detach().clone()))
        y.register_hook(lambda g: seen.__setitem__("g_y", g.detach().clone()))
        return y

    x_out = layer(x, f)
    (x_out.float() * G.float()).sum().backward()
    torch.cuda.synchronize()

    xs, W, b, al = to_np64(x), to_np64(layer.W), to_np64(layer.b), to_np64(layer.alpha)
    if res_mode == "lite":
        H_res, H_pre, H_post = oracle.coeffs_lite(xs, W, b, al)
    else:
        H_res, H_pre, H_post = oracle.coeffs_sk(xs, W, b, al)
    y = to_np64(seen["y"])
    ref_out = oracle.post(xs, y, H_res, H_post)
    ref = oracle.backward(xs, W, b, al, y, to_np64(G), to_np64(seen["g_h"]), res_mode=res_mode)
    t_stream, t_par = (1e-5, 1e-5) if io == "f32" else (2e-2, 2e-4)
    assert rel_err(to_np64(seen["h"]), oracle.pre(xs, H_pre)) <= t_stream
    assert rel_err(to_np64(x_out), ref_out) <= t_stream
    assert rel_err(to_np64(seen["g_y"]), ref["g_y"]) <= t_stream
    assert rel_err(to_np64(x.grad), ref["g_x"]) <= t_stream
    assert rel_err(to_np64(layer.W.grad), ref["g_W"]) <= t_par
    assert rel_err(to_np64(layer.b.grad), ref["g_b"]) <= t_par
    assert rel_err(to_np64(layer.alpha.grad), ref["g_alpha"]) <= t_par


def test_single_layer_gradients_permutation_subset():
    """The module passes the permutation-subset form through (Sec. 5, larger n): n = 6 with
    12 of the 720 permutations, the identity first."""
    n, C, T, K = 6, 128, 90, 12
    perm = torch.from_numpy(si.subset_permutations(n, K, seed=3)).cuda()
    g = torch.Generator(device="cuda").manual_seed(8)
    x = torch.randn(T, n, C, device="cuda", generator=g).to(torch.bfloat16).requires_grad_(True)
    G = torch.randn(T, n, C, device="cuda", generator=g).to(torch.bfloat16)
    layer = HyperConnection(n, C, "subset", perm=perm)
    assert tuple(layer.W.shape) == (n * C, K + 2 * n) and float(layer.b.detach()[0]) == 0.0
    wl = si.Workload("p", n=n, C=C, T=1, io="f32", res_mode="subset", n_perm=K, backward=False)
    inp = si.make_inputs(wl, seed=9, device="cuda")
    with torch.no_grad():
        layer.W.copy_(inp["W"] * 5)
        layer.b.copy_(inp["b"])
        layer.alpha.copy_(torch.tensor([0.7, 1.2, 0.9], device="cuda"))
    seen = {}

    def f(h):
        y = _f(h)
        seen["y"] = y.detach()
        h.register_hook(lambda g: seen.__setitem__("g_h", g.detach().clone()))
        return y

    x_out = layer(x, f)
    (x_out.float() * G.float()).sum().backward()
    torch.cuda.synchronize()
    sigma = perm.cpu().numpy().astype(np.int32)
    ref = oracle.backward(to_np64(x), to_np64(layer.W), to_np64(layer.b), to_np64(layer.alpha),
                          to_np64(seen["y"]), to_np64(G), to_np64(seen["g_h"]), res_mode="subset", sigma=sigma)
    assert rel_err(to_np64(x_out), ref["x_out"]) <= 2e-2
    assert rel_err(to_np64(x.grad), ref["g_x"]) <= 2e-2
    for got, name in ((layer.W.grad, "g_W"), (layer.b.grad, "g_b"), (layer.alpha.grad, "g_alpha")):
        assert rel_err(to_np64(got), ref[name]) <= 2e-4, name


def test_layer_at_initialisation_is_a_plain_residual_connection():
    """Sec. 4, "Initialization": each block starts close to x_out[s] = x[s] + [s = s0] f(x[s0])
    up to the softmax / logistic leakage of the initial biases."""
    n, C, T = 4, 64, 40
    x = torch.randn(T, n, C, device="cuda")
    layer = HyperConnection(n, C, "lite", one_index=2)
    out = layer(x, _f)
    W, b, al = init_params(n, C, mhcl.RES_LITE, 2)
    H_res, H_pre, H_post = oracle.coeffs_lite(to_np64(x), to_np64(W), to_np64(b), to_np64(al))
    ref = oracle.post(to_np64(x), _f_np(oracle.pre(to_np64(x), H_pre)), H_res, H_post)
    assert rel_err(to_np64(out.detach()), ref) <= 1e-5
    assert np.abs(H_res - np.eye(n)).max() < 0.01 and H_pre[0].argmax() == 2 and H_post[0].argmax() == 2


def test_stack_gradients_match_hand_chained_oracle():
    n, C, T, L = 4, 64, 30, 3
    g = torch.Generator(device="cuda").manual_seed(9)
    x0 = torch.randn(T, C, device="cuda", generator=g).requires_grad_(True)
    G = torch.randn(T, C, device="cuda", generator=g)
    stack = HyperConnectionStack(n, C, [_f] * L, "lite")
    for l, layer in enumerate(stack.layers):
        _set_random_params(layer, 20 + l, "lite")
    out = stack(x0)
    (out * G).sum().backward()
    torch.cuda.synchronize()

    P = [(to_np64(m.W), to_np64(m.b), to_np64(m.alpha)) for m in stack.layers]
    xs = [np.repeat(to_np64(x0)[:, None, :], n, axis=1)]
    hs, ys = [], []
    for l in range(L):
        fw_c = oracle.coeffs_lite(xs[l], *P[l])
        h = oracle.pre(xs[l], fw_c[1])
        y = _f_np(h)
        hs.append(h); ys.append(y)
        xs.append(oracle.post(xs[l], y, fw_c[0], fw_c[2]))
    assert rel_err(to_np64(out), xs[L].sum(axis=1)) <= 1e-5
    g_x = np.repeat(to_np64(G)[:, None, :], n, axis=1)          # sum over streams
    grads = [None] * L
    for l in reversed(range(L)):
        fw_c = oracle.coeffs_lite(xs[l], *P[l])
        g_y = oracle.post_bwd(xs[l], ys[l], fw_c[0], fw_c[2], g_x)[1]
        r = oracle.backward(xs[l], *P[l], ys[l], g_x, g_y * _df_np(hs[l]))
        grads[l] = r
        g_x = r["g_x"]
    assert rel_err(to_np64(x0.grad), g_x.sum(axis=1)) <= 2e-5     # copy into n streams
    for l, m in enumerate(stack.layers):
        assert rel_err(to_np64(m.W.grad), grads[l]["g_W"]) <= 2e-5, l
        assert rel_err(to_np64(m.b.grad), grads[l]["g_b"]) <= 2e-5, l
        assert rel_err(to_np64(m.alpha.grad), grads[l]["g_alpha"]) <= 2e-5, l


def test_layer_function_with_parameters_and_unused_branch():
    """f with its own weights gets gradients through g_y; a layer function that
    ignores h still lets x, W, b, alpha receive theirs."""
    n, C, T = 4, 64, 25
    lin = torch.nn.Linear(C, C, device="cuda")
    x = torch.randn(T, n, C, device="cuda", requires_grad=True)
    layer = HyperConnection(n, C)
    _set_random_params(layer, 3, "lite")
    layer(x, lin).square().sum().backward()
    assert lin.weight.grad is not None and float(lin.weight.grad.abs().sum()) > 0
    const = torch.randn(T, C, device="cuda")
    x2 = x.detach().clone().requires_grad_(True)
    layer.zero_grad()
    layer(x2, lambda h: const).square().sum().backward()
    torch.cuda.synchronize()
    assert x2.grad is not None and layer.W.grad is not None
    H_res, H_pre, H_post = oracle.coeffs_lite(to_np64(x2), to_np64(layer.W), to_np64(layer.b), to_np64(layer.alpha))
    out = oracle.post(to_np64(x2), to_np64(const), H_res, H_post)
    r = oracle.backward(to_np64(x2), to_np64(layer.W), to_np64(layer.b), to_np64(layer.alpha),
                        to_np64(const), 2 * out, np.zeros((T, C)))
    assert rel_err(to_np64(x2.grad), r["g_x"]) <= 1e-5
    assert rel_err(to_np64(layer.W.grad), r["g_W"]) <= 1e-5
