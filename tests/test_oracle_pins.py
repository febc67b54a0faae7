"""Pins for the fp64 CPU oracle: everything the paper and the mathematics fix.

None of these tests touches the GPU library.  Each check is chosen so that a
plausible slip in the oracle (dropped term, wrong sign or index, transposed
operand, wrong SK order) fails at least one of them.
"""
import itertools
import math
import os

import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si


# ----------------------------------------------------------------------------
# Permutation table and P_stack  (Theorem 3.1; Sec. 3.2 "constant 0/1 matrix")
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 6])
def test_perm_table_brute_force(n):
    sig = oracle.perm_table(n)
    assert sig.shape == (math.factorial(n), n)
    rows = [tuple(r) for r in sig.tolist()]
    # every row a bijection of {0..n-1}; all distinct; complete
    assert all(sorted(r) == list(range(n)) for r in rows)
    assert len(set(rows)) == math.factorial(n)
    # lexicographic, identity first: the library enumeration is the reference
    assert rows == list(itertools.permutations(range(n)))
    assert rows[0] == tuple(range(n))


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5])
def test_pstack_is_all_permutation_matrices(n):
    P = oracle.pstack(n)
    nf = math.factorial(n)
    assert P.shape == (nf, n, n)
    assert set(np.unique(P).tolist()) <= {0.0, 1.0}
    assert np.all(P.sum(axis=1) == 1) and np.all(P.sum(axis=2) == 1)
    # each cell (i, j) is hit by exactly (n-1)! permutations
    assert np.all(P.sum(axis=0) == math.factorial(n - 1))
    # placement convention: P_k[i][sigma_k(i)] = 1
    for k, s in enumerate(itertools.permutations(range(n))):
        for i in range(n):
            assert P[k, i, s[i]] == 1.0
    # distinct
    assert len({P[k].tobytes() for k in range(nf)}) == nf


# ----------------------------------------------------------------------------
# H_res lives in the Birkhoff polytope  (Sec. 2 definition of B_n; Sec. 3.2)
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("n", [1, 2, 3, 4, 5])
def test_h_res_doubly_stochastic_and_gate_ranges(n):
    d = si.small_case(n, C=8, T=17, seed=n)
    H_res, H_pre, H_post, a = oracle.coeffs_lite(d["x"], d["W"], d["b"], d["alpha"],
                                                 return_a=True)
    assert np.all(H_res >= 0)
    assert np.abs(H_res.sum(axis=1) - 1).max() < 1e-12
    assert np.abs(H_res.sum(axis=2) - 1).max() < 1e-12
    assert np.all(a >= 0) and np.abs(a.sum(axis=1) - 1).max() < 1e-12
    assert np.all((H_pre > 0) & (H_pre < 1))
    assert np.all((H_post > 0) & (H_post < 2))
    # spectral norm <= 1 and closure under products (Sec. 1, Sec. 2)
    prod = np.eye(n)
    for t in range(H_res.shape[0]):
        assert np.linalg.norm(H_res[t], 2) <= 1 + 1e-12
        prod = prod @ H_res[t]
    assert np.abs(prod.sum(axis=0) - 1).max() < 1e-12
    assert np.abs(prod.sum(axis=1) - 1).max() < 1e-12
    assert np.all(oracle.ds_l1_error(H_res) < 1e-11)


@pytest.mark.parametrize("n", [2, 3, 4])
def test_one_hot_weights_reproduce_each_permutation(n):
    nf = math.factorial(n)
    C, T = 4, 2
    rng = np.random.default_rng(0)
    x = rng.standard_normal((T, n, C))
    W = np.zeros((n * C, nf + 2 * n))
    for k, s in enumerate(itertools.permutations(range(n))):
        b = np.zeros(nf + 2 * n)
        b[:nf] = -1e4
        b[k] = 0.0
        H_res, _, _ = oracle.coeffs_lite(x, W, b, np.ones(3))
        expect = np.zeros((n, n))
        for i in range(n):
            expect[i, s[i]] = 1.0
        assert np.array_equal(H_res[0], expect) and np.array_equal(H_res[1], expect)


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5])
def test_uniform_logits_give_uniform_matrix(n):
    nf = math.factorial(n)
    x = np.random.default_rng(1).standard_normal((3, n, 4))
    H_res, H_pre, H_post = oracle.coeffs_lite(x, np.zeros((n * 4, nf + 2 * n)),
                                              np.zeros(nf + 2 * n), np.ones(3))
    assert np.allclose(H_res, 1.0 / n, rtol=0, atol=1e-15)
    assert np.allclose(H_pre, 0.5, atol=1e-15) and np.allclose(H_post, 1.0, atol=1e-15)


def test_n2_closed_form_logistic():
    # n = 2: permutations (id, swap); H_res = [[s, 1-s], [1-s, s]], s = sigmoid(z0 - z1)
    d = si.small_case(2, C=8, T=9, seed=3)
    x, W, b, al = d["x"], d["W"], d["b"], d["alpha"]
    H_res, _, _ = oracle.coeffs_lite(x, W, b, al, eps=0.0)
    xh = x.reshape(9, -1)
    xn = xh / np.sqrt((xh ** 2).mean(axis=1, keepdims=True))
    z = al[0] * (xn @ W[:, :2]) + b[:2]
    s = 1.0 / (1.0 + np.exp(-(z[:, 0] - z[:, 1])))
    assert np.allclose(H_res[:, 0, 0], s, atol=1e-14) and np.allclose(H_res[:, 1, 1], s, atol=1e-14)
    assert np.allclose(H_res[:, 0, 1], 1 - s, atol=1e-14)
    assert np.allclose(H_res[:, 1, 0], 1 - s, atol=1e-14)


def test_paper_initialisation_closed_form():
    # Sec. 4 "Initialization": W = 0, b_res = 0 at the identity and -8 elsewhere
    # => a_id = 1 / (1 + 23 e^-8); each off-diagonal cell is hit by 6 of the 24
    # permutations, none of them the identity; each diagonal cell by the
    # identity and 5 others.  b_pre, b_post = -1 except one entry at +1.
    n, C = 4, 16
    W, b, alpha = si.paper_init_params(n, C, "lite", one_index=2)
    x = np.random.default_rng(5).standard_normal((6, n, C))
    H_res, H_pre, H_post, a = oracle.coeffs_lite(x, W, b, alpha, return_a=True)
    e8 = math.exp(-8.0)
    den = 1.0 + 23.0 * e8
    assert np.allclose(a[:, 0], 1.0 / den, rtol=1e-13)
    assert np.allclose(a[:, 1:], e8 / den, rtol=1e-13)
    diag = (1.0 + 5.0 * e8) / den
    off = 6.0 * e8 / den
    for t in range(6):
        assert np.allclose(np.diag(H_res[t]), diag, rtol=1e-13)
        assert np.allclose(H_res[t][~np.eye(n, dtype=bool)], off, rtol=1e-13)
    # the digits quoted for this closed form
    assert abs(1.0 / den - 0.9923434349) < 1e-9 and abs(diag - 0.9940079055) < 1e-9
    assert abs(off - 0.0019973648) < 1e-9
    sig = lambda t: 1.0 / (1.0 + math.exp(-t))
    expect = np.full(n, sig(-1.0)); expect[2] = sig(1.0)
    assert np.allclose(H_pre, expect, rtol=1e-13) and np.allclose(H_post, 2 * expect, rtol=1e-13)
    # the block then acts almost as an ordinary residual connection
    y = np.random.default_rng(6).standard_normal((6, C))
    x_out = oracle.post(x, y, H_res, H_post)
    resid = x + (2 * expect)[None, :, None] * y[:, None, :]
    assert np.abs(x_out - resid).max() < 0.05


def test_scale_invariance_with_eps_zero():
    d = si.small_case(4, C=8, T=5, seed=7)
    A = oracle.coeffs_lite(d["x"], d["W"], d["b"], d["alpha"], eps=0.0)
    B = oracle.coeffs_lite(37.5 * d["x"], d["W"], d["b"], d["alpha"], eps=0.0)
    for p, q in zip(A, B):
        assert np.allclose(p, q, rtol=1e-12, atol=1e-15)


def test_zero_input_gives_bias_only_logits():
    n, C = 3, 8
    d = si.small_case(n, C, 2, seed=8)
    x0 = np.zeros((2, n, C))
    H_res, H_pre, H_post, a = oracle.coeffs_lite(x0, d["W"], d["b"], d["alpha"], eps=1e-6,
                                                 return_a=True)
    nf = 6
    e = np.exp(d["b"][:nf] - d["b"][:nf].max())
    assert np.allclose(a[0], e / e.sum(), rtol=1e-13)
    assert np.allclose(H_pre[0], 1 / (1 + np.exp(-d["b"][nf:nf + n])), rtol=1e-13)


# ----------------------------------------------------------------------------
# Forward against an independent library implementation (torch CPU fp64)
# ----------------------------------------------------------------------------
def _torch_forward(x, W, b, alpha, y, eps, res_mode="lite", iters=20):
    """The forward written with library routines (rms_norm, softmax, sigmoid,
    matmul); autograd of this graph is the independent backward."""
    T, n, C = x.shape
    R = math.factorial(n) if res_mode == "lite" else n * n
    xh = x.reshape(T, n * C)
    xn = torch.nn.functional.rms_norm(xh, (n * C,), eps=eps)
    u = xn @ W
    z_res = alpha[0] * u[:, :R] + b[:R]
    z_pre = alpha[1] * u[:, R:R + n] + b[R:R + n]
    z_post = alpha[2] * u[:, R + n:] + b[R + n:]
    if res_mode == "lite":
        P = torch.zeros(R, n * n, dtype=x.dtype)
        for k, s in enumerate(itertools.permutations(range(n))):
            for i in range(n):
                P[k, i * n + s[i]] = 1.0
        H_res = (torch.softmax(z_res, dim=-1) @ P).reshape(T, n, n)
    else:
        X = torch.exp(z_res).reshape(T, n, n)
        for _ in range(iters):
            X = X / X.sum(dim=1, keepdim=True)   # columns sum to 1
            X = X / X.sum(dim=2, keepdim=True)   # rows sum to 1
        H_res = X
    H_pre = torch.sigmoid(z_pre)
    H_post = 2 * torch.sigmoid(z_post)
    h = torch.einsum("tj,tjc->tc", H_pre, x)
    x_out = torch.einsum("tij,tjc->tic", H_res, x) + H_post[:, :, None] * y[:, None, :]
    return H_res, H_pre, H_post, h, x_out


@pytest.mark.parametrize("res_mode", ["lite", "sk"])
@pytest.mark.parametrize("n", [1, 2, 3, 4, 5])
def test_forward_matches_library_implementation(n, res_mode):
    d = si.small_case(n, C=16, T=11, seed=10 + n, res_mode=res_mode)
    tt = {k: torch.tensor(v, dtype=torch.float64) for k, v in d.items()}
    ref = _torch_forward(tt["x"], tt["W"], tt["b"], tt["alpha"], tt["y"], 1e-6, res_mode)
    got = oracle.forward(d["x"], d["W"], d["b"], d["alpha"], d["y"], eps=1e-6, res_mode=res_mode)
    for name, r in zip(["H_res", "H_pre", "H_post", "h", "x_out"], ref):
        assert np.allclose(got[name], r.numpy(), rtol=1e-11, atol=1e-13), name


# ----------------------------------------------------------------------------
# Stream mixing  (Eq. 1)
# ----------------------------------------------------------------------------
def test_identity_coefficients_reduce_to_plain_residual():
    n, C, T = 4, 8, 5
    rng = np.random.default_rng(11)
    x = rng.standard_normal((T, n, C)); y = rng.standard_normal((T, C))
    H_res = np.tile(np.eye(n), (T, 1, 1))
    H_pre = np.zeros((T, n)); H_pre[:, 2] = 1.0
    H_post = np.ones((T, n))
    assert np.array_equal(oracle.pre(x, H_pre), x[:, 2, :])
    assert np.array_equal(oracle.post(x, y, H_res, H_post), x + y[:, None, :])


def test_post_is_not_transposed():
    # a single off-diagonal entry: x_out[i] must pick up x[j] for H_res[i][j]
    n, C = 3, 4
    x = np.arange(n * C, dtype=float).reshape(1, n, C) + 1
    H = np.zeros((1, n, n)); H[0, 0, 2] = 1.0
    out = oracle.post(x, np.zeros((1, C)), H, np.zeros((1, n)))
    assert np.array_equal(out[0, 0], x[0, 2]) and np.all(out[0, 1:] == 0)


def test_stream_sum_conservation():
    # column sums of H_res are 1  =>  sum_i x_out[i] = sum_j x[j] + (sum_i H_post[i]) y
    d = si.small_case(4, C=8, T=7, seed=12)
    f = oracle.forward(d["x"], d["W"], d["b"], d["alpha"], d["y"])
    lhs = f["x_out"].sum(axis=1)
    rhs = d["x"].sum(axis=1) + f["H_post"].sum(axis=1, keepdims=True) * d["y"]
    assert np.allclose(lhs, rhs, rtol=1e-12, atol=1e-12)


# ----------------------------------------------------------------------------
# Sinkhorn-Knopp  (Sec. 1 worked example; Sec. 2 below Eq. 2)
# ----------------------------------------------------------------------------
def _read_golden(path):
    kv = {}
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, v = line.split("=", 1)
        kv[k.strip()] = v.strip()
    return kv


def test_sk_worked_example_from_the_paper(golden_dir):
    g = _read_golden(os.path.join(golden_dir, "sk_example_sec1.txt"))
    al = float(g["alpha"])
    X0 = np.array([[0.5, al, al], [0.5, al, al], [al, 1.0, 1.0]])
    out = oracle.sk(X0, iters=int(g["iters"]))
    printed = np.array([float(v) for v in g["out"].split()]).reshape(3, 3)
    # to the printed digits: two significant digits for 0.91 / 0.045, one for 0.5 / 0.
    half_ulp = np.array([[0.005, 0.0005, 0.0005]] * 2 + [[0.05, 0.05, 0.05]])
    assert np.all(np.abs(out - printed) <= half_ulp), out
    cs = out.sum(axis=0)
    want = [float(v) for v in g["colsums_from_printed_matrix"].split()]
    assert abs(cs[0] - want[0]) < 0.01 and abs(cs[1] - want[1]) < 0.005 and abs(cs[2] - want[2]) < 0.005
    # the last half step is a row normalisation
    assert np.abs(out.sum(axis=1) - 1).max() < 1e-14
    # one iteration more or fewer, or rows before columns, does not print as 0.91
    assert abs(oracle.sk(X0, iters=19)[0, 0] - 0.91) > 0.005
    assert abs(oracle.sk(X0, iters=21)[0, 0] - 0.91) > 0.005
    assert np.abs(oracle.sk(X0.T, iters=20).T.sum(axis=0) - 1).max() < 1e-14  # rows-first ends on columns


def test_sk_fixed_point_and_row_sums():
    d = si.small_case(4, C=8, T=4, seed=13)
    H_res, _, _ = oracle.coeffs_lite(d["x"], d["W"], d["b"], d["alpha"])
    for t in range(4):   # an exactly doubly stochastic positive matrix is left alone
        assert np.allclose(oracle.sk(H_res[t], iters=20), H_res[t], rtol=1e-12)
    X = np.random.default_rng(14).random((5, 5)) + 0.1
    for it in (1, 2, 7):
        assert np.abs(oracle.sk(X, it).sum(axis=1) - 1).max() < 1e-14
    # converges to doubly stochastic on a well-conditioned input
    assert oracle.ds_l1_error(oracle.sk(X, 200)[None])[0] < 1e-12
    # invariance to a global scale of the input
    assert np.allclose(oracle.sk(X, 5), oracle.sk(1e3 * X, 5), rtol=1e-12)


def test_sk_paper_initialisation_is_near_identity():
    n, C = 4, 8
    W, b, alpha = si.paper_init_params(n, C, "sk")
    x = np.random.default_rng(15).standard_normal((3, n, C))
    H_res, _, _ = oracle.coeffs_sk(x, W, b, alpha)
    assert np.abs(H_res - np.eye(n)).max() < 2e-3
    assert np.all(oracle.ds_l1_error(H_res) < 1e-10)


def test_l1_error_and_relative_range_definitions():
    X = np.array([[[0.5, 0.25], [0.0, 1.0]]])
    # rows: 0.75, 1.0 ; columns: 0.5, 1.25  -> 0.25 + 0 + 0.5 + 0.25
    assert abs(oracle.ds_l1_error(X)[0] - 1.0) < 1e-15
    assert oracle.relative_range(X)[0] == 0.25   # min positive / max


# ----------------------------------------------------------------------------
# Backward: central finite differences and library autograd
# ----------------------------------------------------------------------------
def _loss(d, res_mode):
    f = oracle.forward(d["x"], d["W"], d["b"], d["alpha"], d["y"], eps=1e-6, res_mode=res_mode)
    return float((d["g_xout"] * f["x_out"]).sum() + (d["g_h"] * f["h"]).sum())


@pytest.mark.parametrize("res_mode", ["lite", "sk"])
@pytest.mark.parametrize("n", [1, 2, 3, 4])
def test_backward_central_finite_differences(n, res_mode):
    d = si.small_case(n, C=8, T=3, seed=20 + n, res_mode=res_mode)
    g = oracle.backward(d["x"], d["W"], d["b"], d["alpha"], d["y"], d["g_xout"], d["g_h"],
                        eps=1e-6, res_mode=res_mode)
    rng = np.random.default_rng(99)
    step = 1e-6
    for name, gname in [("x", "g_x"), ("y", "g_y"), ("W", "g_W"), ("b", "g_b"),
                        ("alpha", "g_alpha")]:
        base = d[name]
        idx = [tuple(rng.integers(0, s) for s in base.shape) for _ in range(12)]
        if base.size <= 12:
            idx = list(np.ndindex(*base.shape))
        scale = max(1.0, float(np.abs(g[gname]).max()))
        for ix in idx:
            dp = dict(d); dm = dict(d)
            p = base.copy(); p[ix] += step; dp[name] = p
            m = base.copy(); m[ix] -= step; dm[name] = m
            fd = (_loss(dp, res_mode) - _loss(dm, res_mode)) / (2 * step)
            assert abs(fd - g[gname][ix]) <= 5e-7 * scale, (name, ix, fd, g[gname][ix])


@pytest.mark.parametrize("res_mode", ["lite", "sk"])
@pytest.mark.parametrize("n", [1, 2, 3, 4, 5])
def test_backward_matches_library_autograd(n, res_mode):
    d = si.small_case(n, C=8, T=6, seed=30 + n, res_mode=res_mode)
    tt = {k: torch.tensor(v, dtype=torch.float64) for k, v in d.items()}
    for k in ("x", "W", "b", "alpha", "y"):
        tt[k].requires_grad_(True)
    H_res, H_pre, H_post, h, x_out = _torch_forward(tt["x"], tt["W"], tt["b"], tt["alpha"],
                                                    tt["y"], 1e-6, res_mode)
    L = (tt["g_xout"] * x_out).sum() + (tt["g_h"] * h).sum()
    L.backward()
    g = oracle.backward(d["x"], d["W"], d["b"], d["alpha"], d["y"], d["g_xout"], d["g_h"],
                        eps=1e-6, res_mode=res_mode)
    for name, gname in [("x", "g_x"), ("y", "g_y"), ("W", "g_W"), ("b", "g_b"),
                        ("alpha", "g_alpha")]:
        ref = tt[name].grad.numpy()
        scale = max(1e-30, np.abs(ref).max())
        assert np.abs(g[gname] - ref).max() <= 1e-10 * scale, gname


def test_separable_backwards_individually_against_autograd():
    # each separable backward with its coefficient inputs treated as independent
    n, C, T = 3, 8, 4
    rng = np.random.default_rng(40)
    x = torch.tensor(rng.standard_normal((T, n, C)), requires_grad=True)
    y = torch.tensor(rng.standard_normal((T, C)), requires_grad=True)
    H_res = torch.tensor(rng.random((T, n, n)), requires_grad=True)
    H_post = torch.tensor(rng.random((T, n)), requires_grad=True)
    H_pre = torch.tensor(rng.random((T, n)), requires_grad=True)
    g_xout = rng.standard_normal((T, n, C)); g_h = rng.standard_normal((T, C))
    x_out = torch.einsum("tij,tjc->tic", H_res, x) + H_post[:, :, None] * y[:, None, :]
    (torch.tensor(g_xout) * x_out).sum().backward()
    g_x, g_y, g_H_res, g_H_post = oracle.post_bwd(x.detach().numpy(), y.detach().numpy(),
                                                  H_res.detach().numpy(), H_post.detach().numpy(),
                                                  g_xout)
    assert np.allclose(g_x, x.grad.numpy(), rtol=1e-12, atol=1e-13)
    assert np.allclose(g_y, y.grad.numpy(), rtol=1e-12, atol=1e-13)
    assert np.allclose(g_H_res, H_res.grad.numpy(), rtol=1e-12, atol=1e-13)
    assert np.allclose(g_H_post, H_post.grad.numpy(), rtol=1e-12, atol=1e-13)
    x.grad = None
    h = torch.einsum("tj,tjc->tc", H_pre, x)
    (torch.tensor(g_h) * h).sum().backward()
    acc = np.ones((T, n, C))          # pre_bwd accumulates into g_x
    g_H_pre = oracle.pre_bwd(x.detach().numpy(), H_pre.detach().numpy(), g_h, acc)
    assert np.allclose(acc - 1.0, x.grad.numpy(), rtol=1e-12, atol=1e-13)
    assert np.allclose(g_H_pre, H_pre.grad.numpy(), rtol=1e-12, atol=1e-13)


def test_backward_identities():
    d = si.small_case(4, C=8, T=5, seed=41)
    args = (d["x"], d["W"], d["b"], d["alpha"], d["y"])
    g1 = oracle.backward(*args, d["g_xout"], d["g_h"])
    # softmax: the gradient on the n! residual logits sums to zero over k
    assert abs(g1["g_b"][:24].sum()) < 1e-12 * np.abs(g1["g_b"][:24]).max() * 24
    # linear in the upstream gradients
    g2 = oracle.backward(*args, 2.0 * d["g_xout"], -3.0 * d["g_h"])
    ga = oracle.backward(*args, d["g_xout"], 0 * d["g_h"])
    gb = oracle.backward(*args, 0 * d["g_xout"], d["g_h"])
    for k in ("g_x", "g_y", "g_W", "g_b", "g_alpha"):
        assert np.allclose(g2[k], 2.0 * ga[k] - 3.0 * gb[k], rtol=1e-11, atol=1e-12), k
