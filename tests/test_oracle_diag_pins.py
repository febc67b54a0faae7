"""Pins for the oracle's diagnostics: the logits (Sec. 3.2), and the column
sums / l1 errors of single residual matrices and of their product over the
layers (Sec. 3.1, Sec. 4.3).  No GPU involved.
"""
import itertools
import os

import numpy as np
import pytest

import oracle
import synth_inputs as si


@pytest.mark.parametrize("res_mode", ["lite", "sk"])
@pytest.mark.parametrize("n", [1, 3, 4])
def test_logits_plain_formula_and_consistency(n, res_mode):
    d = si.small_case(n, C=8, T=5, seed=31, res_mode=res_mode)
    x, W, b, alpha = d["x"], d["W"], d["b"], d["alpha"] * np.array([0.7, 1.3, -0.9])
    z = oracle.logits(x, W, b, alpha, eps=1e-6, res_mode=res_mode)
    T, _, C = x.shape
    R = z.shape[1] - 2 * n
    xh = x.reshape(T, n * C)
    xn = xh / np.sqrt((xh * xh).mean(axis=1, keepdims=True) + 1e-6)
    scale = np.concatenate([np.full(R, alpha[0]), np.full(n, alpha[1]), np.full(n, alpha[2])])
    assert np.allclose(z, (xn @ W) * scale + b, rtol=1e-12, atol=1e-13)
    # the gates are the logistic function of exactly these logits
    coeffs = oracle.coeffs_lite if res_mode == "lite" else oracle.coeffs_sk
    H = coeffs(x, W, b, alpha)
    assert np.allclose(H[1], 1 / (1 + np.exp(-z[:, R:R + n])), rtol=1e-13)
    assert np.allclose(H[2], 2 / (1 + np.exp(-z[:, R + n:])), rtol=1e-13)
    if res_mode == "lite":
        a = oracle.coeffs_lite(x, W, b, alpha, return_a=True)[3]
        e = np.exp(z[:, :R] - z[:, :R].max(axis=1, keepdims=True))
        assert np.allclose(a, e / e.sum(axis=1, keepdims=True), rtol=1e-13)
    else:   # SK is started from exp of the reshaped residual logits
        for t in range(T):
            assert np.allclose(H[0][t], oracle.sk(np.exp(z[t, :R]).reshape(n, n), 20), rtol=1e-12)


def test_logits_of_zero_input_are_the_bias():
    d = si.small_case(4, C=8, T=2, seed=32)
    z = oracle.logits(np.zeros_like(d["x"]), d["W"], d["b"], d["alpha"])
    assert np.array_equal(z, np.broadcast_to(d["b"], z.shape))


def test_chain_of_permutations_composes_in_application_order():
    n, L = 4, 5
    sig = oracle.perm_table(n)
    P = oracle.pstack(n)
    rng = np.random.default_rng(33)
    ks = rng.integers(0, len(sig), size=(L, 6))
    out = oracle.ds_chain(P[ks])                      # H[l][t] = P_{ks[l][t]}
    for t in range(ks.shape[1]):
        # Q_L = H_L ... H_1 : row i of the product has its 1 in column s_1(s_2(...s_L(i)))
        want = np.zeros((n, n))
        for i in range(n):
            j = i
            for l in reversed(range(L)):
                j = sig[ks[l, t]][j]
            want[i, j] = 1.0
        assert np.array_equal(out["prod"][t], want)
    assert np.all(out["colsum"] == 1) and np.all(out["prod_colsum"] == 1)
    assert np.all(out["l1"] == 0) and np.all(out["prod_l1"] == 0)
    # the order matters for this pick (a reversed product would differ somewhere)
    rev = oracle.ds_chain(P[ks[::-1]])["prod"]
    assert not np.array_equal(rev, out["prod"])


def test_chain_of_scaled_doubly_stochastic_matrices_closed_form():
    n, L, T = 4, 6, 3
    d = si.small_case(n, C=8, T=L * T, seed=34)
    D = oracle.coeffs_lite(d["x"], d["W"], d["b"], d["alpha"])[0].reshape(L, T, n, n)
    s = np.array([1.1, 0.8, 1.0, 1.25, 0.9, 1.3])
    out = oracle.ds_chain(D * s[:, None, None, None])
    cum = np.cumprod(s)
    assert np.allclose(out["colsum"], s[:, None, None], rtol=1e-13)
    assert np.allclose(out["l1"], (2 * n * np.abs(s - 1))[:, None], rtol=1e-12, atol=1e-13)
    assert np.allclose(out["prod_colsum"], cum[:, None, None], rtol=1e-12)
    assert np.allclose(out["prod_l1"], (2 * n * np.abs(cum - 1))[:, None], rtol=1e-11, atol=1e-13)
    # row sums of the product too (l1 counts both): Q_L 1 = prod(s) 1
    assert np.allclose(out["prod"].sum(axis=2), cum[-1], rtol=1e-12)


def test_chain_matches_library_matmul_on_general_matrices():
    rng = np.random.default_rng(35)
    L, T, n = 4, 3, 3
    H = rng.random((L, T, n, n))
    out = oracle.ds_chain(H)
    for t in range(T):
        Q = np.eye(n)
        for l in range(L):
            Q = H[l, t] @ Q
            assert np.allclose(out["prod_colsum"][l, t], Q.sum(axis=0), rtol=1e-13)
            assert np.isclose(out["prod_l1"][l, t],
                              np.abs(Q.sum(axis=1) - 1).sum() + np.abs(Q.sum(axis=0) - 1).sum(), rtol=1e-13)
        assert np.allclose(out["prod"][t], Q, rtol=1e-13)
        assert np.allclose(out["colsum"][:, t], H[:, t].sum(axis=1), rtol=1e-14)


def test_paper_example_column_sums_and_their_growth(golden_dir):
    """Sec. 1's 3x3 example after 20 SK iterations: column sums as printed, and
    since every row sums to 1 the product over layers keeps row sums 1 while
    its column sums are those of the matrix power (library routine)."""
    al = 1e-13
    X0 = np.array([[0.5, al, al], [0.5, al, al], [al, 1.0, 1.0]])
    H = oracle.sk(X0, 20)
    out = oracle.ds_chain(np.broadcast_to(H, (24, 1, 3, 3)))
    assert np.allclose(out["colsum"][0, 0], [1.82, 0.59, 0.59], atol=0.005)
    assert abs(out["l1"][0, 0] - (0.82 + 0.41 + 0.41)) < 0.02
    for l in (1, 6, 24):
        Q = np.linalg.matrix_power(H, l)
        assert np.allclose(out["prod_colsum"][l - 1, 0], Q.sum(axis=0), rtol=1e-12)
    assert np.allclose(out["prod"][0].sum(axis=1), 1, atol=1e-13)


def test_relative_range_equals_logit_spread():
    """Eq. (3) on X = exp(Z): log(1/nu) = max Z - min Z."""
    Z = np.random.default_rng(36).normal(0, 9, size=(7, 4, 4))
    nu = oracle.relative_range(np.exp(Z))
    assert np.allclose(np.log(1 / nu), Z.max(axis=(1, 2)) - Z.min(axis=(1, 2)), rtol=1e-12)
