"""Pins for the oracle's permutation-subset form (Sec. 5, the paragraph on
larger n: only some of the n! permutation matrices are kept, the result is
still doubly stochastic).  No GPU involved.
"""
import itertools
import math

import numpy as np
import pytest

import oracle
import synth_inputs as si


def _case(n, K, C=4, T=3, seed=0):
    rng = np.random.default_rng(seed)
    M = K + 2 * n
    return dict(x=rng.standard_normal((T, n, C)), W=0.3 * rng.standard_normal((n * C, M)),
                b=0.3 * rng.standard_normal(M), alpha=0.5 + rng.random(3),
                y=rng.standard_normal((T, C)), g_xout=rng.standard_normal((T, n, C)),
                g_h=rng.standard_normal((T, C)))


def _random_subset(n, K, seed):
    rng = np.random.default_rng(seed)
    rows = set()
    while len(rows) < K:
        rows.add(tuple(rng.permutation(n).tolist()))
    return np.array(sorted(rows), dtype=np.int32)


@pytest.mark.parametrize("n", [2, 3, 4])
def test_all_permutations_in_lexicographic_order_is_the_full_form(n):
    d = si.small_case(n, C=8, T=4, seed=41)
    sig = oracle.perm_table(n)
    full = oracle.coeffs_lite(d["x"], d["W"], d["b"], d["alpha"], return_a=True)
    sub = oracle.coeffs_subset(d["x"], d["W"], d["b"], d["alpha"], sig, return_a=True)
    for u, v in zip(full, sub):
        assert np.array_equal(u, v)
    bf = oracle.backward(d["x"], d["W"], d["b"], d["alpha"], d["y"], d["g_xout"], d["g_h"])
    bs = oracle.backward(d["x"], d["W"], d["b"], d["alpha"], d["y"], d["g_xout"], d["g_h"],
                         res_mode="subset", sigma=sig)
    for k in ("g_x", "g_W", "g_b", "g_alpha", "g_y"):
        assert np.array_equal(bf[k], bs[k]), k


@pytest.mark.parametrize("n,K", [(5, 7), (6, 12), (8, 20)])
def test_doubly_stochastic_with_support_on_the_chosen_permutations(n, K):
    d = _case(n, K, seed=42)
    sig = _random_subset(n, K, 43)
    H_res, H_pre, H_post, a = oracle.coeffs_subset(d["x"], d["W"], d["b"], d["alpha"], sig, return_a=True)
    assert np.abs(H_res.sum(axis=1) - 1).max() < 1e-13 and np.abs(H_res.sum(axis=2) - 1).max() < 1e-13
    assert np.abs(a.sum(axis=1) - 1).max() < 1e-13 and (a > 0).all()
    support = np.zeros((n, n), dtype=bool)
    for row in sig:
        support[np.arange(n), row] = True
    assert (H_res[:, ~support] == 0).all() and (H_res[:, support] > 0).all()
    assert ((H_pre > 0) & (H_pre < 1)).all() and ((H_post > 0) & (H_post < 2)).all()


def test_cyclic_shifts_give_a_circulant_matrix_of_the_softmax_weights():
    """K = n cyclic shifts have disjoint supports: H_res[i][(i + k) % n] = a_k."""
    n = 6
    sig = np.array([[(i + k) % n for i in range(n)] for k in range(n)], dtype=np.int32)
    d = _case(n, n, seed=44)
    H_res = oracle.coeffs_subset(d["x"], d["W"], d["b"], d["alpha"], sig)[0]
    z = oracle.logits(d["x"], d["W"], d["b"], d["alpha"], res_mode="subset", n_perm=n)[:, :n]
    a = np.exp(z - z.max(axis=1, keepdims=True))
    a /= a.sum(axis=1, keepdims=True)
    want = np.zeros_like(H_res)
    for k in range(n):
        for i in range(n):
            want[:, i, (i + k) % n] = a[:, k]
    assert np.allclose(H_res, want, rtol=1e-13, atol=0)
    # row i -> column sigma(i), not the transpose: shift by +1 puts row 0's weight in column 1
    assert np.allclose(H_res[:, 0, 1], a[:, 1], rtol=1e-13)


def test_single_permutation_is_that_matrix_and_has_no_gradient_on_its_logit():
    n, K = 7, 1
    sig = _random_subset(n, 1, 45)
    d = _case(n, K, seed=46)
    H_res = oracle.coeffs_subset(d["x"], d["W"], d["b"], d["alpha"], sig)[0]
    P = np.zeros((n, n)); P[np.arange(n), sig[0]] = 1
    assert np.array_equal(H_res, np.broadcast_to(P, H_res.shape))
    r = oracle.backward(d["x"], d["W"], d["b"], d["alpha"], d["y"], d["g_xout"], d["g_h"],
                        res_mode="subset", sigma=sig)
    assert np.abs(r["g_W"][:, 0]).max() < 1e-14 and abs(r["g_b"][0]) < 1e-14
    assert abs(r["g_alpha"][0]) < 1e-14 and np.abs(r["g_W"][:, 1:]).max() > 1e-3


def test_relabelling_the_subset_permutes_the_logit_columns():
    n, K = 5, 6
    sig = _random_subset(n, K, 47)
    d = _case(n, K, seed=48)
    order = np.random.default_rng(49).permutation(K)
    cols = np.concatenate([order, K + np.arange(2 * n)])
    H1 = oracle.coeffs_subset(d["x"], d["W"], d["b"], d["alpha"], sig)
    H2 = oracle.coeffs_subset(d["x"], d["W"][:, cols], d["b"][cols], d["alpha"], sig[order])
    for u, v in zip(H1, H2):
        assert np.allclose(u, v, rtol=1e-13, atol=1e-15)


def test_one_hot_bias_selects_one_permutation():
    n, K = 6, 9
    sig = _random_subset(n, K, 50)
    d = _case(n, K, seed=51)
    W = np.zeros_like(d["W"])
    for k in (0, 4, 8):
        b = d["b"].copy(); b[:K] = -1e4; b[k] = 0.0
        H_res = oracle.coeffs_subset(d["x"], W, b, d["alpha"], sig)[0]
        P = np.zeros((n, n)); P[np.arange(n), sig[k]] = 1
        assert np.array_equal(H_res[0], P)


def _loss(d, sig):
    f = oracle.forward(d["x"], d["W"], d["b"], d["alpha"], d["y"], res_mode="subset", sigma=sig)
    return float((d["g_xout"] * f["x_out"]).sum() + (d["g_h"] * f["h"]).sum())


@pytest.mark.parametrize("n,K", [(3, 4), (6, 5)])
def test_backward_central_finite_differences(n, K):
    sig = _random_subset(n, K, 52)
    d = _case(n, K, C=4, T=2, seed=53)
    r = oracle.backward(d["x"], d["W"], d["b"], d["alpha"], d["y"], d["g_xout"], d["g_h"],
                        res_mode="subset", sigma=sig)
    rng = np.random.default_rng(54)
    for name, grad in (("x", r["g_x"]), ("W", r["g_W"]), ("b", r["g_b"]), ("alpha", r["g_alpha"]),
                       ("y", r["g_y"])):
        flat = d[name].reshape(-1)
        for idx in rng.choice(flat.size, size=min(12, flat.size), replace=False):
            old = flat[idx]
            eps = 1e-6
            flat[idx] = old + eps; lp = _loss(d, sig)
            flat[idx] = old - eps; lm = _loss(d, sig)
            flat[idx] = old
            num = (lp - lm) / (2 * eps)
            assert abs(num - grad.reshape(-1)[idx]) <= 2e-6 * max(1.0, abs(num)), (name, idx)
