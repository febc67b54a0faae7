"""fp64 CPU oracle for the mHC-lite hyper-connection path: TEST INFRASTRUCTURE.

A thin ctypes wrapper over ``mhcl_oracle.c`` (plain C, fp64, written from the
paper's definitions; see that file's header for what each function follows
and how it is pinned).  Only tests, the smoke check and the benchmark's CPU
baseline may import this package; the GPU library never does, and this
package never imports the GPU library.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mhcl_oracle.c")
_LIB = os.path.join(_HERE, "libmhcl_oracle.so")

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-Wall", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_D = ctypes.POINTER(ctypes.c_double)
_I = ctypes.POINTER(ctypes.c_int)


def _load():
    global _lib
    if _lib is None:
        # MHCLO_LIB: a library built elsewhere from (a changed copy of) the source; the tests
        # use it to show that the pins fail when a mistake is planted in the oracle
        other = os.environ.get("MHCLO_LIB")
        if other:
            _lib = ctypes.CDLL(other)
        else:
            build()
            _lib = ctypes.CDLL(_LIB)
        _lib.mhclo_factorial.restype = ctypes.c_int
    return _lib


def _p(a):
    return a.ctypes.data_as(_D)


def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def perm_table(n: int) -> np.ndarray:
    """[n!, n] int32, sigma[k][i]; lexicographic, k=0 identity."""
    out = np.zeros((math.factorial(n), n), dtype=np.int32)
    _load().mhclo_perm_table(ctypes.c_int(n), out.ctypes.data_as(_I))
    return out


def pstack(n: int) -> np.ndarray:
    """[n!, n, n] float64 stack of all permutation matrices."""
    out = np.zeros((math.factorial(n), n, n), dtype=np.float64)
    _load().mhclo_pstack(ctypes.c_int(n), _p(out))
    return out


def _dims(x):
    T, n, C = x.shape
    return ctypes.c_int(n), ctypes.c_int(C), ctypes.c_long(T)


def coeffs_lite(x, W, b, alpha, eps=1e-6, return_a=False):
    x, W, b, alpha = _f64(x), _f64(W), _f64(b), _f64(alpha)
    T, n, C = x.shape
    R = math.factorial(n)
    assert W.shape == (n * C, R + 2 * n) and b.shape == (R + 2 * n,) and alpha.shape == (3,)
    H_res = np.empty((T, n, n)); H_pre = np.empty((T, n)); H_post = np.empty((T, n))
    a = np.empty((T, R))
    _load().mhclo_coeffs_lite(*_dims(x), _p(x), _p(W), _p(b), _p(alpha), ctypes.c_double(eps),
                              _p(H_res), _p(H_pre), _p(H_post), _p(a))
    return (H_res, H_pre, H_post, a) if return_a else (H_res, H_pre, H_post)


def _sigma32(sigma, n):
    sigma = np.ascontiguousarray(np.asarray(sigma, dtype=np.int32))
    assert sigma.ndim == 2 and sigma.shape[1] == n
    assert all(sorted(row) == list(range(n)) for row in sigma.tolist()), "rows must be permutations"
    return sigma


def coeffs_subset(x, W, b, alpha, sigma, eps=1e-6, return_a=False):
    """Permutation form restricted to the K permutations sigma [K, n]."""
    x, W, b, alpha = _f64(x), _f64(W), _f64(b), _f64(alpha)
    T, n, C = x.shape
    sigma = _sigma32(sigma, n)
    K = sigma.shape[0]
    assert W.shape == (n * C, K + 2 * n) and b.shape == (K + 2 * n,) and alpha.shape == (3,)
    H_res = np.empty((T, n, n)); H_pre = np.empty((T, n)); H_post = np.empty((T, n))
    a = np.empty((T, K))
    _load().mhclo_coeffs_subset(*_dims(x), ctypes.c_int(K), sigma.ctypes.data_as(_I), _p(x), _p(W),
                                _p(b), _p(alpha), ctypes.c_double(eps), _p(H_res), _p(H_pre),
                                _p(H_post), _p(a))
    return (H_res, H_pre, H_post, a) if return_a else (H_res, H_pre, H_post)


def sk(X0, iters=20):
    X0 = _f64(X0)
    n = X0.shape[0]
    assert X0.shape == (n, n)
    X = np.empty((n, n))
    _load().mhclo_sk(ctypes.c_int(n), _p(X0), ctypes.c_int(iters), _p(X))
    return X


def coeffs_sk(x, W, b, alpha, eps=1e-6, iters=20):
    x, W, b, alpha = _f64(x), _f64(W), _f64(b), _f64(alpha)
    T, n, C = x.shape
    M = n * n + 2 * n
    assert W.shape == (n * C, M) and b.shape == (M,) and alpha.shape == (3,)
    H_res = np.empty((T, n, n)); H_pre = np.empty((T, n)); H_post = np.empty((T, n))
    _load().mhclo_coeffs_sk(*_dims(x), _p(x), _p(W), _p(b), _p(alpha), ctypes.c_double(eps),
                            ctypes.c_int(iters), _p(H_res), _p(H_pre), _p(H_post))
    return H_res, H_pre, H_post


def pre(x, H_pre):
    x, H_pre = _f64(x), _f64(H_pre)
    T, n, C = x.shape
    assert H_pre.shape == (T, n)
    h = np.empty((T, C))
    _load().mhclo_pre(*_dims(x), _p(x), _p(H_pre), _p(h))
    return h


def post(x, y, H_res, H_post):
    x, y, H_res, H_post = _f64(x), _f64(y), _f64(H_res), _f64(H_post)
    T, n, C = x.shape
    assert y.shape == (T, C) and H_res.shape == (T, n, n) and H_post.shape == (T, n)
    out = np.empty((T, n, C))
    _load().mhclo_post(*_dims(x), _p(x), _p(y), _p(H_res), _p(H_post), _p(out))
    return out


def post_bwd(x, y, H_res, H_post, g_xout):
    """-> g_x (H_res path only), g_y, g_H_res, g_H_post"""
    x, y, H_res, H_post, g_xout = map(_f64, (x, y, H_res, H_post, g_xout))
    T, n, C = x.shape
    assert g_xout.shape == (T, n, C)
    g_x = np.empty((T, n, C)); g_y = np.empty((T, C))
    g_H_res = np.empty((T, n, n)); g_H_post = np.empty((T, n))
    _load().mhclo_post_bwd(*_dims(x), _p(x), _p(y), _p(H_res), _p(H_post), _p(g_xout),
                           _p(g_x), _p(g_y), _p(g_H_res), _p(g_H_post))
    return g_x, g_y, g_H_res, g_H_post


def pre_bwd(x, H_pre, g_h, g_x):
    """g_x is accumulated into in place (must be a contiguous float64 array).
    -> g_H_pre"""
    x, H_pre, g_h = map(_f64, (x, H_pre, g_h))
    T, n, C = x.shape
    assert g_x.dtype == np.float64 and g_x.flags.c_contiguous and g_x.shape == (T, n, C)
    g_H_pre = np.empty((T, n))
    _load().mhclo_pre_bwd(*_dims(x), _p(x), _p(H_pre), _p(g_h), _p(g_x), _p(g_H_pre))
    return g_H_pre


def coeffs_bwd(x, W, b, alpha, g_H_res, g_H_pre, g_H_post, g_x, eps=1e-6, res_mode="lite",
               iters=20, sigma=None):
    """g_x is accumulated into in place.  -> g_W, g_b, g_alpha"""
    x, W, b, alpha, g_H_res, g_H_pre, g_H_post = map(
        _f64, (x, W, b, alpha, g_H_res, g_H_pre, g_H_post))
    T, n, C = x.shape
    assert g_x.dtype == np.float64 and g_x.flags.c_contiguous and g_x.shape == (T, n, C)
    g_W = np.empty_like(W); g_b = np.empty_like(b); g_alpha = np.empty(3)
    lib = _load()
    if res_mode == "lite":
        assert W.shape[1] == math.factorial(n) + 2 * n
        lib.mhclo_coeffs_lite_bwd(*_dims(x), _p(x), _p(W), _p(b), _p(alpha), ctypes.c_double(eps),
                                  _p(g_H_res), _p(g_H_pre), _p(g_H_post),
                                  _p(g_x), _p(g_W), _p(g_b), _p(g_alpha))
    elif res_mode == "subset":
        sigma = _sigma32(sigma, n)
        assert W.shape[1] == sigma.shape[0] + 2 * n
        lib.mhclo_coeffs_subset_bwd(*_dims(x), ctypes.c_int(sigma.shape[0]),
                                    sigma.ctypes.data_as(_I), _p(x), _p(W), _p(b), _p(alpha),
                                    ctypes.c_double(eps), _p(g_H_res), _p(g_H_pre), _p(g_H_post),
                                    _p(g_x), _p(g_W), _p(g_b), _p(g_alpha))
    else:
        assert W.shape[1] == n * n + 2 * n
        lib.mhclo_coeffs_sk_bwd(*_dims(x), _p(x), _p(W), _p(b), _p(alpha), ctypes.c_double(eps),
                                ctypes.c_int(iters), _p(g_H_res), _p(g_H_pre), _p(g_H_post),
                                _p(g_x), _p(g_W), _p(g_b), _p(g_alpha))
    return g_W, g_b, g_alpha


def ds_l1_error(X):
    X = _f64(X)
    T, n, _ = X.shape
    err = np.empty(T)
    _load().mhclo_ds_l1_error(ctypes.c_int(n), ctypes.c_long(T), _p(X), _p(err))
    return err


def relative_range(X):
    X = _f64(X)
    T, n, _ = X.shape
    nu = np.empty(T)
    _load().mhclo_relative_range(ctypes.c_int(n), ctypes.c_long(T), _p(X), _p(nu))
    return nu


def logits(x, W, b, alpha, eps=1e-6, res_mode="lite", n_perm=None):
    """z [T, M]: all logits, columns [res | pre | post]."""
    x, W, b, alpha = _f64(x), _f64(W), _f64(b), _f64(alpha)
    T, n, C = x.shape
    R = {"lite": math.factorial(n), "sk": n * n, "subset": n_perm}[res_mode]
    M = R + 2 * n
    assert W.shape == (n * C, M) and b.shape == (M,) and alpha.shape == (3,)
    z = np.empty((T, M))
    _load().mhclo_logits(*_dims(x), ctypes.c_int(R), _p(x), _p(W), _p(b), _p(alpha),
                         ctypes.c_double(eps), _p(z))
    return z


def ds_chain(H):
    """H [L, T, n, n] -> dict of colsum [L,T,n], l1 [L,T], prod [T,n,n],
    prod_colsum [L,T,n], prod_l1 [L,T]."""
    H = _f64(H)
    L, T, n, _ = H.shape
    out = dict(colsum=np.empty((L, T, n)), l1=np.empty((L, T)), prod=np.empty((T, n, n)),
               prod_colsum=np.empty((L, T, n)), prod_l1=np.empty((L, T)))
    _load().mhclo_ds_chain(ctypes.c_int(n), ctypes.c_int(L), ctypes.c_long(T), _p(H),
                           _p(out["colsum"]), _p(out["l1"]), _p(out["prod"]),
                           _p(out["prod_colsum"]), _p(out["prod_l1"]))
    return out


def forward(x, W, b, alpha, y, eps=1e-6, res_mode="lite", iters=20, sigma=None):
    """Whole forward of one layer with y = f(h) supplied: coefficients, h, x_out."""
    if res_mode == "lite":
        H_res, H_pre, H_post = coeffs_lite(x, W, b, alpha, eps)
    elif res_mode == "subset":
        H_res, H_pre, H_post = coeffs_subset(x, W, b, alpha, sigma, eps)
    else:
        H_res, H_pre, H_post = coeffs_sk(x, W, b, alpha, eps, iters)
    h = pre(x, H_pre)
    x_out = post(x, y, H_res, H_post)
    return {"H_res": H_res, "H_pre": H_pre, "H_post": H_post, "h": h, "x_out": x_out}


def backward(x, W, b, alpha, y, g_xout, g_h, eps=1e-6, res_mode="lite", iters=20, sigma=None):
    """Whole backward of one layer for L = <g_xout, x_out> + <g_h, h> with y an
    independent input: the three separable backwards chained."""
    fw = forward(x, W, b, alpha, y, eps, res_mode, iters, sigma)
    g_x, g_y, g_H_res, g_H_post = post_bwd(x, y, fw["H_res"], fw["H_post"], g_xout)
    g_H_pre = pre_bwd(x, fw["H_pre"], g_h, g_x)
    g_W, g_b, g_alpha = coeffs_bwd(x, W, b, alpha, g_H_res, g_H_pre, g_H_post, g_x, eps,
                                   res_mode, iters, sigma)
    return {"g_x": g_x, "g_y": g_y, "g_W": g_W, "g_b": g_b, "g_alpha": g_alpha,
            "g_H_res": g_H_res, "g_H_pre": g_H_pre, "g_H_post": g_H_post, **fw}
