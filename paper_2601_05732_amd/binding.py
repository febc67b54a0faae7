"""ctypes binding of libmhcl's C ABI (include/mhcl.h): argument marshalling only.

Every function takes torch tensors that already live on the GPU, checks
dtype / shape / contiguity on the host, and passes raw device pointers and the
current HIP stream to the library.  All arithmetic happens in the library's
kernels.
"""
from __future__ import annotations

import ctypes
import math
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmhcl.so")

BF16, F32 = 0, 1
RES_LITE, RES_SK, RES_SUBSET = 0, 1, 2
OP_COEFFS, OP_COEFFS_BWD, OP_FWD_COEFFS_PRE, OP_BWD_FUSED = 0, 1, 2, 3

_SYMBOLS = [
    "mhcl_status_string", "mhcl_validate", "mhcl_logit_count", "mhcl_workspace_bytes",
    "mhcl_perm_table", "mhcl_coeffs", "mhcl_pre", "mhcl_post", "mhcl_fwd_coeffs_pre",
    "mhcl_post_bwd", "mhcl_pre_bwd", "mhcl_coeffs_bwd", "mhcl_bwd_fused",
    "mhcl_logits", "mhcl_ds_chain", "mhcl_profile_next_call", "mhcl_debug_copy",
    "mhcl_fwd_coeffs_pre_static",
]
STATIC_SCRATCH_BYTES = 16 << 20   # MHCL_STATIC_SCRATCH_BYTES


class MhclError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({_status_string(status)})")


class _CDesc(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int32), ("C", ctypes.c_int32), ("T", ctypes.c_int64),
                ("io_dtype", ctypes.c_int32), ("res_mode", ctypes.c_int32),
                ("sk_iters", ctypes.c_int32), ("eps", ctypes.c_float),
                ("n_perm", ctypes.c_int32), ("perm", ctypes.c_void_p)]


class Desc:
    """Mirror of ``mhcl_desc``."""

    def __init__(self, n, C, T, io_dtype=BF16, res_mode=RES_LITE, sk_iters=20, eps=1e-6, perm=None):
        """perm: for RES_SUBSET, an int8 GPU tensor [K, n] of permutations (kept alive here)."""
        self.n, self.C, self.T = int(n), int(C), int(T)
        self.io_dtype, self.res_mode, self.sk_iters, self.eps = io_dtype, res_mode, sk_iters, eps
        self.perm = perm
        n_perm, pptr = 0, None
        if perm is not None:
            if perm.dtype != torch.int8 or perm.dim() != 2 or perm.shape[1] != self.n \
                    or not perm.is_contiguous():
                raise ValueError("perm must be a contiguous int8 tensor [K, n]")
            if T > 0 and not perm.is_cuda:
                raise ValueError("perm must be a GPU tensor")
            n_perm, pptr = int(perm.shape[0]), perm.data_ptr()
        self.n_perm = n_perm
        self.c = _CDesc(self.n, self.C, self.T, io_dtype, res_mode, sk_iters, eps, n_perm, pptr)

    @property
    def R(self):
        if self.res_mode == RES_SUBSET:
            return self.n_perm
        return math.factorial(self.n) if self.res_mode == RES_LITE else self.n * self.n

    @property
    def M(self):
        return self.R + 2 * self.n

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.io_dtype == BF16 else torch.float32


_lib = None


def lib_path() -> str:
    return _LIB_PATH


def lib():
    """Loads libmhcl.so; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2601_05732_amd.build` "
                "(there is no fallback implementation)")
        L = ctypes.CDLL(_LIB_PATH)
        L.mhcl_status_string.restype = ctypes.c_char_p
        L.mhcl_status_string.argtypes = [ctypes.c_int]
        L.mhcl_workspace_bytes.restype = ctypes.c_size_t
        L.mhcl_workspace_bytes.argtypes = [ctypes.POINTER(_CDesc), ctypes.c_int]
        L.mhcl_logit_count.restype = ctypes.c_int32
        L.mhcl_logit_count.argtypes = [ctypes.POINTER(_CDesc)]
        L.mhcl_validate.argtypes = [ctypes.POINTER(_CDesc)]
        L.mhcl_perm_table.argtypes = [ctypes.c_int32, ctypes.c_void_p]
        P, V, Z = ctypes.POINTER(_CDesc), ctypes.c_void_p, ctypes.c_size_t
        L.mhcl_coeffs.argtypes = [P] + [V] * 8 + [Z, V]
        L.mhcl_pre.argtypes = [P] + [V] * 4
        L.mhcl_post.argtypes = [P] + [V] * 6
        L.mhcl_fwd_coeffs_pre.argtypes = [P] + [V] * 9 + [Z, V]
        L.mhcl_fwd_coeffs_pre_static.argtypes = [P] + [V] * 9
        L.mhcl_post_bwd.argtypes = [P] + [V] * 10
        L.mhcl_pre_bwd.argtypes = [P] + [V] * 6
        L.mhcl_coeffs_bwd.argtypes = [P] + [V] * 12 + [Z, V]
        L.mhcl_bwd_fused.argtypes = [P] + [V] * 13 + [Z, V]
        L.mhcl_logits.argtypes = [P] + [V] * 7 + [Z, V]
        L.mhcl_ds_chain.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int64] + [V] * 7
        _lib = L
    return _lib


def exported_symbols():
    """Names include/mhcl.h declares; each must resolve in the loaded library."""
    L = lib()
    return {name: hasattr(L, name) for name in _SYMBOLS}


def _status_string(status: int) -> str:
    return lib().mhcl_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != 0:
        raise MhclError(status, where)


def logit_count(d: Desc) -> int:
    return lib().mhcl_logit_count(ctypes.byref(d.c))


def workspace_bytes(d: Desc, op: int) -> int:
    return lib().mhcl_workspace_bytes(ctypes.byref(d.c), op)


def perm_table(n: int):
    import numpy as np
    out = np.zeros((math.factorial(n), n), dtype=np.int8)
    _check(lib().mhcl_perm_table(n, out.ctypes.data), "mhcl_perm_table")
    return out


def _ptr(t, dtype, shape, name):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must be a GPU tensor")
    if t.dtype != dtype:
        raise ValueError(f"{name}: dtype {t.dtype}, expected {dtype}")
    if tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: shape {tuple(t.shape)}, expected {tuple(shape)}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr() or None     # an empty tensor has no storage: pass NULL


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _ws(ws):
    if ws is None:
        return None, 0
    return ws.data_ptr(), ws.numel() * ws.element_size()


def new_workspace(d: Desc, op: int, device="cuda"):
    return torch.empty(workspace_bytes(d, op), dtype=torch.uint8, device=device)


def mhcl_coeffs(d, x, W, b, alpha, H_res, H_pre, H_post, ws):
    f, io = torch.float32, d.torch_dtype
    wp, wb = _ws(ws)
    _check(lib().mhcl_coeffs(
        ctypes.byref(d.c), _ptr(x, io, (d.T, d.n, d.C), "x"), _ptr(W, f, (d.n * d.C, d.M), "W"),
        _ptr(b, f, (d.M,), "b"), _ptr(alpha, f, (3,), "alpha"),
        _ptr(H_res, f, (d.T, d.n, d.n), "H_res"), _ptr(H_pre, f, (d.T, d.n), "H_pre"),
        _ptr(H_post, f, (d.T, d.n), "H_post"), wp, wb, _stream()), "mhcl_coeffs")


def mhcl_pre(d, x, H_pre, h):
    f, io = torch.float32, d.torch_dtype
    _check(lib().mhcl_pre(ctypes.byref(d.c), _ptr(x, io, (d.T, d.n, d.C), "x"),
                          _ptr(H_pre, f, (d.T, d.n), "H_pre"), _ptr(h, io, (d.T, d.C), "h"),
                          _stream()), "mhcl_pre")


def mhcl_post(d, x, y, H_res, H_post, x_out):
    f, io = torch.float32, d.torch_dtype
    _check(lib().mhcl_post(
        ctypes.byref(d.c), _ptr(x, io, (d.T, d.n, d.C), "x"), _ptr(y, io, (d.T, d.C), "y"),
        _ptr(H_res, f, (d.T, d.n, d.n), "H_res"), _ptr(H_post, f, (d.T, d.n), "H_post"),
        _ptr(x_out, io, (d.T, d.n, d.C), "x_out"), _stream()), "mhcl_post")


def mhcl_fwd_coeffs_pre(d, x, W, b, alpha, H_res, H_pre, H_post, h, ws):
    f, io = torch.float32, d.torch_dtype
    wp, wb = _ws(ws)
    _check(lib().mhcl_fwd_coeffs_pre(
        ctypes.byref(d.c), _ptr(x, io, (d.T, d.n, d.C), "x"), _ptr(W, f, (d.n * d.C, d.M), "W"),
        _ptr(b, f, (d.M,), "b"), _ptr(alpha, f, (3,), "alpha"),
        _ptr(H_res, f, (d.T, d.n, d.n), "H_res"), _ptr(H_pre, f, (d.T, d.n), "H_pre"),
        _ptr(H_post, f, (d.T, d.n), "H_post"), _ptr(h, io, (d.T, d.C), "h"), wp, wb, _stream()),
        "mhcl_fwd_coeffs_pre")


def mhcl_fwd_coeffs_pre_static(d, x, W, b, alpha, H_res, H_pre, H_post, h):
    f, io = torch.float32, d.torch_dtype
    _check(lib().mhcl_fwd_coeffs_pre_static(
        ctypes.byref(d.c), _ptr(x, io, (d.T, d.n, d.C), "x"), _ptr(W, f, (d.n * d.C, d.M), "W"),
        _ptr(b, f, (d.M,), "b"), _ptr(alpha, f, (3,), "alpha"),
        _ptr(H_res, f, (d.T, d.n, d.n), "H_res"), _ptr(H_pre, f, (d.T, d.n), "H_pre"),
        _ptr(H_post, f, (d.T, d.n), "H_post"), _ptr(h, io, (d.T, d.C), "h"), _stream()),
        "mhcl_fwd_coeffs_pre_static")


def mhcl_post_bwd(d, x, y, H_res, H_post, g_xout, g_x, g_y, g_H_res, g_H_post):
    f, io = torch.float32, d.torch_dtype
    _check(lib().mhcl_post_bwd(
        ctypes.byref(d.c), _ptr(x, io, (d.T, d.n, d.C), "x"), _ptr(y, io, (d.T, d.C), "y"),
        _ptr(H_res, f, (d.T, d.n, d.n), "H_res"), _ptr(H_post, f, (d.T, d.n), "H_post"),
        _ptr(g_xout, io, (d.T, d.n, d.C), "g_xout"), _ptr(g_x, io, (d.T, d.n, d.C), "g_x"),
        _ptr(g_y, io, (d.T, d.C), "g_y"), _ptr(g_H_res, f, (d.T, d.n, d.n), "g_H_res"),
        _ptr(g_H_post, f, (d.T, d.n), "g_H_post"), _stream()), "mhcl_post_bwd")


def mhcl_pre_bwd(d, x, H_pre, g_h, g_x, g_H_pre):
    f, io = torch.float32, d.torch_dtype
    _check(lib().mhcl_pre_bwd(
        ctypes.byref(d.c), _ptr(x, io, (d.T, d.n, d.C), "x"), _ptr(H_pre, f, (d.T, d.n), "H_pre"),
        _ptr(g_h, io, (d.T, d.C), "g_h"), _ptr(g_x, io, (d.T, d.n, d.C), "g_x"),
        _ptr(g_H_pre, f, (d.T, d.n), "g_H_pre"), _stream()), "mhcl_pre_bwd")


def mhcl_coeffs_bwd(d, x, W, b, alpha, g_H_res, g_H_pre, g_H_post, g_x, g_W, g_b, g_alpha, ws):
    f, io = torch.float32, d.torch_dtype
    wp, wb = _ws(ws)
    _check(lib().mhcl_coeffs_bwd(
        ctypes.byref(d.c), _ptr(x, io, (d.T, d.n, d.C), "x"), _ptr(W, f, (d.n * d.C, d.M), "W"),
        _ptr(b, f, (d.M,), "b"), _ptr(alpha, f, (3,), "alpha"),
        _ptr(g_H_res, f, (d.T, d.n, d.n), "g_H_res"), _ptr(g_H_pre, f, (d.T, d.n), "g_H_pre"),
        _ptr(g_H_post, f, (d.T, d.n), "g_H_post"), _ptr(g_x, io, (d.T, d.n, d.C), "g_x"),
        _ptr(g_W, f, (d.n * d.C, d.M), "g_W"), _ptr(g_b, f, (d.M,), "g_b"),
        _ptr(g_alpha, f, (3,), "g_alpha"), wp, wb, _stream()), "mhcl_coeffs_bwd")


def mhcl_bwd_fused(d, x, y, W, b, alpha, g_xout, g_h, g_x, g_y, g_W, g_b, g_alpha, ws):
    f, io = torch.float32, d.torch_dtype
    wp, wb = _ws(ws)
    _check(lib().mhcl_bwd_fused(
        ctypes.byref(d.c), _ptr(x, io, (d.T, d.n, d.C), "x"), _ptr(y, io, (d.T, d.C), "y"),
        _ptr(W, f, (d.n * d.C, d.M), "W"), _ptr(b, f, (d.M,), "b"),
        _ptr(alpha, f, (3,), "alpha"), _ptr(g_xout, io, (d.T, d.n, d.C), "g_xout"),
        _ptr(g_h, io, (d.T, d.C), "g_h"), _ptr(g_x, io, (d.T, d.n, d.C), "g_x"),
        None if g_y is None else _ptr(g_y, io, (d.T, d.C), "g_y"),
        _ptr(g_W, f, (d.n * d.C, d.M), "g_W"),
        _ptr(g_b, f, (d.M,), "g_b"), _ptr(g_alpha, f, (3,), "g_alpha"), wp, wb, _stream()),
        "mhcl_bwd_fused")


def mhcl_logits(d, x, W, b, alpha, z, log_inv_nu, ws):
    f, io = torch.float32, d.torch_dtype
    wp, wb = _ws(ws)
    _check(lib().mhcl_logits(
        ctypes.byref(d.c), _ptr(x, io, (d.T, d.n, d.C), "x"), _ptr(W, f, (d.n * d.C, d.M), "W"),
        _ptr(b, f, (d.M,), "b"), _ptr(alpha, f, (3,), "alpha"), _ptr(z, f, (d.T, d.M), "z"),
        _ptr(log_inv_nu, f, (d.T,), "log_inv_nu"), wp, wb, _stream()), "mhcl_logits")


def mhcl_ds_chain(n, L, T, H, colsum, l1, prod, prod_colsum, prod_l1):
    f = torch.float32
    _check(lib().mhcl_ds_chain(
        n, L, T, _ptr(H, f, (L, T, n, n), "H"), _ptr(colsum, f, (L, T, n), "colsum"),
        _ptr(l1, f, (L, T), "l1"), _ptr(prod, f, (T, n, n), "prod"),
        _ptr(prod_colsum, f, (L, T, n), "prod_colsum"), _ptr(prod_l1, f, (L, T), "prod_l1"),
        _stream()), "mhcl_ds_chain")
