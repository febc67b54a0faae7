"""Host-side checks of the C ABI: the library loads, exports every symbol the
header declares, validates arguments before touching a GPU, and its
permutation table equals the library enumeration.  No GPU needed."""
import ctypes
import itertools
import os
import re

import numpy as np
import pytest

import paper_2601_05732_amd as mhcl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "mhcl.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mhcl_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    declared = _declared_symbols()
    assert len(declared) >= 13
    L = mhcl.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert all(mhcl.exported_symbols().values())


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5])
def test_perm_table_matches_library_enumeration(n):
    got = mhcl.perm_table(n)
    assert got.tolist() == [list(p) for p in itertools.permutations(range(n))]


def test_logit_count_and_workspace():
    d = mhcl.Desc(4, 4096, 32768, mhcl.BF16, mhcl.RES_LITE)
    assert mhcl.logit_count(d) == 32
    assert mhcl.logit_count(mhcl.Desc(5, 2560, 16, mhcl.BF16)) == 130
    assert mhcl.logit_count(mhcl.Desc(4, 4096, 16, mhcl.BF16, mhcl.RES_SK)) == 24
    for op in (mhcl.OP_COEFFS, mhcl.OP_COEFFS_BWD, mhcl.OP_FWD_COEFFS_PRE, mhcl.OP_BWD_FUSED):
        assert mhcl.workspace_bytes(d, op) >= 256
        assert mhcl.workspace_bytes(mhcl.Desc(4, 64, 0, mhcl.F32), op) >= 256
    assert mhcl.workspace_bytes(d, 99) == 0


@pytest.mark.parametrize("kw", [
    dict(n=0), dict(n=6), dict(C=0), dict(C=12), dict(T=-1), dict(io_dtype=7), dict(res_mode=3),
    dict(res_mode=mhcl.RES_SK, sk_iters=0), dict(res_mode=mhcl.RES_SK, sk_iters=1000),
    dict(eps=-1.0), dict(eps=float("nan")),
])
def test_invalid_descriptors_are_rejected(kw):
    base = dict(n=4, C=64, T=16, io_dtype=mhcl.BF16, res_mode=mhcl.RES_LITE, sk_iters=20, eps=1e-6)
    base.update(kw)
    d = mhcl.Desc(**base)
    assert mhcl.lib().mhcl_validate(ctypes.byref(d.c)) == 1
    assert mhcl.logit_count(d) == -1
    assert mhcl.workspace_bytes(d, mhcl.OP_COEFFS) == 0


def test_null_and_misaligned_pointers_fail_before_any_launch():
    L = mhcl.lib()
    d = mhcl.Desc(4, 64, 16, mhcl.F32)
    ok = 4096  # an aligned, never dereferenced address: validation fails first
    assert L.mhcl_pre(ctypes.byref(d.c), None, ok, ok, None) == 1
    assert L.mhcl_pre(ctypes.byref(d.c), ok, ok + 4, ok, None) == 1
    assert L.mhcl_post(ctypes.byref(d.c), ok, ok, ok, ok, ok, None) == 1     # x_out aliases x
    assert L.mhcl_coeffs(ctypes.byref(d.c), ok, ok, ok, ok, ok, ok, ok, None, 0, None) == 3
    assert L.mhcl_coeffs(ctypes.byref(d.c), ok, ok, ok, ok, ok, ok, ok, ok, 16, None) == 3
    assert L.mhcl_bwd_fused(ctypes.byref(d.c), *([ok] * 12), None, 0, None) == 3
    # g_y (9th tensor) is optional: NULL passes the pointer checks, a misaligned one does not
    args = [ok] * 12
    args[8] = None
    assert L.mhcl_bwd_fused(ctypes.byref(d.c), *args, None, 0, None) == 3
    args[8] = ok + 4
    assert L.mhcl_bwd_fused(ctypes.byref(d.c), *args, None, 0, None) == 1
    args[8], args[7] = ok, None                                              # g_x is not optional
    assert L.mhcl_bwd_fused(ctypes.byref(d.c), *args, None, 0, None) == 1
    assert L.mhcl_coeffs(None, ok, ok, ok, ok, ok, ok, ok, ok, 1 << 20, None) == 1
    assert mhcl.lib().mhcl_status_string(3).decode().startswith("workspace")
    # diagnostics
    assert L.mhcl_logits(ctypes.byref(d.c), ok, ok, ok, ok, None, None, ok, 1 << 20, None) == 1
    assert L.mhcl_logits(ctypes.byref(d.c), ok, ok, ok, ok, ok, None, None, 0, None) == 3
    assert L.mhcl_ds_chain(4, 2, 16, None, ok, ok, ok, ok, ok, None) == 1
    assert L.mhcl_ds_chain(4, 2, 16, ok, None, None, None, None, None, None) == 1
    assert L.mhcl_ds_chain(9, 2, 16, ok, ok, ok, ok, ok, ok, None) == 1
    assert L.mhcl_ds_chain(4, 0, 16, ok, ok, ok, ok, ok, ok, None) == 1
    assert L.mhcl_ds_chain(4, 2, 16, ok, ok + 4, ok, ok, ok, ok, None) == 1
    assert L.mhcl_ds_chain(4, 2, 0, None, None, None, None, None, None, None) == 0


def test_binding_refuses_cpu_tensors():
    import torch
    d = mhcl.Desc(2, 8, 4, mhcl.F32)
    x = torch.zeros(4, 2, 8)
    with pytest.raises(ValueError):
        mhcl.mhcl_pre(d, x, torch.zeros(4, 2), torch.zeros(4, 8))


def test_subset_descriptor_fields_are_validated_on_the_host():
    class FakePerm:                      # any non-null address: validation never dereferences it
        pass
    d = mhcl.Desc(6, 64, 16, mhcl.BF16, mhcl.RES_SUBSET)
    assert mhcl.lib().mhcl_validate(ctypes.byref(d.c)) == 1          # no table
    d.c.n_perm, d.c.perm = 12, 4096
    assert mhcl.lib().mhcl_validate(ctypes.byref(d.c)) == 0
    assert mhcl.lib().mhcl_logit_count(ctypes.byref(d.c)) == 12 + 12
    assert mhcl.lib().mhcl_workspace_bytes(ctypes.byref(d.c), mhcl.OP_BWD_FUSED) > 0
    d.c.n_perm = 129
    assert mhcl.lib().mhcl_validate(ctypes.byref(d.c)) == 1
    d.c.n_perm, d.c.n = 12, 9
    assert mhcl.lib().mhcl_validate(ctypes.byref(d.c)) == 1
    full = mhcl.Desc(6, 64, 16)                                      # n = 6 only in the subset form
    assert mhcl.lib().mhcl_validate(ctypes.byref(full.c)) == 1


def test_workspace_of_the_fused_forward_follows_the_header():
    """mhcl_fwd_coeffs_pre: where the single-read kernel applies (bf16, at most 32 logits,
    C a multiple of 256 from 1024 to 8192, at least 512 * floor(65536 / C) tokens) the workspace holds one slice of
    the projection per 256 columns; everywhere else it is the workspace of mhcl_coeffs."""
    def sizes(n, C, T, io=mhcl.BF16, res_mode=mhcl.RES_LITE):
        d = mhcl.Desc(n, C, T, io, res_mode=res_mode)
        return d, mhcl.workspace_bytes(d, mhcl.OP_FWD_COEFFS_PRE), mhcl.workspace_bytes(d, mhcl.OP_COEFFS)
    for n, C, T in ((4, 4096, 32768), (4, 4096, 8192), (3, 1024, 65536), (2, 2048, 16384),
                    (4, 5120, 6144), (4, 8192, 4096), (3, 1280, 26112)):
        d, fused, plain = sizes(n, C, T)
        slices = (C // 256) * T * (d.M + 1) * 4
        assert fused > plain and slices <= fused <= slices + (8 << 20), (n, C, T, fused, slices)
    for n, C, T, io, mode in ((4, 4096, 8191, mhcl.BF16, mhcl.RES_LITE),     # too few tokens
                              (4, 4096 + 64, 32768, mhcl.BF16, mhcl.RES_LITE),   # C not a multiple of 256
                              (4, 768, 65536, mhcl.BF16, mhcl.RES_LITE),         # fewer than four parts
                              (2, 16384, 8192, mhcl.BF16, mhcl.RES_LITE),        # more than 32 parts
                              (4, 5120, 6143, mhcl.BF16, mhcl.RES_LITE),         # too few tokens
                              (5, 1024, 65536, mhcl.BF16, mhcl.RES_LITE),    # 130 logits
                              (4, 4096, 32768, mhcl.F32, mhcl.RES_LITE)):    # f32 streams
        _, fused, plain = sizes(n, C, T, io, mode)
        assert fused == plain, (n, C, T)
