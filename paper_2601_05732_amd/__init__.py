"""mHC-lite hyper-connection hot path for AMD MI355X (gfx950).

The work is done by ``libmhcl.so`` (hand-written HIP, C ABI in
``include/mhcl.h``); :mod:`paper_2601_05732_amd.binding` only marshals torch
tensors into its arguments.  There is no CPU or eager fallback: if the
library is missing, loading it raises.
"""
from .binding import (  # noqa: F401
    BF16, F32, RES_LITE, RES_SK, RES_SUBSET, OP_COEFFS, OP_COEFFS_BWD, OP_FWD_COEFFS_PRE, OP_BWD_FUSED,
    MhclError, Desc, lib, lib_path, exported_symbols, logit_count, workspace_bytes, perm_table,
    mhcl_coeffs, mhcl_pre, mhcl_post, mhcl_fwd_coeffs_pre, mhcl_post_bwd, mhcl_pre_bwd,
    mhcl_coeffs_bwd, mhcl_bwd_fused, mhcl_logits, mhcl_ds_chain, mhcl_fwd_coeffs_pre_static,
    STATIC_SCRATCH_BYTES,
)
from .layer import GpuLayer, desc_for, empty_stream, place_stream  # noqa: F401,E402
from .autograd import HyperConnection, HyperConnectionStack, init_params  # noqa: F401,E402
