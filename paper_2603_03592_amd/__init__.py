"""MI355X (gfx950) stage verifier: Python binding over libstageverify.so.

The binding only marshals arguments (device pointers of torch tensors, the current HIP
stream) into the C ABI declared in include/stageverify.h; every step of the check runs in
the library's HIP kernels.  Importing this package fails loudly when the library has not
been built (python -m paper_2603_03592_amd.build, or __graft_entry__.build()).
"""
from .binding import (  # noqa: F401
    LIB_PATH, METRIC_BITS, OP_NAMES, METRIC_NAMES, RESULT_DTYPE, Policy, Sentinel, SVError, Verifier, adaptive_iqr, fuse_norm_pays, lib,
    score_and_flag_noalloc, sv_check_desc, sv_gemm_bf16, sv_workspace_bytes,
)
