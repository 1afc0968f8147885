"""MI355X-native batched Cholesky operator family (potrf, trsm, trmm, syrk, sumlogdiag and
the potrf backward expression) of arXiv 1710.08717, section 4.2.

The work is done by hand-written HIP kernels behind the C ABI declared in ``include/la.h``;
this package is only a thin ctypes binding that marshals ``torch`` device tensors
(pointer + stream) into those calls.  There is no CPU or PyTorch fallback: if the shared
library is missing, importing the binding raises.
"""
from .binding import (  # noqa: F401
    LaError,
    potrf_noalloc,
    workspace_bytes,
    gemm2,
    gemm2_backward,
    gp_glue,
    lib_path,
    load,
    potrf,
    sgp_criterion,
    kalman_filter,
    gp_criterion,
    potri,
    potri_backward,
    potrf_backward,
    sumlogdiag,
    syrk,
    syrk_backward,
    trmm,
    trmm_backward,
    trsm,
    trsm_backward,
)

__all__ = ["potrf", "potrf_backward", "trsm", "trmm", "syrk", "trsm_backward", "trmm_backward", "syrk_backward", "gemm2_backward", "potri", "potri_backward", "sgp_criterion", "kalman_filter", "gp_criterion", "sumlogdiag",
           "gp_glue", "gemm2", "load", "lib_path", "LaError", "workspace_bytes", "potrf_noalloc"]
