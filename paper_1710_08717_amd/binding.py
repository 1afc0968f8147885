"""ctypes binding of ``libla_mi355x.so``: argument marshalling only.

Each function mirrors one ``la_*`` entry point of ``include/la.h``.  Tensors must live on
the GPU, be contiguous and be float32 or float64; all leading axes are flattened into the
batch ("batch mode", section 4.1 of the paper).  Work is enqueued on torch's current
stream.
"""
import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libla_mi355x.so")
_lib = None

SYMBOLS = [
    "la_potrf_batched", "la_potrf_backward", "la_trsm_batched", "la_trmm_batched", "la_syrk_batched",
    "la_sumlogdiag", "la_gp_glue", "la_gemm2_batched", "la_trsm_backward", "la_trmm_backward", "la_syrk_backward",
    "la_gemm2_backward", "la_potri", "la_potri_backward", "la_sgp_workspace_bytes", "la_sgp_criterion",
    "la_kalman_filter", "la_gp_workspace_bytes", "la_gp_criterion",
    "la_last_error", "la_version",
    "la_workspace_bytes", "la_potrf_batched_ws", "la_potrf_backward_ws", "la_trsm_batched_ws", "la_trmm_batched_ws",
    "la_syrk_batched_ws", "la_gemm2_batched_ws", "la_trsm_backward_ws", "la_trmm_backward_ws", "la_syrk_backward_ws",
    "la_gemm2_backward_ws", "la_potri_ws", "la_potri_backward_ws", "la_potrf_batched_noalloc",
]

# la_op of include/la.h
OP_POTRF, OP_POTRF_BACKWARD, OP_TRSM, OP_TRMM, OP_SYRK, OP_GEMM2 = 0, 1, 2, 3, 4, 5
OP_TRSM_BACKWARD, OP_TRMM_BACKWARD, OP_SYRK_BACKWARD, OP_GEMM2_BACKWARD, OP_POTRI, OP_POTRI_BACKWARD = 6, 7, 8, 9, 10, 11


class LaError(RuntimeError):
    pass


def lib_path():
    return _LIB_PATH


def load():
    """Load the HIP library (built beforehand by ``paper_1710_08717_amd.build``); raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise LaError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_1710_08717_amd.build` "
            "(there is no fallback path)"
        )
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64, f64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_double
    lib.la_potrf_batched.argtypes = [i32, i32, i64, i32, vp, vp, vp, vp]
    lib.la_potrf_backward.argtypes = [i32, i32, i64, i32, vp, vp, vp, vp]
    lib.la_trsm_batched.argtypes = [i32, i32, i32, i32, f64, i64, i32, i32, vp, vp, vp, vp]
    lib.la_trmm_batched.argtypes = [i32, i32, i32, i32, f64, i64, i32, i32, vp, vp, vp, vp]
    lib.la_syrk_batched.argtypes = [i32, i32, f64, i64, i32, i32, vp, vp, vp]
    lib.la_sumlogdiag.argtypes = [i32, i64, i32, vp, vp, vp]
    lib.la_gp_glue.argtypes = [i32, i64, i32, vp, vp, vp, vp, vp, vp, vp]
    lib.la_gemm2_batched.argtypes = [i32, i32, i32, f64, i64, i32, i32, i32, vp, vp, vp, vp]
    lib.la_gemm2_batched.restype = i32
    lib.la_trsm_backward.argtypes = [i32, i32, i32, i32, f64, i64, i32, i32, vp, vp, vp, vp, vp, vp]
    lib.la_trmm_backward.argtypes = [i32, i32, i32, i32, f64, i64, i32, i32, vp, vp, vp, vp, vp, vp]
    lib.la_syrk_backward.argtypes = [i32, i32, f64, i64, i32, i32, vp, vp, vp, vp]
    lib.la_gemm2_backward.argtypes = [i32, i32, i32, f64, i64, i32, i32, i32, vp, vp, vp, vp, vp, vp]
    lib.la_potri.argtypes = [i32, i32, i64, i32, vp, vp, vp]
    lib.la_potri_backward.argtypes = [i32, i32, i64, i32, vp, vp, vp, vp, vp]
    for name in ("la_trsm_backward", "la_trmm_backward", "la_syrk_backward", "la_gemm2_backward", "la_potri",
                 "la_potri_backward"):
        getattr(lib, name).restype = i32
    lib.la_sgp_workspace_bytes.argtypes = [i32, i32, i32]
    lib.la_sgp_workspace_bytes.restype = ctypes.c_size_t
    lib.la_sgp_criterion.argtypes = [i32, i32, i32, vp, vp, vp, vp, f64, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.la_sgp_criterion.restype = i32
    lib.la_kalman_filter.argtypes = [i32, i64, i32, i32, i32, i32] + [vp] * 12
    lib.la_kalman_filter.restype = i32
    lib.la_gp_workspace_bytes.argtypes = [i32, i64, i32]
    lib.la_gp_workspace_bytes.restype = ctypes.c_size_t
    lib.la_gp_criterion.argtypes = [i32, i64, i32, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.la_gp_criterion.restype = i32
    lib.la_last_error.restype = ctypes.c_char_p
    lib.la_version.restype = i32
    for name in SYMBOLS[:7]:
        getattr(lib, name).restype = i32
    lib.la_potrf_batched_noalloc.argtypes = lib.la_potrf_batched.argtypes
    lib.la_potrf_batched_noalloc.restype = i32
    lib.la_workspace_bytes.argtypes = [i32, i32, i64, i32, i32, i32]
    lib.la_workspace_bytes.restype = ctypes.c_size_t
    # the _ws form of an entry point: its arguments with (workspace, workspace_bytes) before the stream
    for name in SYMBOLS:
        if name.endswith("_ws"):
            plain = getattr(lib, name[:-3])
            f = getattr(lib, name)
            f.argtypes = plain.argtypes[:-1] + [vp, ctypes.c_size_t, vp]
            f.restype = i32
    _lib = lib
    return lib


_STATUS = {1: "LA_ERR_INVALID_ARG", 2: "LA_ERR_UNSUPPORTED", 3: "LA_ERR_RUNTIME", 4: "LA_ERR_WORKSPACE"}


def _check(rc, name):
    if rc != 0:
        msg = f"{name}: {_STATUS.get(rc, rc)}"
        if rc in (3, 4):
            msg += f" ({load().la_last_error().decode()})"
        raise LaError(msg)


def _dt(t):
    if t.dtype == torch.float32:
        return 0
    if t.dtype == torch.float64:
        return 1
    raise LaError(f"unsupported dtype {t.dtype}")


def _chk(*ts):
    d = ts[0]
    for t in ts:
        if not t.is_cuda:
            raise LaError("tensors must be on the GPU")
        if not t.is_contiguous():
            raise LaError("tensors must be contiguous")
        if t.dtype != d.dtype or t.device != d.device:
            raise LaError("tensors must share dtype and device")


def _stream(t):
    return ctypes.c_void_p(torch.cuda.current_stream(t.device).cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def _batch(t, trailing=2):
    b = 1
    for s in t.shape[: t.dim() - trailing]:
        b *= s
    return b


_ws_sizes = {}


def workspace_bytes(op, t, batch, n=0, m=0, k=0):
    """la_workspace_bytes for tensors of t's dtype (the answers are remembered: they depend on the sizes only)."""
    key = (op, t.dtype, batch, n, m, k)
    need = _ws_sizes.get(key)
    if need is None:
        need = _ws_sizes[key] = int(load().la_workspace_bytes(op, _dt(t), batch, n, m, k))
    return need


def _ws(workspace, op, t, batch, n=0, m=0, k=0):
    """(tensor, pointer, bytes) of the scratch memory of one call: the caller's uint8 device tensor, or, when the call
    needs one and none was given, a fresh one from torch's allocator (stream-ordered on the current stream)."""
    if workspace is not None:
        assert workspace.dtype == torch.uint8 and workspace.is_cuda and workspace.is_contiguous()
        return workspace, ctypes.c_void_p(workspace.data_ptr()), workspace.numel()
    need = workspace_bytes(op, t, batch, n, m, k)
    if need == 0:
        return None, ctypes.c_void_p(0), 0
    buf = torch.empty(need, dtype=torch.uint8, device=t.device)
    return buf, ctypes.c_void_p(buf.data_ptr()), need  # the caller keeps buf until the call is enqueued


def potrf(A, lower=True, out=None, info=None, workspace=None):
    """la_potrf_batched.  ``out`` may be ``A`` itself (in place).  ``info``: int32 [batch] or None."""
    _chk(A)
    n = A.shape[-1]
    assert A.shape[-2] == n
    L = torch.empty_like(A) if out is None else out
    _chk(A, L)
    if info is not None:
        assert info.dtype == torch.int32 and info.is_cuda and info.numel() == _batch(A)
    with torch.cuda.device(A.device):
        keep, wp, wb = _ws(workspace, OP_POTRF, A, _batch(A), n)
        _check(load().la_potrf_batched_ws(_dt(A), int(lower), _batch(A), n, _ptr(A), _ptr(L), _ptr(info), wp, wb,
                                          _stream(A)), "la_potrf_batched_ws")
    return L


NOALLOC_SCRATCH_BYTES = 64 << 20  # LA_NOALLOC_SCRATCH_BYTES of include/la.h


def potrf_noalloc(A, out, lower=True, info=None):
    """la_potrf_batched_noalloc: potrf on the library's static scratch array; the caller supplies ``out``
    (which may be ``A``), nothing is allocated here or in the library."""
    _chk(A, out)
    n = A.shape[-1]
    assert A.shape[-2] == n and out.shape == A.shape
    if info is not None:
        assert info.dtype == torch.int32 and info.is_cuda and info.numel() == _batch(A)
    with torch.cuda.device(A.device):
        _check(load().la_potrf_batched_noalloc(_dt(A), int(lower), _batch(A), n, _ptr(A), _ptr(out), _ptr(info),
                                               _stream(A)), "la_potrf_batched_noalloc")
    return out


def potrf_backward(L, Lbar, lower=True, out=None, workspace=None):
    """la_potrf_backward.  ``out`` may be ``Lbar`` itself."""
    _chk(L, Lbar)
    n = L.shape[-1]
    assert L.shape == Lbar.shape and L.shape[-2] == n
    Abar = torch.empty_like(Lbar) if out is None else out
    _chk(L, Abar)
    with torch.cuda.device(L.device):
        keep, wp, wb = _ws(workspace, OP_POTRF_BACKWARD, L, _batch(L), n)
        _check(load().la_potrf_backward_ws(_dt(L), int(lower), _batch(L), n, _ptr(L), _ptr(Lbar), _ptr(Abar), wp, wb,
                                           _stream(L)), "la_potrf_backward_ws")
    return Abar


def _tri(op, name, L, A, lower, trans, rightside, alpha, out, workspace):
    _chk(L, A)
    n = L.shape[-1]
    assert L.shape[-2] == n
    m = A.shape[-2] if rightside else A.shape[-1]
    assert (A.shape[-1] if rightside else A.shape[-2]) == n
    assert _batch(L) == _batch(A)
    B = torch.empty_like(A) if out is None else out
    _chk(A, B)
    with torch.cuda.device(L.device):
        keep, wp, wb = _ws(workspace, op, L, _batch(L), n, m)
        _check(getattr(load(), name)(_dt(L), int(lower), int(trans), int(rightside), float(alpha), _batch(L), n, m,
                                     _ptr(L), _ptr(A), _ptr(B), wp, wb, _stream(L)), name)
    return B


def trsm(L, A, lower=True, trans=False, rightside=False, alpha=1.0, out=None, workspace=None):
    return _tri(OP_TRSM, "la_trsm_batched_ws", L, A, lower, trans, rightside, alpha, out, workspace)


def trmm(L, A, lower=True, trans=False, rightside=False, alpha=1.0, out=None, workspace=None):
    return _tri(OP_TRMM, "la_trmm_batched_ws", L, A, lower, trans, rightside, alpha, out, workspace)


def _tri_backward(op, name, L, X, Bbar, lower, trans, rightside, alpha, out_a, out_l, workspace):
    _chk(L, X)
    _chk(L, Bbar)
    n = L.shape[-1]
    assert L.shape[-2] == n and X.shape == Bbar.shape
    m = X.shape[-2] if rightside else X.shape[-1]
    assert (X.shape[-1] if rightside else X.shape[-2]) == n and _batch(L) == _batch(X)
    Abar = torch.empty_like(Bbar) if out_a is None else out_a
    Lbar = torch.empty_like(L) if out_l is None else out_l
    _chk(L, Abar)
    _chk(L, Lbar)
    with torch.cuda.device(L.device):
        keep, wp, wb = _ws(workspace, op, L, _batch(L), n, m)
        _check(getattr(load(), name)(_dt(L), int(lower), int(trans), int(rightside), float(alpha), _batch(L), n, m,
                                     _ptr(L), _ptr(X), _ptr(Bbar), _ptr(Abar), _ptr(Lbar), wp, wb, _stream(L)), name)
    return Abar, Lbar


def trsm_backward(L, B, Bbar, lower=True, trans=False, rightside=False, alpha=1.0, out_a=None, out_l=None,
                  workspace=None):
    """la_trsm_backward: (Abar, Lbar) from the forward OUTPUT B.  out_a may be Bbar, out_l may be L."""
    return _tri_backward(OP_TRSM_BACKWARD, "la_trsm_backward_ws", L, B, Bbar, lower, trans, rightside, alpha, out_a,
                         out_l, workspace)


def trmm_backward(L, A, Bbar, lower=True, trans=False, rightside=False, alpha=1.0, out_a=None, out_l=None,
                  workspace=None):
    """la_trmm_backward: (Abar, Lbar) from the forward INPUT A.  out_a may be Bbar."""
    return _tri_backward(OP_TRMM_BACKWARD, "la_trmm_backward_ws", L, A, Bbar, lower, trans, rightside, alpha, out_a,
                         out_l, workspace)


def syrk_backward(A, Bbar, trans=False, alpha=1.0, out=None, workspace=None):
    """la_syrk_backward: Abar = alpha (Bbar + Bbar^T) A  or  alpha A (Bbar + Bbar^T)."""
    _chk(A, Bbar)
    n, k = (A.shape[-1], A.shape[-2]) if trans else (A.shape[-2], A.shape[-1])
    assert Bbar.shape[-2:] == (n, n) and _batch(A) == _batch(Bbar)
    Abar = torch.empty_like(A) if out is None else out
    _chk(A, Abar)
    with torch.cuda.device(A.device):
        keep, wp, wb = _ws(workspace, OP_SYRK_BACKWARD, A, _batch(A), n, 0, k)
        _check(load().la_syrk_backward_ws(_dt(A), int(trans), float(alpha), _batch(A), n, k, _ptr(A), _ptr(Bbar),
                                          _ptr(Abar), wp, wb, _stream(A)), "la_syrk_backward_ws")
    return Abar


def gemm2_backward(A, B, Cbar, ta=False, tb=False, alpha=1.0, workspace=None):
    """la_gemm2_backward: (Abar, Bbar) of C = alpha t_a(A) t_b(B)."""
    _chk(A, B)
    _chk(A, Cbar)
    m, k = (A.shape[-1], A.shape[-2]) if ta else (A.shape[-2], A.shape[-1])
    n = B.shape[-2] if tb else B.shape[-1]
    assert Cbar.shape[-2:] == (m, n) and _batch(A) == _batch(B) == _batch(Cbar)
    Abar, Bbar = torch.empty_like(A), torch.empty_like(B)
    with torch.cuda.device(A.device):
        keep, wp, wb = _ws(workspace, OP_GEMM2_BACKWARD, A, _batch(A), n, m, k)
        _check(load().la_gemm2_backward_ws(_dt(A), int(ta), int(tb), float(alpha), _batch(A), m, n, k, _ptr(A), _ptr(B),
                                           _ptr(Cbar), _ptr(Abar), _ptr(Bbar), wp, wb, _stream(A)),
               "la_gemm2_backward_ws")
    return Abar, Bbar


def potri(L, lower=True, out=None, workspace=None):
    """la_potri: A^-1 from the Cholesky factor of A.  ``out`` may be ``L`` itself."""
    _chk(L)
    n = L.shape[-1]
    assert L.shape[-2] == n
    B = torch.empty_like(L) if out is None else out
    _chk(L, B)
    with torch.cuda.device(L.device):
        keep, wp, wb = _ws(workspace, OP_POTRI, L, _batch(L), n)
        _check(load().la_potri_ws(_dt(L), int(lower), _batch(L), n, _ptr(L), _ptr(B), wp, wb, _stream(L)), "la_potri_ws")
    return B


def potri_backward(L, B, Bbar, lower=True, out=None, workspace=None):
    """la_potri_backward: gradient of the factor from B = A^-1 and Bbar."""
    _chk(L, B)
    _chk(L, Bbar)
    n = L.shape[-1]
    assert L.shape == B.shape == Bbar.shape
    Lbar = torch.empty_like(L) if out is None else out
    _chk(L, Lbar)
    with torch.cuda.device(L.device):
        keep, wp, wb = _ws(workspace, OP_POTRI_BACKWARD, L, _batch(L), n)
        _check(load().la_potri_backward_ws(_dt(L), int(lower), _batch(L), n, _ptr(L), _ptr(B), _ptr(Bbar), _ptr(Lbar),
                                           wp, wb, _stream(L)), "la_potri_backward_ws")
    return Lbar


def sgp_criterion(Kuu, Kuf, Kff_diag, y, noise_var, workspace=None):
    """la_sgp_criterion: dict with phi, Kuu_bar, Kuf_bar, Kff_diag_bar, y_bar, noise_bar (device tensors).
    ``workspace``: a uint8 device tensor of at least la_sgp_workspace_bytes bytes (allocated here if absent)."""
    _chk(Kuu, Kuf)
    _chk(Kuu, Kff_diag)
    _chk(Kuu, y)
    U, n = Kuf.shape
    assert Kuu.shape == (U, U) and Kff_diag.shape == (n,) and y.shape == (n,)
    need = int(load().la_sgp_workspace_bytes(_dt(Kuu), U, n))
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=Kuu.device)
    out = {"phi": torch.empty(1, dtype=Kuu.dtype, device=Kuu.device), "Kuu_bar": torch.empty_like(Kuu),
           "Kuf_bar": torch.empty_like(Kuf), "Kff_diag_bar": torch.empty_like(Kff_diag), "y_bar": torch.empty_like(y),
           "noise_bar": torch.empty(1, dtype=Kuu.dtype, device=Kuu.device)}
    with torch.cuda.device(Kuu.device):
        _check(load().la_sgp_criterion(_dt(Kuu), U, n, _ptr(Kuu), _ptr(Kuf), _ptr(Kff_diag), _ptr(y), float(noise_var),
                                       _ptr(out["phi"]), _ptr(out["Kuu_bar"]), _ptr(out["Kuf_bar"]),
                                       _ptr(out["Kff_diag_bar"]), _ptr(out["y_bar"]), _ptr(out["noise_bar"]),
                                       workspace.data_ptr(), workspace.numel(), _stream(Kuu)), "la_sgp_criterion")
    return out


def gp_criterion(A, y, out=None, loss=None, info=None, workspace=None):
    """la_gp_criterion: (loss [batch], Abar [batch, n, n]).  ``out`` may be ``A`` itself."""
    _chk(A, y)
    n = A.shape[-1]
    batch = _batch(A)
    assert A.shape[-2] == n and y.shape[-1] == n and _batch(y, 1) == batch
    Abar = torch.empty_like(A) if out is None else out
    _chk(A, Abar)
    if loss is None:
        loss = torch.empty(A.shape[:-2], dtype=A.dtype, device=A.device)
    _chk(A, loss)
    need = int(load().la_gp_workspace_bytes(_dt(A), batch, n))
    if need and workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=A.device)
    if info is not None:
        assert info.dtype == torch.int32 and info.is_cuda and info.numel() == batch
    with torch.cuda.device(A.device):
        _check(load().la_gp_criterion(_dt(A), batch, n, _ptr(A), _ptr(y), _ptr(loss), _ptr(Abar), _ptr(info),
                                      ctypes.c_void_p(workspace.data_ptr() if need else 0),
                                      workspace.numel() if need else 0, _stream(A)), "la_gp_criterion")
    return loss, Abar


def kalman_filter(A, B, Sh, Sv, mu0, S0, v, want_states=True, info=None):
    """la_kalman_filter.  Parameters without a batch axis are shared by all sequences of v [batch, T, dv];
    otherwise they carry v's batch axis.  Returns (nll [batch], f [batch, T, dh] or None, F [batch, T, dh, dh] or None)."""
    for x in (B, Sh, Sv, mu0, S0, v):
        _chk(A, x)
    batch, T, dv = v.shape
    shared = A.dim() == 2
    dh = A.shape[-1]
    pb = () if shared else (batch,)
    assert tuple(A.shape) == pb + (dh, dh) and tuple(B.shape) == pb + (dv, dh) and tuple(Sh.shape) == pb + (dh, dh)
    assert tuple(Sv.shape) == pb + (dv, dv) and tuple(mu0.shape) == pb + (dh,) and tuple(S0.shape) == pb + (dh, dh)
    nll = torch.empty(batch, dtype=v.dtype, device=v.device)
    f = torch.empty((batch, T, dh), dtype=v.dtype, device=v.device) if want_states else None
    F = torch.empty((batch, T, dh, dh), dtype=v.dtype, device=v.device) if want_states else None
    if info is not None:
        assert info.dtype == torch.int32 and info.is_cuda and info.numel() == batch
    with torch.cuda.device(v.device):
        _check(load().la_kalman_filter(_dt(v), batch, T, dh, dv, int(shared), _ptr(A), _ptr(B), _ptr(Sh), _ptr(Sv),
                                       _ptr(mu0), _ptr(S0), _ptr(v), _ptr(f), _ptr(F), _ptr(nll), _ptr(info),
                                       _stream(v)), "la_kalman_filter")
    return nll, f, F


def syrk(A, trans=False, alpha=1.0, out=None, workspace=None):
    _chk(A)
    n, k = (A.shape[-1], A.shape[-2]) if trans else (A.shape[-2], A.shape[-1])
    B = torch.empty(A.shape[:-2] + (n, n), dtype=A.dtype, device=A.device) if out is None else out
    _chk(A, B)
    with torch.cuda.device(A.device):
        keep, wp, wb = _ws(workspace, OP_SYRK, A, _batch(A), n, 0, k)
        _check(load().la_syrk_batched_ws(_dt(A), int(trans), float(alpha), _batch(A), n, k, _ptr(A), _ptr(B), wp, wb,
                                         _stream(A)), "la_syrk_batched_ws")
    return B


def gemm2(A, B, ta=False, tb=False, alpha=1.0, out=None, workspace=None):
    """la_gemm2_batched: C = alpha * t_a(A) t_b(B)."""
    _chk(A, B)
    m, k = (A.shape[-1], A.shape[-2]) if ta else (A.shape[-2], A.shape[-1])
    n = B.shape[-2] if tb else B.shape[-1]
    assert (B.shape[-1] if tb else B.shape[-2]) == k and _batch(A) == _batch(B)
    C = torch.empty(A.shape[:-2] + (m, n), dtype=A.dtype, device=A.device) if out is None else out
    _chk(A, C)
    with torch.cuda.device(A.device):
        keep, wp, wb = _ws(workspace, OP_GEMM2, A, _batch(A), n, m, k)
        _check(load().la_gemm2_batched_ws(_dt(A), int(ta), int(tb), float(alpha), _batch(A), m, n, k, _ptr(A), _ptr(B),
                                          _ptr(C), wp, wb, _stream(A)), "la_gemm2_batched_ws")
    return C


def sumlogdiag(L, out=None):
    _chk(L)
    n = L.shape[-1]
    o = torch.empty(L.shape[:-2], dtype=L.dtype, device=L.device) if out is None else out
    with torch.cuda.device(L.device):
        _check(load().la_sumlogdiag(_dt(L), _batch(L), n, _ptr(L), _ptr(o), _stream(L)), "la_sumlogdiag")
    return o


def gp_glue(L, y, z, alpha, loss=None, Lbar=None):
    _chk(L, y, z, alpha)
    n = L.shape[-1]
    loss = torch.empty(L.shape[:-2], dtype=L.dtype, device=L.device) if loss is None else loss
    Lbar = torch.empty_like(L) if Lbar is None else Lbar
    with torch.cuda.device(L.device):
        _check(load().la_gp_glue(_dt(L), _batch(L), n, _ptr(L), _ptr(y), _ptr(z), _ptr(alpha), _ptr(loss), _ptr(Lbar),
                                 _stream(L)), "la_gp_glue")
    return loss, Lbar
