"""CPU oracle for the batched Cholesky operator family -- TEST INFRASTRUCTURE ONLY.

Thin ctypes access to ``oracle.c`` (plain fp64 loops written from the paper's
operator statements, sections 3.1, 4.1, 4.2 and the appendix).  It shares nothing
with the HIP library and must never be imported by it.  Inputs are numpy arrays;
fp32 inputs are widened to fp64 exactly, results are always fp64.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force=False):
    """Compile oracle.c with gcc (OpenMP over the batch / independent right-hand sides)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int32)
        i64, i32, f64 = ctypes.c_int64, ctypes.c_int, ctypes.c_double
        lib.orc_potrf.argtypes = [i32, i64, i32, dp, dp, ip]
        lib.orc_potrf_backward.argtypes = [i32, i64, i32, dp, dp, dp]
        lib.orc_potrf_backward_phi.argtypes = [i64, i32, dp, dp, dp]
        lib.orc_trsm.argtypes = [i32, i32, i32, f64, i64, i32, i32, dp, dp, dp]
        lib.orc_trmm.argtypes = [i32, i32, i32, f64, i64, i32, i32, dp, dp, dp]
        lib.orc_syrk.argtypes = [i32, f64, i64, i32, i32, dp, dp]
        lib.orc_trmm_backward.argtypes = [i32, i32, i32, f64, i64, i32, i32, dp, dp, dp, dp, dp]
        lib.orc_trsm_backward.argtypes = [i32, i32, i32, f64, i64, i32, i32, dp, dp, dp, dp, dp]
        lib.orc_syrk_backward.argtypes = [i32, f64, i64, i32, i32, dp, dp, dp]
        lib.orc_gemm2_backward.argtypes = [i32, i32, f64, i64, i32, i32, i32, dp, dp, dp, dp, dp]
        lib.orc_potri.argtypes = [i32, i64, i32, dp, dp]
        lib.orc_potri_backward.argtypes = [i32, i64, i32, dp, dp, dp, dp]
        lib.orc_sgp_criterion.argtypes = [i32, i32, dp, dp, dp, dp, f64, dp, dp, dp, dp, dp, dp]
        lib.orc_sumlogdiag.argtypes = [i64, i32, dp, dp]
        lib.orc_kalman_filter.argtypes = [i64, i32, i32, i32, i32, dp, dp, dp, dp, dp, dp, dp, dp, dp, dp, ip]
        lib.orc_gemm2.argtypes = [i32, i32, f64, i64, i32, i32, i32, dp, dp, dp]
        lib.orc_gp_glue.argtypes = [i64, i32, dp, dp, dp, dp, dp, dp]
        lib.orc_llt_entry.argtypes = [i32, i32, dp, i32, i32]
        lib.orc_llt_entry.restype = f64
        lib.orc_ltxl_entry.argtypes = [i32, dp, dp, i32, i32]
        lib.orc_ltxl_entry.restype = f64
        lib.orc_ltlbar_entry.argtypes = [i32, dp, dp, i32, i32]
        lib.orc_ltlbar_entry.restype = f64
        lib.orc_num_threads.restype = i32
        _lib = lib
    return _lib


def num_threads():
    """Threads the OpenMP loops of the oracle use (what a timing of it ran on)."""
    return int(_load().orc_num_threads())


def _p(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _f64(a):
    return np.ascontiguousarray(np.asarray(a), dtype=np.float64)


def _check(rc, name):
    if rc != 0:
        raise ValueError(f"{name}: oracle rejected the arguments (status {rc})")


def _batch_of(a, trailing):
    """Flatten every leading axis into one batch count ("batch mode", section 4.1)."""
    lead = a.shape[: a.ndim - trailing]
    return int(np.prod(lead, dtype=np.int64)) if lead else 1


def potrf(A, lower=True, return_info=False):
    A = _f64(A)
    n = A.shape[-1]
    assert A.shape[-2] == n
    b = _batch_of(A, 2)
    L = np.empty_like(A)
    info = np.zeros(b, dtype=np.int32)
    _check(_load().orc_potrf(int(lower), b, n, _p(A), _p(L), info.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))), "potrf")
    return (L, info) if return_info else L


def potrf_inplace(A, lower=True):
    """Factor overwriting its (fp64, contiguous) input, as the paper allows."""
    assert A.dtype == np.float64 and A.flags.c_contiguous
    n = A.shape[-1]
    _check(_load().orc_potrf(int(lower), _batch_of(A, 2), n, _p(A), _p(A), None), "potrf")
    return A


def potrf_backward(L, Lbar, lower=True, inplace=False):
    L = _f64(L)
    Lbar = _f64(Lbar)
    n = L.shape[-1]
    assert L.shape == Lbar.shape and L.shape[-2] == n
    out = Lbar if inplace else np.empty_like(Lbar)
    _check(_load().orc_potrf_backward(int(lower), _batch_of(L, 2), n, _p(L), _p(Lbar), _p(out)), "potrf_backward")
    return out


def potrf_backward_phi(L, Lbar):
    L = _f64(L)
    Lbar = _f64(Lbar)
    n = L.shape[-1]
    out = np.empty_like(Lbar)
    _check(_load().orc_potrf_backward_phi(_batch_of(L, 2), n, _p(L), _p(Lbar), _p(out)), "potrf_backward_phi")
    return out


def _tri_op(fn, name, L, A, lower, trans, rightside, alpha, inplace):
    L = _f64(L)
    A = _f64(A)
    n = L.shape[-1]
    assert L.shape[-2] == n
    m = A.shape[-2] if rightside else A.shape[-1]
    assert (A.shape[-1] if rightside else A.shape[-2]) == n
    b = _batch_of(L, 2)
    assert _batch_of(A, 2) == b
    out = A if inplace else np.empty_like(A)
    _check(fn(int(lower), int(trans), int(rightside), float(alpha), b, n, m, _p(L), _p(A), _p(out)), name)
    return out


def trsm(L, A, lower=True, trans=False, rightside=False, alpha=1.0, inplace=False):
    return _tri_op(_load().orc_trsm, "trsm", L, A, lower, trans, rightside, alpha, inplace)


def trmm(L, A, lower=True, trans=False, rightside=False, alpha=1.0, inplace=False):
    return _tri_op(_load().orc_trmm, "trmm", L, A, lower, trans, rightside, alpha, inplace)


def syrk(A, trans=False, alpha=1.0):
    A = _f64(A)
    n, k = (A.shape[-1], A.shape[-2]) if trans else (A.shape[-2], A.shape[-1])
    b = _batch_of(A, 2)
    out = np.empty(A.shape[:-2] + (n, n), dtype=np.float64)
    _check(_load().orc_syrk(int(trans), float(alpha), b, n, k, _p(A), _p(out)), "syrk")
    return out


def _tri_backward(fn, name, L, X, Bbar, lower, trans, rightside, alpha):
    L, X, Bbar = _f64(L), _f64(X), _f64(Bbar)
    n = L.shape[-1]
    assert L.shape[-2] == n and X.shape == Bbar.shape
    m = X.shape[-2] if rightside else X.shape[-1]
    assert (X.shape[-1] if rightside else X.shape[-2]) == n
    b = _batch_of(L, 2)
    assert _batch_of(X, 2) == b
    Abar = np.empty_like(X)
    Lbar = np.empty_like(L)
    _check(fn(int(lower), int(trans), int(rightside), float(alpha), b, n, m, _p(L), _p(X), _p(Bbar), _p(Abar), _p(Lbar)),
           name)
    return Abar, Lbar


def trmm_backward(L, A, Bbar, lower=True, trans=False, rightside=False, alpha=1.0):
    """(Abar, Lbar) of B = alpha t(L) A / alpha A t(L); needs the forward input A."""
    return _tri_backward(_load().orc_trmm_backward, "trmm_backward", L, A, Bbar, lower, trans, rightside, alpha)


def trsm_backward(L, B, Bbar, lower=True, trans=False, rightside=False, alpha=1.0):
    """(Abar, Lbar) of B = alpha t(L)^-1 A / alpha A t(L)^-1; needs the forward OUTPUT B."""
    return _tri_backward(_load().orc_trsm_backward, "trsm_backward", L, B, Bbar, lower, trans, rightside, alpha)


def syrk_backward(A, Bbar, trans=False, alpha=1.0):
    A, Bbar = _f64(A), _f64(Bbar)
    n, k = (A.shape[-1], A.shape[-2]) if trans else (A.shape[-2], A.shape[-1])
    assert Bbar.shape[-2:] == (n, n)
    out = np.empty_like(A)
    _check(_load().orc_syrk_backward(int(trans), float(alpha), _batch_of(A, 2), n, k, _p(A), _p(Bbar), _p(out)),
           "syrk_backward")
    return out


def gemm2(A, B, ta=False, tb=False, alpha=1.0):
    A, B = _f64(A), _f64(B)
    m, k = (A.shape[-1], A.shape[-2]) if ta else (A.shape[-2], A.shape[-1])
    n = B.shape[-2] if tb else B.shape[-1]
    assert (B.shape[-1] if tb else B.shape[-2]) == k
    b = _batch_of(A, 2)
    out = np.empty(A.shape[:-2] + (m, n), dtype=np.float64)
    _check(_load().orc_gemm2(int(ta), int(tb), float(alpha), b, m, n, k, _p(A), _p(B), _p(out)), "gemm2")
    return out


def gemm2_backward(A, B, Cbar, ta=False, tb=False, alpha=1.0):
    """(Abar, Bbar) of C = alpha t_a(A) t_b(B), each in the shape of its operand."""
    A, B, Cbar = _f64(A), _f64(B), _f64(Cbar)
    m, k = (A.shape[-1], A.shape[-2]) if ta else (A.shape[-2], A.shape[-1])
    n = B.shape[-2] if tb else B.shape[-1]
    assert Cbar.shape[-2:] == (m, n)
    Abar, Bbar = np.empty_like(A), np.empty_like(B)
    _check(_load().orc_gemm2_backward(int(ta), int(tb), float(alpha), _batch_of(A, 2), m, n, k, _p(A), _p(B), _p(Cbar),
                                      _p(Abar), _p(Bbar)), "gemm2_backward")
    return Abar, Bbar


def potri(L, lower=True):
    """A^-1 from the Cholesky factor of A."""
    L = _f64(L)
    n = L.shape[-1]
    out = np.empty_like(L)
    _check(_load().orc_potri(int(lower), _batch_of(L, 2), n, _p(L), _p(out)), "potri")
    return out


def potri_backward(L, B, Bbar, lower=True):
    L, B, Bbar = _f64(L), _f64(B), _f64(Bbar)
    n = L.shape[-1]
    out = np.empty_like(L)
    _check(_load().orc_potri_backward(int(lower), _batch_of(L, 2), n, _p(L), _p(B), _p(Bbar), _p(out)), "potri_backward")
    return out


def sgp_criterion(Kuu, Kuf, Kff_diag, y, noise_var):
    """Sparse-GP criterion of section 3.2 and its gradient: dict with phi, Kuu_bar, Kuf_bar,
    Kff_diag_bar, y_bar, noise_bar."""
    Kuu, Kuf, Kff_diag, y = _f64(Kuu), _f64(Kuf), _f64(Kff_diag), _f64(y)
    U, n = Kuf.shape
    assert Kuu.shape == (U, U) and Kff_diag.shape == (n,) and y.shape == (n,)
    phi, lb = np.zeros(1), np.zeros(1)
    out = {"Kuu_bar": np.empty_like(Kuu), "Kuf_bar": np.empty_like(Kuf), "Kff_diag_bar": np.empty_like(Kff_diag),
           "y_bar": np.empty_like(y)}
    _check(_load().orc_sgp_criterion(U, n, _p(Kuu), _p(Kuf), _p(Kff_diag), _p(y), float(noise_var), _p(phi),
                                     _p(out["Kuu_bar"]), _p(out["Kuf_bar"]), _p(out["Kff_diag_bar"]), _p(out["y_bar"]),
                                     _p(lb)), "sgp_criterion")
    out["phi"], out["noise_bar"] = float(phi[0]), float(lb[0])
    return out


def kalman_filter(A, B, Sh, Sv, mu0, S0, v, want_states=True):
    """Section 3.4.  Parameters either without a batch axis (shared by all sequences) or with
    the batch axis of v ([batch, T, dv]).  Returns (nll [batch], f [batch, T, dh] or None,
    F [batch, T, dh, dh] or None, info [batch])."""
    v = _f64(v)
    batch, T, dv = v.shape
    A, B, Sh, Sv, mu0, S0 = (_f64(x) for x in (A, B, Sh, Sv, mu0, S0))
    shared = A.ndim == 2
    dh = A.shape[-1]
    pb = () if shared else (batch,)
    assert A.shape == pb + (dh, dh) and B.shape == pb + (dv, dh) and Sh.shape == pb + (dh, dh)
    assert Sv.shape == pb + (dv, dv) and mu0.shape == pb + (dh,) and S0.shape == pb + (dh, dh)
    nll = np.empty(batch)
    f = np.empty((batch, T, dh)) if want_states else None
    F = np.empty((batch, T, dh, dh)) if want_states else None
    info = np.zeros(batch, dtype=np.int32)
    _check(_load().orc_kalman_filter(batch, T, dh, dv, int(shared), _p(A), _p(B), _p(Sh), _p(Sv), _p(mu0), _p(S0),
                                     _p(v), _p(f) if want_states else None, _p(F) if want_states else None, _p(nll),
                                     info.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))), "kalman_filter")
    return nll, f, F, info


def sumlogdiag(L):
    L = _f64(L)
    n = L.shape[-1]
    out = np.empty(L.shape[:-2], dtype=np.float64)
    outf = out.reshape(-1) if out.ndim else out.reshape(1)
    _check(_load().orc_sumlogdiag(_batch_of(L, 2), n, _p(L), _p(outf)), "sumlogdiag")
    return out


def gp_glue(L, y, z, alpha):
    """loss = 1/2 y^T alpha + sum log l_ii and Lbar = -tril(alpha z^T) + diag(1/l_ii)."""
    L, y, z, alpha = _f64(L), _f64(y), _f64(z), _f64(alpha)
    n = L.shape[-1]
    b = _batch_of(L, 2)
    loss = np.empty(L.shape[:-2], dtype=np.float64)
    lossf = loss.reshape(-1) if loss.ndim else loss.reshape(1)
    Lbar = np.empty_like(L)
    _check(_load().orc_gp_glue(b, n, _p(L), _p(y), _p(z), _p(alpha), _p(lossf), _p(Lbar)), "gp_glue")
    return loss, Lbar


def llt_entry(L, i, j, lower=True):
    L = _f64(L)
    return _load().orc_llt_entry(int(lower), L.shape[-1], _p(L), int(i), int(j))


def ltxl_entry(L, X, i, j):
    L, X = _f64(L), _f64(X)
    return _load().orc_ltxl_entry(L.shape[-1], _p(L), _p(X), int(i), int(j))


def ltlbar_entry(L, Lbar, i, j):
    L, Lbar = _f64(L), _f64(Lbar)
    return _load().orc_ltlbar_entry(L.shape[-1], _p(L), _p(Lbar), int(i), int(j))
