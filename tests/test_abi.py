"""The C-ABI library loads, exports every symbol include/la.h declares, and rejects bad
arguments on the host before anything is launched (no GPU needed for any of this)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_1710_08717_amd import binding

    if not os.path.exists(binding.lib_path()):
        from paper_1710_08717_amd import build

        build.build(force=False)
    return binding.load()


def declared_symbols():
    hdr = open(os.path.join(ROOT, "include", "la.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    return sorted(set(re.findall(r"\b(la_[a-z_0-9]+)\s*\(", hdr)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert {"la_potrf_batched", "la_potrf_backward", "la_trsm_batched", "la_trmm_batched", "la_syrk_batched",
            "la_sumlogdiag"} <= set(names)
    for n in names:
        assert getattr(lib, n) is not None
    from paper_1710_08717_amd import binding

    assert set(binding.SYMBOLS) == set(names)


def test_version_and_error_text(lib):
    assert lib.la_version() >= 100
    assert isinstance(lib.la_last_error(), bytes)


def test_host_side_argument_checks(lib):
    OK, INVALID = 0, 1
    p = ctypes.c_void_p(4096)  # never dereferenced: every call below stops at validation or is empty
    q = ctypes.c_void_p(8192 + 4096)
    none = ctypes.c_void_p(0)
    # empty work is fine, even with null pointers
    assert lib.la_potrf_batched(1, 1, 0, 8, none, none, none, none) == OK
    assert lib.la_potrf_batched(1, 1, 5, 0, none, none, none, none) == OK
    assert lib.la_potrf_backward(0, 1, 0, 8, none, none, none, none) == OK
    assert lib.la_trsm_batched(0, 1, 0, 0, 1.0, 3, 4, 0, none, none, none, none) == OK
    assert lib.la_trmm_batched(0, 1, 0, 0, 1.0, 0, 4, 4, none, none, none, none) == OK
    assert lib.la_syrk_batched(0, 0, 1.0, 0, 4, 4, none, none, none) == OK
    assert lib.la_sumlogdiag(0, 0, 4, none, none, none) == OK
    assert lib.la_gp_glue(0, 0, 4, none, none, none, none, none, none, none) == OK
    # bad enum, negative sizes, null pointers with real work
    assert lib.la_potrf_batched(7, 1, 1, 4, p, q, none, none) == INVALID
    assert lib.la_potrf_batched(1, 1, -1, 4, p, q, none, none) == INVALID
    assert lib.la_potrf_batched(1, 1, 1, -4, p, q, none, none) == INVALID
    assert lib.la_potrf_batched(1, 1, 1, 4, none, q, none, none) == INVALID
    assert lib.la_potrf_backward(1, 1, 1, 4, p, none, q, none) == INVALID
    assert lib.la_trsm_batched(1, 1, 0, 0, 1.0, 1, 4, 2, p, none, q, none) == INVALID
    assert lib.la_trmm_batched(1, 1, 0, 0, 1.0, 1, 4, -2, p, p, q, none) == INVALID
    assert lib.la_syrk_batched(1, 0, 1.0, 1, 4, 4, none, q, none) == INVALID
    assert lib.la_sumlogdiag(1, 2, 4, p, none, none) == INVALID
    # forbidden aliasing: partial overlap, output over the factor, syrk in place
    part = ctypes.c_void_p(4096 + 64)
    assert lib.la_potrf_batched(1, 1, 1, 4, p, part, none, none) == INVALID
    assert lib.la_potrf_backward(1, 1, 1, 4, p, q, p, none) == INVALID
    assert lib.la_trsm_batched(1, 1, 0, 0, 1.0, 1, 4, 4, p, q, p, none) == INVALID
    assert lib.la_syrk_batched(1, 0, 1.0, 1, 4, 4, p, p, none) == INVALID


def test_binding_refuses_cpu_tensors():
    import torch

    import paper_1710_08717_amd as la

    with pytest.raises(la.LaError):
        la.potrf(torch.eye(4)[None])
