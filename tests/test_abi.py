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


def test_workspace_sizes_are_host_only_and_cover_the_blocked_paths(lib):
    lib.la_workspace_bytes.restype = ctypes.c_size_t
    POTRF, BACKWARD, TRSM, TRMM, SYRK = 0, 1, 2, 3, 4
    # the register / one-workgroup paths need none
    for (dt, batch, n) in [(0, 65536, 16), (1, 16, 32), (0, 256, 128), (1, 7, 64)]:
        assert lib.la_workspace_bytes(POTRF, dt, batch, n, 0, 0) == 0
    assert lib.la_workspace_bytes(BACKWARD, 0, 256, 128, 0, 0) == 0
    assert lib.la_workspace_bytes(BACKWARD, 1, 16, 96, 0, 0) == 0
    assert lib.la_workspace_bytes(TRSM, 1, 16, 128, 48, 0) == 0
    # the blocked paths: a few matrices' worth, growing with the problem
    for dt, es in ((0, 4), (1, 8)):
        prev = 0
        for n in (256, 512, 1024, 4096, 8192):
            w = lib.la_workspace_bytes(POTRF, dt, 1, n, 0, 0)
            assert 2 * n * n * es <= w <= 3 * n * n * es + (64 << 20)
            assert w > prev and w % 256 == 0
            prev = w
        assert lib.la_workspace_bytes(BACKWARD, dt, 32, 512, 0, 0) >= 2 * 32 * 512 * 512 * es
        assert lib.la_workspace_bytes(TRSM, dt, 32, 512, 64, 0) == 0  # one launch that streams the factor
        assert lib.la_workspace_bytes(TRSM, dt, 8, 1024, 64, 0) >= 8 * 1024 * 1024 * es
    # bad arguments
    assert lib.la_workspace_bytes(99, 0, 1, 512, 0, 0) == 0
    assert lib.la_workspace_bytes(POTRF, 5, 1, 512, 0, 0) == 0
    assert lib.la_workspace_bytes(POTRF, 0, -1, 512, 0, 0) == 0


def test_blocked_call_without_enough_workspace_is_refused_before_any_launch(lib):
    WORKSPACE, INVALID = 4, 1
    p = ctypes.c_void_p(1 << 30)
    q = ctypes.c_void_p(2 << 30)
    w = ctypes.c_void_p(3 << 30)
    none = ctypes.c_void_p(0)
    n = 512
    lib.la_workspace_bytes.restype = ctypes.c_size_t
    need = lib.la_workspace_bytes(0, 1, 1, n, 0, 0)
    assert need > 0
    # the plain form is the _ws form without a workspace
    assert lib.la_potrf_batched(1, 1, 1, n, p, q, none, none) == WORKSPACE
    assert b"workspace" in lib.la_last_error()
    assert lib.la_potrf_batched_ws(1, 1, 1, n, p, q, none, none, 0, none) == WORKSPACE
    assert lib.la_potrf_batched_ws(1, 1, 1, n, p, q, none, w, need - 256, none) == WORKSPACE
    assert lib.la_potrf_backward(1, 1, 1, n, p, q, w, none) == WORKSPACE
    assert lib.la_trsm_batched(1, 1, 0, 0, 1.0, 1, 1024, 64, p, q, w, none) == WORKSPACE  # (n <= 512 needs none)
    # misaligned workspace, workspace over an operand
    assert lib.la_potrf_batched_ws(1, 1, 1, n, p, q, none, ctypes.c_void_p((3 << 30) + 8), need, none) == INVALID
    assert lib.la_potrf_batched_ws(1, 1, 1, n, p, q, none, ctypes.c_void_p((1 << 30) + 256), need, none) == INVALID
    # the noalloc form checks its arguments before it looks at the device
    assert lib.la_potrf_batched_noalloc(7, 1, 1, 4, p, q, none, none) == INVALID
    assert lib.la_potrf_batched_noalloc(1, 1, 0, 4, none, none, none, none) == 0
