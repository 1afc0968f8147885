"""la_potrf_batched_noalloc (the entry point for callers that cannot allocate) against
la_potrf_batched_ws, through the C ABI (ctypes), two calls in a row on the same static scratch
array, the second with a smaller input; and its refusal of a problem beyond the array's size."""
import ctypes
import sys

import numpy as np
import pytest

import workloads

pytestmark = pytest.mark.gpu

TOL = {"f32": 2e-4, "f64": 1e-10}


def _spd(rng, batch, n, dtype):
    X = rng.standard_normal((batch, n, 2 * n))
    A = X @ X.transpose(0, 2, 1) / (2 * n) + np.eye(n)
    return A.astype(workloads.np_dtype(dtype))


def _relerr(x, ref):
    x = x.reshape(x.shape[0], -1).astype(np.float64)
    ref = ref.reshape(ref.shape[0], -1).astype(np.float64)
    return float(np.max(np.linalg.norm(x - ref, axis=1) / np.linalg.norm(ref, axis=1)))


@pytest.mark.parametrize("dtype", ["f64", "f32"])
def test_noalloc_potrf_matches_workspace_potrf_twice_in_a_row(dtype):
    import torch

    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1710_08717_amd import binding

    lib = binding.load()
    vp = ctypes.c_void_p
    dt = 0 if dtype == "f32" else 1
    rng = np.random.default_rng(20240607)
    stream = vp(torch.cuda.current_stream().cuda_stream)
    # first a problem that fills most of the static array, then a smaller one on what it left behind,
    # then one that needs no scratch at all
    for (batch, n, lower) in [(2, 1024, 1), (3, 384, 0), (5, 96, 1)]:
        sys.stderr.write(f"[noalloc] dtype={dtype} batch={batch} n={n} lower={lower}\n")
        sys.stderr.flush()
        A = torch.from_numpy(_spd(rng, batch, n, dtype)).cuda()
        need = int(lib.la_workspace_bytes(binding.OP_POTRF, dt, batch, n, 0, 0))
        assert need <= binding.NOALLOC_SCRATCH_BYTES
        assert (n <= 128) == (need == 0)
        ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
        L_ref = torch.full_like(A, float("nan"))
        L_new = torch.full_like(A, float("nan"))
        info_ref = torch.full((batch,), -1, dtype=torch.int32, device="cuda")
        info_new = torch.full((batch,), -1, dtype=torch.int32, device="cuda")
        rc = lib.la_potrf_batched_ws(dt, lower, batch, n, vp(A.data_ptr()), vp(L_ref.data_ptr()), vp(info_ref.data_ptr()),
                                     vp(ws.data_ptr()), ws.numel(), stream)
        assert rc == 0, lib.la_last_error()
        rc = lib.la_potrf_batched_noalloc(dt, lower, batch, n, vp(A.data_ptr()), vp(L_new.data_ptr()),
                                          vp(info_new.data_ptr()), stream)
        assert rc == 0, lib.la_last_error()
        torch.cuda.synchronize()
        ref, new = L_ref.cpu().numpy(), L_new.cpu().numpy()
        assert np.isfinite(new).all()
        assert (info_new.cpu().numpy() == 0).all() and (info_ref.cpu().numpy() == 0).all()
        assert _relerr(new, ref) <= TOL[dtype]
        tri = np.triu(np.ones((n, n), bool), 1) if lower else np.tril(np.ones((n, n), bool), -1)
        assert (new[:, tri] == 0).all()  # the other triangle is exact zeros
        # and the factor reproduces A to rounding
        Lf = new.astype(np.float64)
        R = Lf @ Lf.transpose(0, 2, 1) if lower else Lf.transpose(0, 2, 1) @ Lf
        assert _relerr(R, A.cpu().numpy().astype(np.float64)) <= TOL[dtype]


def test_noalloc_potrf_refuses_what_does_not_fit():
    import torch

    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1710_08717_amd import binding

    lib = binding.load()
    vp = ctypes.c_void_p
    batch, n = 32, 512  # 192 MiB of scratch in fp64
    assert int(lib.la_workspace_bytes(binding.OP_POTRF, 1, batch, n, 0, 0)) > binding.NOALLOC_SCRATCH_BYTES
    A = torch.eye(n, dtype=torch.float64, device="cuda").repeat(batch, 1, 1).contiguous()
    L = torch.full_like(A, 7.0)
    rc = lib.la_potrf_batched_noalloc(1, 1, batch, n, vp(A.data_ptr()), vp(L.data_ptr()), vp(0),
                                      vp(torch.cuda.current_stream().cuda_stream))
    assert rc == 4  # LA_ERR_WORKSPACE
    assert b"static buffer holds" in lib.la_last_error()
    torch.cuda.synchronize()
    assert (L == 7.0).all()  # nothing was launched
