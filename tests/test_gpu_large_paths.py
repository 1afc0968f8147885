"""Element-by-element parity with the CPU oracle on the code paths only a large single matrix takes
(section 4.2: potrf and its backward expression): potrf right-looking over panels of 2048 columns
(one matrix of n >= 4096), the backward pass as the closed expression on a 2048 x 2048 block with
every merge level of the explicit inverse, and the reverse sweep over the blocked factorisation
with 2048-row base blocks (n = 4096: halving; n = 5376: a first block of 2048 peeled off, ragged
remainder).  Spec tolerances, relative Frobenius error of the whole matrix."""
import sys
import time

import numpy as np
import pytest

import workloads

pytestmark = pytest.mark.gpu

TOL = {"f32": 2e-4, "f64": 1e-10}


@pytest.fixture(scope="module")
def la():
    import torch

    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1710_08717_amd as la_mod

    la_mod.load()
    return la_mod


@pytest.fixture(autouse=True)
def _announce(request):
    sys.stderr.write(f"\n[gpu-case] {request.node.nodeid}\n")
    sys.stderr.flush()
    yield


def dev(a):
    import torch

    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    import torch

    torch.cuda.synchronize()
    return t.cpu().numpy()


def relerr(x, ref):
    x = np.asarray(x, dtype=np.float64).ravel()
    ref = np.asarray(ref, dtype=np.float64).ravel()
    return float(np.linalg.norm(x - ref) / np.linalg.norm(ref))


def note(msg):
    sys.stderr.write(f"[large-paths] {msg}\n")
    sys.stderr.flush()


_cache = {}


def problem(n, dtype):
    """One SPD matrix of the C5 recipe at size n (A = X X^T / 2n + I), its oracle factor, Lbar and 512 right-hand sides."""
    key = (n, dtype)
    if key not in _cache:
        _cache.clear()  # one problem at a time: these are big
        w = workloads.make("C5", n=n, m=512, dtype=dtype)
        t = time.time()
        w["L_oracle"] = __import__("oracle").potrf(w["A"])
        note(f"oracle potrf n={n} {dtype}: {time.time() - t:.1f} s")
        _cache[key] = w
    return _cache[key]


@pytest.mark.parametrize("dtype", ["f64", "f32"])
def test_potrf_panel_path_n4096_full_compare(la, orc, dtype):
    w = problem(4096, dtype)
    L = host(la.potrf(dev(w["A"])))
    assert np.all(np.triu(L[0], 1) == 0)
    assert relerr(L, w["L_oracle"]) <= TOL[dtype]
    # the upper factor of the same matrix is the transposed view of the same path
    R = host(la.potrf(dev(w["A"]), lower=False))
    assert np.all(np.tril(R[0], -1) == 0)
    assert relerr(R[0], w["L_oracle"][0].T) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f64", "f32"])
def test_trsm_block_substitution_n4096_full_compare(la, orc, dtype):
    w = problem(4096, dtype)
    Lr = w["L_oracle"].astype(workloads.np_dtype(dtype))  # the factor as the GPU operator would receive it
    R = w["rhs"]
    for kw in (dict(), dict(trans=True)):
        X = host(la.trsm(dev(Lr), dev(R), **kw))
        assert relerr(X, orc.trsm(Lr, R, **kw)) <= TOL[dtype], kw


@pytest.mark.parametrize("dtype", ["f64", "f32"])
def test_backward_closed_expression_n2048_full_compare(la, orc, dtype):
    w = problem(2048, dtype)
    Lr = w["L_oracle"].astype(workloads.np_dtype(dtype))
    t = time.time()
    ref = orc.potrf_backward(Lr, w["Lbar"])
    note(f"oracle backward n=2048 {dtype}: {time.time() - t:.1f} s")
    Abar = host(la.potrf_backward(dev(Lr), dev(w["Lbar"])))
    assert np.array_equal(Abar[0], Abar[0].T)
    assert relerr(Abar, ref) <= TOL[dtype]
    # in place (Abar over Lbar) takes the same path with one more copy
    G = dev(w["Lbar"])
    la.potrf_backward(dev(Lr), G, out=G)
    assert relerr(host(G), ref) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f64", "f32"])
def test_backward_sweep_n4096_full_compare(la, orc, dtype):
    w = problem(4096, dtype)
    Lr = w["L_oracle"].astype(workloads.np_dtype(dtype))
    t = time.time()
    ref = orc.potrf_backward(Lr, w["Lbar"])
    note(f"oracle backward n=4096 {dtype}: {time.time() - t:.1f} s")
    Abar = host(la.potrf_backward(dev(Lr), dev(w["Lbar"])))
    assert np.array_equal(Abar[0], Abar[0].T)
    assert relerr(Abar, ref) <= TOL[dtype]


def test_potrf_and_backward_sweep_ragged_n5376_full_compare(la, orc):
    """n = 5376 = 2048 + 2048 + 1280: three potrf panels with a ragged last one; the sweep peels a first
    block of 2048 columns and halves the remaining 3328 into base blocks of 1664."""
    dtype = "f64"
    w = problem(5376, dtype)
    L = host(la.potrf(dev(w["A"])))
    assert relerr(L, w["L_oracle"]) <= TOL[dtype]
    t = time.time()
    ref = orc.potrf_backward(w["L_oracle"], w["Lbar"])
    note(f"oracle backward n=5376 {dtype}: {time.time() - t:.1f} s")
    Abar = host(la.potrf_backward(dev(w["L_oracle"]), dev(w["Lbar"])))
    assert np.array_equal(Abar[0], Abar[0].T)
    assert relerr(Abar, ref) <= TOL[dtype]
