"""Parity of la_sgp_criterion (sparse-GP criterion of section 3.2 and its gradient, composed of the
library's operators) against the oracle's plain composition on the same seeded synthetic inputs.
Every output is held to the operators' own tolerance (relative Frobenius error 1e-10 in fp64, 2e-4 in fp32)."""
import sys

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


def rel(a, b):
    return float(np.linalg.norm(np.asarray(a, dtype=np.float64) - b) / max(np.linalg.norm(b), 1e-300))


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("U,n", [(1, 3), (7, 20), (50, 300), (64, 128), (100, 513), (200, 1000), (384, 2048),
                                 (1024, 2048)])
def test_sgp_parity(la, orc, dtype, U, n):
    import torch

    # U = 1024 takes the blocked potrf and the blocked backward pass inside the criterion; more jitter
    # on Kuu keeps its condition number within the tolerance's range there
    w = workloads.make_sgp(U, n, dtype=dtype, jitter=0.3 if U >= 1024 else 0.1)
    assert np.linalg.cond(w["Kuu"].astype(np.float64)) <= 1e3
    ref = orc.sgp_criterion(w["Kuu"], w["Kuf"], w["Kff_diag"], w["y"], w["noise_var"])
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    out = la.sgp_criterion(dev(w["Kuu"]), dev(w["Kuf"]), dev(w["Kff_diag"]), dev(w["y"]), w["noise_var"])
    torch.cuda.synchronize()
    got = {k: v.cpu().numpy() for k, v in out.items()}
    tol = TOL[dtype]
    assert abs(float(got["phi"][0]) - ref["phi"]) <= tol * max(1.0, abs(ref["phi"]))
    assert abs(float(got["noise_bar"][0]) - ref["noise_bar"]) <= tol * max(1.0, abs(ref["noise_bar"]))
    for key in ("Kuu_bar", "Kuf_bar", "Kff_diag_bar", "y_bar"):
        assert rel(got[key], ref[key]) <= tol, key
    assert np.array_equal(got["Kuu_bar"], got["Kuu_bar"].T)


def test_sgp_argument_errors(la):
    import torch

    w = workloads.make_sgp(8, 16)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    with pytest.raises(la.LaError):
        la.sgp_criterion(dev(w["Kuu"]), dev(w["Kuf"]), dev(w["Kff_diag"]), dev(w["y"]), -1.0)
    with pytest.raises(la.LaError):
        la.sgp_criterion(dev(w["Kuu"]), dev(w["Kuf"]), dev(w["Kff_diag"]), dev(w["y"]), 0.1,
                         workspace=torch.empty(64, dtype=torch.uint8, device="cuda"))
