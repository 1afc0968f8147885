"""Parity of la_trsm_backward, la_trmm_backward and la_syrk_backward (through the C ABI / ctypes
binding) against the CPU oracle on the same seeded inputs: every (lower, trans, rightside) case,
both element types, sizes on both sides of every dispatch threshold, the aliasing the paper
allows, junk in the triangle that must not be read.  Tolerances as for the other operators:
relative Frobenius error per matrix <= 1e-10 (fp64), <= 2e-4 (fp32); structural zeros exact.
"""
import itertools
import sys

import numpy as np
import pytest

import workloads

pytestmark = pytest.mark.gpu

TOL = {"f32": 2e-4, "f64": 1e-10}
FLAGS = list(itertools.product([True, False], [False, True], [False, True]))  # lower, trans, rightside
SHAPES = [(1, 1), (5, 3), (16, 16), (48, 64), (64, 20), (100, 130), (128, 48), (200, 33), (260, 96)]


@pytest.fixture(scope="module")
def la():
    import torch

    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1710_08717_amd as la_mod

    la_mod.load()  # raises if the HIP library is missing: there is no fallback
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


def npdt(dtype):
    return workloads.np_dtype(dtype)


def relerr(x, ref):
    x = np.asarray(x, dtype=np.float64).reshape(x.shape[0], -1)
    ref = np.asarray(ref, dtype=np.float64).reshape(ref.shape[0], -1)
    num = np.linalg.norm(x - ref, axis=1)
    den = np.maximum(np.linalg.norm(ref, axis=1), 1e-300)
    return float(np.max(num / den)) if len(num) else 0.0


def tri(seed, batch, n, lower, dtype):
    rng = np.random.default_rng(seed)
    T = rng.standard_normal((batch, n, n)) * (0.5 / np.sqrt(max(n, 1)))
    T = np.tril(T) if lower else np.triu(T)
    idx = np.arange(n)
    T[:, idx, idx] = 1.0 + rng.uniform(0.0, 1.0, size=(batch, n))
    return T.astype(npdt(dtype))


def case(seed, n, m, lower, rightside, dtype, batch=3):
    T = tri(seed, batch, n, lower, dtype)
    rng = np.random.default_rng(seed + 1)
    shape = (batch, m, n) if rightside else (batch, n, m)
    X = rng.standard_normal(shape).astype(npdt(dtype))
    G = rng.standard_normal(shape).astype(npdt(dtype))
    other = np.triu_indices(n, 1) if lower else np.tril_indices(n, -1)
    Tj = T.copy()
    Tj[:, other[0], other[1]] = np.nan  # never read
    return T, Tj, X, G, other


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("lower,trans,rightside", FLAGS)
@pytest.mark.parametrize("n,m", SHAPES)
def test_trmm_backward_parity(la, orc, dtype, lower, trans, rightside, n, m):
    T, Tj, A, G, other = case(1000 + n + m, n, m, lower, rightside, dtype)
    alpha = -1.5 if (n + m) % 2 else 1.0
    ra, rl = orc.trmm_backward(T, A, G, lower=lower, trans=trans, rightside=rightside, alpha=alpha)
    ga, gl = la.trmm_backward(dev(Tj), dev(A), dev(G), lower=lower, trans=trans, rightside=rightside, alpha=alpha)
    ga, gl = host(ga), host(gl)
    assert relerr(ga, ra) <= TOL[dtype]
    assert relerr(gl, rl) <= TOL[dtype]
    assert np.all(gl[:, other[0], other[1]] == 0.0)
    g = dev(G)  # Abar over Bbar
    ga2, gl2 = la.trmm_backward(dev(Tj), dev(A), g, lower=lower, trans=trans, rightside=rightside, alpha=alpha, out_a=g)
    assert np.array_equal(host(ga2), ga) and np.array_equal(host(gl2), gl)


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("lower,trans,rightside", FLAGS)
@pytest.mark.parametrize("n,m", SHAPES)
def test_trsm_backward_parity(la, orc, dtype, lower, trans, rightside, n, m):
    T, Tj, A, G, other = case(2000 + n + m, n, m, lower, rightside, dtype)
    alpha = 0.5 if (n + m) % 2 else 1.0
    B = orc.trsm(T, A, lower=lower, trans=trans, rightside=rightside, alpha=alpha).astype(npdt(dtype))
    ra, rl = orc.trsm_backward(T, B, G, lower=lower, trans=trans, rightside=rightside, alpha=alpha)
    ga, gl = la.trsm_backward(dev(Tj), dev(B), dev(G), lower=lower, trans=trans, rightside=rightside, alpha=alpha)
    ga, gl = host(ga), host(gl)
    assert relerr(ga, ra) <= TOL[dtype]
    assert relerr(gl, rl) <= TOL[dtype]
    assert np.all(gl[:, other[0], other[1]] == 0.0)
    g, t = dev(G), dev(T)  # Abar over Bbar, Lbar over L (L holds zeros, not junk, in its other triangle here)
    ga2, gl2 = la.trsm_backward(t, dev(B), g, lower=lower, trans=trans, rightside=rightside, alpha=alpha, out_a=g,
                                out_l=t)
    assert np.array_equal(host(ga2), ga) and np.array_equal(host(gl2), gl)


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("lower,trans,rightside", FLAGS)
@pytest.mark.parametrize("op", ["trsm", "trmm"])
@pytest.mark.parametrize("n,m,batch", [(16, 16, 1031), (16, 32, 70), (13, 7, 515), (8, 8, 4101), (5, 20, 66), (4, 4, 4111),
                                       (3, 1, 1037), (1, 1, 5), (16, 33, 9),
                                       (32, 16, 1027), (32, 32, 9), (24, 16, 515), (19, 5, 130), (27, 32, 7),
                                       (40, 16, 70), (48, 32, 1030), (64, 20, 66), (100, 9, 64), (33, 40, 65), (128, 16, 64)])
def test_small_backward_rules_with_many_matrices(la, orc, dtype, lower, trans, rightside, op, n, m, batch):
    """n <= 16: the solve / multiply and the triangular operand's gradient (outer product over up to 32 vectors, masked)
    run in lane groups of 16, 8 or 4 per matrix; 16 < n <= 32: the outer product in 16 lanes with two rows per lane
    (two fp64 images of 32 x 32 do not fit one workgroup's LDS and take the tiled path, as does m = 33); ragged last
    wavefronts.  From 64 matrices of 32 < n <= 128 on, the outer product of operands of at most eight tiles is one
    workgroup per matrix (with four wavefronts above 1024 matrices)."""
    T, Tj, A, G, other = case(4000 + n + m, n, m, lower, rightside, dtype, batch=batch)
    alpha = 0.5
    if op == "trsm":
        X = orc.trsm(T, A, lower=lower, trans=trans, rightside=rightside, alpha=alpha).astype(npdt(dtype))
        ra, rl = orc.trsm_backward(T, X, G, lower=lower, trans=trans, rightside=rightside, alpha=alpha)
        ga, gl = la.trsm_backward(dev(Tj), dev(X), dev(G), lower=lower, trans=trans, rightside=rightside, alpha=alpha)
    else:
        ra, rl = orc.trmm_backward(T, A, G, lower=lower, trans=trans, rightside=rightside, alpha=alpha)
        ga, gl = la.trmm_backward(dev(Tj), dev(A), dev(G), lower=lower, trans=trans, rightside=rightside, alpha=alpha)
    ga, gl = host(ga), host(gl)
    assert relerr(ga, ra) <= TOL[dtype]
    assert relerr(gl, rl) <= TOL[dtype]
    assert np.all(gl[:, other[0], other[1]] == 0.0)


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("trans", [False, True])
@pytest.mark.parametrize("n,k,batch", [(16, 32, 1031), (16, 1, 70001), (13, 31, 515), (8, 16, 4101), (5, 20, 66), (4, 8, 4111),
                                       (3, 32, 1037), (1, 1, 5), (16, 33, 9),
                                       (32, 32, 1027), (29, 9, 4098), (24, 32, 515), (20, 1, 130), (17, 31, 5), (32, 33, 6)])
def test_small_syrk_backward_with_many_matrices(la, orc, dtype, trans, n, k, batch):
    """n <= 32 with an inner dimension up to 32: one lane-group launch, two rows per lane above n = 16 (k = 33 takes
    the tiled path)."""
    rng = np.random.default_rng(5000 + n + k)
    A = rng.standard_normal((batch, k, n) if trans else (batch, n, k)).astype(npdt(dtype))
    G = (rng.standard_normal((batch, n, n)) / np.sqrt(n)).astype(npdt(dtype))  # not symmetric
    ref = orc.syrk_backward(A, G, trans=trans, alpha=0.7)
    out = host(la.syrk_backward(dev(A), dev(G), trans=trans, alpha=0.7))
    assert out.shape == A.shape
    assert relerr(out, ref) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("trans", [False, True])
@pytest.mark.parametrize("n,k", [(1, 1), (6, 3), (16, 64), (70, 64), (100, 37), (256, 128), (300, 50)])
def test_syrk_backward_parity(la, orc, dtype, trans, n, k):
    batch = 3
    rng = np.random.default_rng(3000 + n + k)
    A = rng.standard_normal((batch, k, n) if trans else (batch, n, k)).astype(npdt(dtype))
    G = (rng.standard_normal((batch, n, n)) / np.sqrt(n)).astype(npdt(dtype))  # not symmetric
    alpha = 0.7
    ref = orc.syrk_backward(A, G, trans=trans, alpha=alpha)
    out = host(la.syrk_backward(dev(A), dev(G), trans=trans, alpha=alpha))
    assert relerr(out, ref) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("trans", [False, True])
@pytest.mark.parametrize("n,k,batch", [(33, 8, 70), (48, 32, 1030), (40, 50, 64), (64, 64, 65), (100, 17, 64), (57, 1, 1100),
                                       (128, 16, 64)])
def test_syrk_backward_one_workgroup_per_matrix(la, orc, dtype, trans, n, k, batch):
    """From 64 matrices of 32 < n <= 128 on, the rule keeps Bbar and A in LDS, one workgroup per matrix (where both fit
    64 KB; four wavefronts above 1024 matrices of at most 16 output tiles)."""
    rng = np.random.default_rng(n * k + batch + 1)
    A = rng.standard_normal((batch, k, n) if trans else (batch, n, k)).astype(npdt(dtype))
    G = (rng.standard_normal((batch, n, n)) / np.sqrt(n)).astype(npdt(dtype))  # not symmetric
    ref = orc.syrk_backward(A, G, trans=trans, alpha=-0.6)
    out = host(la.syrk_backward(dev(A), dev(G), trans=trans, alpha=-0.6))
    assert relerr(out, ref) <= TOL[dtype]


def test_backward_ops_gp_chain(la, orc):
    """The chain the GP criterion of section 3.1 differentiates through: z = L^-1 y, then the trsm
    rule gives ybar and Lbar; checked against the oracle with one right-hand side per matrix."""
    batch, n = 8, 128
    inp = workloads.make("C3", batch=batch)
    L = orc.potrf(inp["A"]).astype(np.float32)
    y = inp["y"].reshape(batch, n, 1).astype(np.float32)
    z = orc.trsm(L, y).astype(np.float32)
    zbar = z.copy()  # gradient of 1/2 z^T z
    ra, rl = orc.trsm_backward(L, z, zbar)
    ga, gl = la.trsm_backward(dev(L), dev(z), dev(zbar))
    assert relerr(host(ga), ra) <= TOL["f32"] and relerr(host(gl), rl) <= TOL["f32"]


def test_backward_ops_empty_and_errors(la):
    import torch

    for dt in (torch.float32, torch.float64):
        L = torch.eye(4, dtype=dt, device="cuda").repeat(2, 1, 1)
        e = torch.zeros((2, 4, 0), dtype=dt, device="cuda")
        ab, lb = la.trsm_backward(L, e, e)
        assert ab.shape == (2, 4, 0) and torch.all(lb == 0)
        ab, lb = la.trmm_backward(L, e, e)
        assert torch.all(lb == 0)
        z = torch.zeros((0, 4, 4), dtype=dt, device="cuda")
        la.trsm_backward(z, torch.zeros((0, 4, 2), dtype=dt, device="cuda"), torch.zeros((0, 4, 2), dtype=dt, device="cuda"))
        la.syrk_backward(torch.zeros((2, 0, 3), dtype=dt, device="cuda"), torch.zeros((2, 0, 0), dtype=dt, device="cuda"))
    L = torch.eye(4, dtype=torch.float64, device="cuda").repeat(2, 1, 1)
    X = torch.ones((2, 4, 3), dtype=torch.float64, device="cuda")
    G = torch.ones((2, 4, 3), dtype=torch.float64, device="cuda")
    with pytest.raises(la.LaError):
        la.trmm_backward(L, X, G, out_l=L)  # Lbar over L is allowed for trsm only
    with pytest.raises(la.LaError):
        la.trsm_backward(L, X, G, out_a=X)  # Abar over B
    with pytest.raises(la.LaError):
        la.syrk_backward(X, torch.ones((2, 4, 4), dtype=torch.float64, device="cuda"), out=X)


# ----------------------------------------------------------------------------
# gemm2 backward, potri forward / backward
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("ta", [False, True])
@pytest.mark.parametrize("tb", [False, True])
@pytest.mark.parametrize("m,n,k", [(1, 1, 1), (3, 5, 4), (64, 64, 64), (70, 33, 130), (256, 128, 192)])
def test_gemm2_backward_parity(la, orc, dtype, ta, tb, m, n, k):
    batch = 3
    rng = np.random.default_rng(4000 + m + n + k)
    A = (rng.standard_normal((batch, k, m) if ta else (batch, m, k)) / np.sqrt(k)).astype(npdt(dtype))
    B = rng.standard_normal((batch, n, k) if tb else (batch, k, n)).astype(npdt(dtype))
    G = rng.standard_normal((batch, m, n)).astype(npdt(dtype))
    ra, rb = orc.gemm2_backward(A, B, G, ta=ta, tb=tb, alpha=0.9)
    ga, gb = la.gemm2_backward(dev(A), dev(B), dev(G), ta=ta, tb=tb, alpha=0.9)
    assert relerr(host(ga), ra) <= TOL[dtype]
    assert relerr(host(gb), rb) <= TOL[dtype]


def spd(seed, batch, n, dtype):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((batch, n, 2 * n))
    A = X @ X.transpose(0, 2, 1) / (2 * n) + np.eye(n)
    return (0.5 * (A + A.transpose(0, 2, 1))).astype(npdt(dtype))


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("lower", [True, False])
@pytest.mark.parametrize("n", [1, 5, 16, 17, 24, 25, 32, 33, 64, 100, 128, 200, 384])
def test_potri_parity(la, orc, dtype, lower, n):
    batch = 3
    A = spd(5000 + n, batch, n, dtype)
    F = orc.potrf(A, lower=lower).astype(npdt(dtype))
    other = np.triu_indices(n, 1) if lower else np.tril_indices(n, -1)
    Fj = F.copy()
    Fj[:, other[0], other[1]] = np.nan  # never read
    ref = orc.potri(F, lower=lower)
    out = host(la.potri(dev(Fj), lower=lower))
    assert np.array_equal(out, out.transpose(0, 2, 1))  # exactly symmetric
    assert relerr(out, ref) <= TOL[dtype]
    t = dev(F)  # B over L
    out2 = host(la.potri(t, lower=lower, out=t))
    assert np.array_equal(out2, out)


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("lower", [True, False])
@pytest.mark.parametrize("n,batch", [(16, 4099), (13, 1030), (8, 4101), (6, 259), (4, 4111), (3, 70001), (2, 19), (1, 70),
                                     (32, 1027), (29, 4098), (24, 515), (20, 130), (17, 5), (40, 1030), (48, 1100), (64, 1025),
                                     (57, 40)])
def test_potri_small_sizes_with_many_matrices(la, orc, dtype, lower, n, batch):
    """n <= 16: 16, 8 or 4 lanes per matrix; 16 < n <= 32: 16 lanes per matrix with two rows per lane and 24 or 32
    columns kept.  Both solves in registers; ragged last wavefronts.  33 <= n <= 128: one workgroup per matrix,
    with four wavefronts instead of sixteen for many matrices of at most four tile rows."""
    A = spd(7000 + n, batch, n, dtype)
    F = orc.potrf(A, lower=lower).astype(npdt(dtype))
    ref = orc.potri(F, lower=lower)
    t = dev(F)
    out = host(la.potri(t, lower=lower, out=t))  # B over L
    assert np.array_equal(out, out.transpose(0, 2, 1))
    assert relerr(out, ref) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("lower", [True, False])
@pytest.mark.parametrize("n", [1, 5, 16, 33, 64, 100, 128, 200])
def test_potri_backward_parity(la, orc, dtype, lower, n):
    batch = 3
    A = spd(6000 + n, batch, n, dtype)
    F = orc.potrf(A, lower=lower).astype(npdt(dtype))
    B = orc.potri(F, lower=lower).astype(npdt(dtype))
    rng = np.random.default_rng(n)
    G = rng.standard_normal((batch, n, n)).astype(npdt(dtype))  # not symmetric
    ref = orc.potri_backward(F, B, G, lower=lower)
    other = np.triu_indices(n, 1) if lower else np.tril_indices(n, -1)
    Fj = F.copy()
    Fj[:, other[0], other[1]] = np.nan
    out = host(la.potri_backward(dev(Fj), dev(B), dev(G), lower=lower))
    assert np.all(out[:, other[0], other[1]] == 0.0)
    assert relerr(out, ref) <= TOL[dtype]


def test_rank2_ops_empty_and_errors(la):
    import torch

    z = torch.zeros((0, 3, 3), dtype=torch.float64, device="cuda")
    assert la.potri(z).shape == (0, 3, 3)
    assert la.potri_backward(z, z.clone(), z.clone()).shape == (0, 3, 3)
    A = torch.ones((2, 3, 0), dtype=torch.float64, device="cuda")
    B = torch.ones((2, 0, 4), dtype=torch.float64, device="cuda")
    ga, gb = la.gemm2_backward(A, B, torch.ones((2, 3, 4), dtype=torch.float64, device="cuda"))
    assert ga.shape == (2, 3, 0) and gb.shape == (2, 0, 4)
    A = torch.ones((2, 3, 5), dtype=torch.float64, device="cuda")
    B = torch.ones((2, 5, 0), dtype=torch.float64, device="cuda")
    ga, gb = la.gemm2_backward(A, B, torch.ones((2, 3, 0), dtype=torch.float64, device="cuda"))
    assert torch.all(ga == 0) and gb.shape == (2, 5, 0)
    L = torch.eye(4, dtype=torch.float64, device="cuda").repeat(2, 1, 1)
    with pytest.raises(la.LaError):
        la.potri_backward(L, L.clone(), L.clone(), out=L)
