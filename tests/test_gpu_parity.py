"""Parity of the HIP library (through the C ABI / ctypes binding) against the CPU oracle.

Every test runs the same seeded inputs through both, element by element.
Tolerances (the benchmark spec): relative Frobenius error per matrix
<= 1e-10 in fp64 and <= 2e-4 in fp32 for matrices with condition number <= 1e3
(the fp32 result is compared with the fp64 oracle evaluated on the same fp32 inputs).
Integer outputs (info) and structural zeros are compared exactly.
"""
import itertools
import sys

import numpy as np
import pytest

import workloads

pytestmark = pytest.mark.gpu

TOL = {"f32": 2e-4, "f64": 1e-10}
FLAGS = list(itertools.product([True, False], [False, True], [False, True]))  # lower, trans, rightside


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
    """max over the batch of ||x - ref||_F / ||ref||_F."""
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if x.ndim < 3:
        x, ref = x[None], ref[None]
    x = x.reshape(x.shape[0], -1)
    ref = ref.reshape(ref.shape[0], -1)
    num = np.linalg.norm(x - ref, axis=1)
    den = np.maximum(np.linalg.norm(ref, axis=1), 1e-300)
    return float(np.max(num / den)) if len(num) else 0.0


def spd(seed, batch, n, dtype):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((batch, n, 2 * n))
    A = X @ X.transpose(0, 2, 1) / (2 * n) + np.eye(n)
    return (0.5 * (A + A.transpose(0, 2, 1))).astype(npdt(dtype))


def tri(seed, batch, n, lower, dtype):
    rng = np.random.default_rng(seed)
    T = rng.standard_normal((batch, n, n)) * (0.5 / np.sqrt(max(n, 1)))
    T = np.tril(T) if lower else np.triu(T)
    idx = np.arange(n)
    T[:, idx, idx] = 1.0 + rng.uniform(0.0, 1.0, size=(batch, n))
    return T.astype(npdt(dtype))


SIZES = [1, 2, 3, 4, 5, 7, 8, 9, 10, 12, 13, 15, 16, 17, 20, 24, 25, 31, 32, 33, 36, 40, 41, 48, 64, 65, 80, 97, 100, 112, 113, 127, 128, 129, 192, 200, 256, 321, 384]


# ----------------------------------------------------------------------------
# potrf forward
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("n", SIZES)
@pytest.mark.parametrize("lower", [True, False])
def test_potrf_parity(la, orc, dtype, n, lower):
    import torch

    batch = 7 if n <= 64 else 3
    A = spd(n * 3 + lower, batch, n, dtype)
    ref = orc.potrf(A, lower=lower)
    info = torch.full((batch,), -1, dtype=torch.int32, device="cuda")
    L = host(la.potrf(dev(A), lower=lower, info=info))
    assert L.dtype == A.dtype
    assert np.all(host(info) == 0)
    other = np.triu_indices(n, 1) if lower else np.tril_indices(n, -1)
    assert np.all(L[:, other[0], other[1]] == 0.0)  # exact zeros in the other triangle
    assert relerr(L, ref) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("n", [8, 16, 32, 50, 100, 128, 150])
@pytest.mark.parametrize("lower", [True, False])
def test_potrf_in_place_and_other_triangle_ignored(la, orc, dtype, n, lower):
    A = spd(n + 11, 5, n, dtype)
    ref = orc.potrf(A, lower=lower)
    junk = A.copy()
    other = np.triu_indices(n, 1) if lower else np.tril_indices(n, -1)
    junk[:, other[0], other[1]] = np.nan
    t = dev(junk)
    out = la.potrf(t, lower=lower, out=t)  # L overwrites A
    L = host(out)
    assert np.all(L[:, other[0], other[1]] == 0.0)
    assert relerr(L, ref) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("n,bad", [(1, 0), (3, 1), (4, 3), (6, 3), (8, 0), (8, 7), (16, 15), (32, 0), (32, 20), (24, 23), (48, 17), (48, 40), (40, 39),
                                   (64, 40), (100, 0), (100, 70), (128, 127), (200, 130), (12, 11), (10, 3), (9, 0), (20, 17),
                                   (36, 33)])
def test_potrf_info_first_bad_pivot(la, orc, dtype, n, bad):
    import torch

    A = spd(n, 3, n, dtype)
    A[1, bad, bad] = -1.0  # leading minor of order bad+1 is not positive definite
    _, ref_info = orc.potrf(A, return_info=True)
    info = torch.zeros(3, dtype=torch.int32, device="cuda")
    L = host(la.potrf(dev(A), info=info))
    assert list(host(info)) == list(ref_info) == [0, bad + 1, 0]
    ok = [0, 2]
    assert relerr(L[ok], orc.potrf(A[ok])) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("lower", [True, False])
@pytest.mark.parametrize("n,bad", [(33, 32), (40, 17), (48, 0), (57, 40), (64, 63)])
def test_potrf_many_matrices_of_up_to_four_tile_rows(la, orc, dtype, lower, n, bad):
    """Above 1024 matrices, 32 < n <= 64 is factored with four wavefronts per matrix and the tiles in LDS; one matrix
    of the batch is not positive definite; the unread triangle holds NaN; in place."""
    import torch

    batch = 1030
    A = spd(n + 1, batch, n, dtype)
    A[7, bad, bad] = -1.0
    ref, ref_info = orc.potrf(A, lower=lower, return_info=True)
    other = np.triu_indices(n, 1) if lower else np.tril_indices(n, -1)
    Aj = A.copy()
    Aj[:, other[0], other[1]] = np.nan
    info = torch.zeros(batch, dtype=torch.int32, device="cuda")
    a = dev(Aj)
    L = host(la.potrf(a, lower=lower, info=info, out=a))
    assert np.array_equal(host(info), ref_info) and ref_info[7] == bad + 1 and ref_info.sum() == bad + 1
    ok = np.arange(batch) != 7
    assert np.all(L[:, other[0], other[1]][ok] == 0.0)
    assert relerr(L[ok], ref[ok]) <= TOL[dtype]


def test_potrf_ragged_batch_and_large_batch(la, orc):
    # batches that do not fill the last wavefront, and more items than one grid dimension holds
    for n, batch, dtype in [(16, 5, "f32"), (16, 70001, "f32"), (9, 3, "f64"), (32, 3, "f64"), (20, 4097, "f32"),
                            (24, 4098, "f64"), (40, 4099, "f32"), (33, 1, "f32"), (48, 9, "f32"), (47, 2, "f64"),
                            (8, 70003, "f32"), (8, 13, "f64"), (7, 9, "f32"), (4, 70001, "f32"), (4, 33, "f64"), (3, 5, "f32"),
                            (2, 17, "f64"), (1, 70, "f32")]:
        A = spd(n + batch, batch, n, dtype)
        assert relerr(host(la.potrf(dev(A))), orc.potrf(A)) <= TOL[dtype]


def test_empty_inputs(la):
    import torch

    for shape in [(0, 4, 4), (3, 0, 0)]:
        A = torch.zeros(shape, dtype=torch.float64, device="cuda")
        assert la.potrf(A).shape == shape
        assert la.potrf_backward(A, A.clone()).shape == shape
        assert la.syrk(A).shape == shape
    L = torch.eye(4, dtype=torch.float32, device="cuda")[None]
    B = torch.zeros((1, 4, 0), dtype=torch.float32, device="cuda")
    assert la.trsm(L, B).shape == (1, 4, 0)
    assert la.trmm(L, B).shape == (1, 4, 0)
    assert la.sumlogdiag(torch.zeros((0, 3, 3), device="cuda")).shape == (0,)


def test_argument_errors(la):
    import torch

    A = torch.eye(4, dtype=torch.float64, device="cuda")[None].contiguous()
    flat = torch.zeros(64, dtype=torch.float64, device="cuda")
    a = flat[:16].view(1, 4, 4)
    b = flat[8:24].view(1, 4, 4)  # partial overlap
    with pytest.raises(la.LaError):
        la.potrf(a, out=b)
    with pytest.raises(la.LaError):
        la.potrf_backward(A, a, out=A)  # Abar must not overlap L
    with pytest.raises(la.LaError):
        la.syrk(A, out=A)
    with pytest.raises(la.LaError):
        la.potrf(A.to(torch.float16))
    with pytest.raises(la.LaError):
        la.potrf(A.cpu())


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("n", [96, 128, 256])
def test_potrf_and_backward_on_pointers_off_the_16_byte_grid(la, orc, dtype, n):
    """Operands that start one element into their allocation: the block kernels and the products have
    to leave their 16-byte paths."""
    import torch

    batch = 3
    A = spd(n + 11, batch, n, dtype)
    rng = np.random.default_rng(n)
    G = np.tril(rng.standard_normal((batch, n, n))).astype(npdt(dtype))

    def shifted(a):
        buf = torch.empty(a.size + 1, dtype=torch.from_numpy(a).dtype, device="cuda")
        v = buf[1:].view(a.shape)
        v.copy_(torch.from_numpy(a))
        assert v.data_ptr() % 16 != 0
        return v

    a, g = shifted(A), shifted(G)
    l = shifted(np.zeros_like(A))
    la.potrf(a, out=l)
    ref = orc.potrf(A)
    assert relerr(host(l), ref) <= TOL[dtype]
    Lf = ref.astype(npdt(dtype))
    out = shifted(np.zeros_like(A))
    la.potrf_backward(shifted(Lf), g, out=out)
    o = host(out)
    assert np.array_equal(o, o.transpose(0, 2, 1))
    assert relerr(o, orc.potrf_backward(Lf, G)) <= TOL[dtype]


# ----------------------------------------------------------------------------
# potrf backward
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("n", SIZES)
@pytest.mark.parametrize("lower", [True, False])
def test_backward_parity(la, orc, dtype, n, lower):
    batch = 6 if n <= 64 else 2
    A = spd(n * 5 + lower, batch, n, dtype)
    Lf = orc.potrf(A, lower=lower).astype(npdt(dtype))  # the factor both sides start from
    rng = np.random.default_rng(n)
    G = rng.standard_normal((batch, n, n))
    G = (np.tril(G) if lower else np.triu(G)).astype(npdt(dtype))
    ref = orc.potrf_backward(Lf, G, lower=lower)
    out = host(la.potrf_backward(dev(Lf), dev(G), lower=lower))
    assert np.array_equal(out, out.transpose(0, 2, 1))  # exactly symmetric
    assert relerr(out, ref) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("n", [3, 4, 6, 8, 17, 24, 32])
@pytest.mark.parametrize("lower", [True, False])
def test_backward_parity_large_batch_register_kernel(la, orc, dtype, n, lower):
    """Above 2048 matrices sizes 17..32 take the register kernel instead of the one-workgroup one; sizes
    up to 4 and up to 8 sit in 4 and 8 lanes per matrix (16 and 8 matrices per wavefront, last one ragged)."""
    batch = 2100
    A = spd(n * 7 + lower, batch, n, dtype)
    Lf = orc.potrf(A, lower=lower).astype(npdt(dtype))
    rng = np.random.default_rng(n + 5)
    G = rng.standard_normal((batch, n, n))
    G = (np.tril(G) if lower else np.triu(G)).astype(npdt(dtype))
    ref = orc.potrf_backward(Lf, G, lower=lower)
    out = host(la.potrf_backward(dev(Lf), dev(G), lower=lower))
    assert np.array_equal(out, out.transpose(0, 2, 1))
    assert relerr(out, ref) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("n", [33, 40, 48, 57, 64])
@pytest.mark.parametrize("lower", [True, False])
def test_backward_parity_many_matrices_of_up_to_four_tile_rows(la, orc, dtype, n, lower):
    """Above 1024 matrices the one-workgroup kernel runs with four wavefronts per matrix for n <= 64."""
    batch = 1030
    A = spd(n * 3 + lower, batch, n, dtype)
    Lf = orc.potrf(A, lower=lower).astype(npdt(dtype))
    rng = np.random.default_rng(n + 9)
    G = rng.standard_normal((batch, n, n))
    G = (np.tril(G) if lower else np.triu(G)).astype(npdt(dtype))
    ref = orc.potrf_backward(Lf, G, lower=lower)
    out = host(la.potrf_backward(dev(Lf), dev(G), lower=lower))
    assert np.array_equal(out, out.transpose(0, 2, 1))
    assert relerr(out, ref) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("n", [7, 16, 32, 40, 130, 256])
@pytest.mark.parametrize("lower", [True, False])
def test_backward_aliasing_and_junk_triangles(la, orc, dtype, n, lower):
    batch = 5
    A = spd(n + 77, batch, n, dtype)
    Lf = orc.potrf(A, lower=lower).astype(npdt(dtype))
    rng = np.random.default_rng(n + 1)
    G = rng.standard_normal((batch, n, n)).astype(npdt(dtype))  # full: the other triangle must be ignored
    ref = orc.potrf_backward(Lf, (np.tril(G) if lower else np.triu(G)), lower=lower)
    other = np.triu_indices(n, 1) if lower else np.tril_indices(n, -1)
    Lj = Lf.copy()
    Lj[:, other[0], other[1]] = np.nan
    Gj = G.copy()
    Gj[:, other[0], other[1]] = np.nan
    g = dev(Gj)
    out = host(la.potrf_backward(dev(Lj), g, lower=lower, out=g))  # Abar overwrites Lbar
    assert np.all(np.isfinite(out))
    assert relerr(out, ref) <= TOL[dtype]


def test_backward_closed_forms(la, orc):
    """Lbar = L gives Abar = I/2; Lbar = diag(1/l_ii) gives Abar = inv(A)/2 (both from phi's definition)."""
    for n, dtype in [(16, "f64"), (32, "f64"), (96, "f64"), (16, "f32")]:
        A = spd(n, 4, n, dtype)
        L = la.potrf(dev(A))
        half_eye = np.broadcast_to(0.5 * np.eye(n), A.shape)
        got = host(la.potrf_backward(L, L.clone()))
        assert np.max(np.abs(got - half_eye)) <= (1e-12 if dtype == "f64" else 1e-5)
        Lh = host(L)
        D = np.zeros_like(Lh)
        idx = np.arange(n)
        D[:, idx, idx] = 1.0 / Lh[:, idx, idx]
        got = host(la.potrf_backward(L, dev(D)))
        assert relerr(got, 0.5 * np.linalg.inv(A.astype(np.float64))) <= TOL[dtype]


# ----------------------------------------------------------------------------
# trsm / trmm
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("lower,trans,rightside", FLAGS)
@pytest.mark.parametrize("n,m", [(1, 1), (5, 3), (17, 17), (32, 8), (64, 64), (65, 7), (100, 33), (100, 130), (113, 20), (128, 1),
                                 (128, 48), (128, 49), (200, 33), (257, 70), (129, 1), (300, 5), (400, 16),
                                 (512, 64)])
def test_trsm_parity(la, orc, dtype, lower, trans, rightside, n, m):
    batch = 3
    T = tri(n + m, batch, n, lower, dtype)
    other = np.triu_indices(n, 1) if lower else np.tril_indices(n, -1)
    Tj = T.copy()
    Tj[:, other[0], other[1]] = np.nan  # never read
    rng = np.random.default_rng(n * m)
    A = rng.standard_normal((batch, m, n) if rightside else (batch, n, m)).astype(npdt(dtype))
    alpha = 0.5 if (n + m) % 2 else 1.0
    ref = orc.trsm(T, A, lower=lower, trans=trans, rightside=rightside, alpha=alpha)
    out = host(la.trsm(dev(Tj), dev(A), lower=lower, trans=trans, rightside=rightside, alpha=alpha))
    assert relerr(out, ref) <= TOL[dtype]
    a = dev(A)
    out2 = host(la.trsm(dev(Tj), a, lower=lower, trans=trans, rightside=rightside, alpha=alpha, out=a))  # in place
    assert np.array_equal(out, out2)


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("lower,trans,rightside", FLAGS)
@pytest.mark.parametrize("op", ["trsm", "trmm"])
@pytest.mark.parametrize("n,m,batch", [(16, 16, 4099), (16, 1, 70001), (13, 7, 1030), (8, 8, 4101), (7, 16, 259), (5, 3, 66),
                                       (4, 4, 4111), (3, 16, 1037), (2, 5, 19), (1, 1, 5), (32, 8, 1031), (24, 16, 130),
                                       (17, 2, 3), (64, 8, 1300), (40, 3, 2100), (33, 1, 1029), (64, 16, 5),
                                       (32, 16, 4098), (24, 16, 1030), (29, 5, 2051), (20, 1, 1500),
                                       (48, 32, 1030), (100, 9, 64), (128, 16, 64), (16, 40, 70), (96, 33, 65)])
def test_small_triangular_operators_with_many_matrices(la, orc, dtype, lower, trans, rightside, op, n, m, batch):
    """n <= 64 with at most 16 vectors: 4 .. 64 lanes per matrix (16 < n <= 32: 16 lanes with two rows per lane),
    operands moved as flat images; batches that
    leave the last wavefront ragged, more items than one grid dimension holds, in place and out of place.  (Solves
    with 16 < n <= 32 take this kernel above 1024 matrices only; solves with n > 32 the one-workgroup substitution
    kernel, with four wavefronts per item above 1024 items of n <= 64.)  Multiplies of 64 items or more with n > 32 or more than
    16 vectors, n and m up to 128: one workgroup per item with the factor's lower tiles and the vectors in LDS."""
    T = tri(n * 3 + m, batch, n, lower, dtype)
    other = np.triu_indices(n, 1) if lower else np.tril_indices(n, -1)
    Tj = T.copy()
    Tj[:, other[0], other[1]] = np.nan  # never read
    rng = np.random.default_rng(n * 100 + m)
    A = rng.standard_normal((batch, m, n) if rightside else (batch, n, m)).astype(npdt(dtype))
    f_o, f_g = (orc.trsm, la.trsm) if op == "trsm" else (orc.trmm, la.trmm)
    ref = f_o(T, A, lower=lower, trans=trans, rightside=rightside, alpha=0.75)
    out = host(f_g(dev(Tj), dev(A), lower=lower, trans=trans, rightside=rightside, alpha=0.75))
    assert relerr(out, ref) <= TOL[dtype]
    a = dev(A)
    out2 = host(f_g(dev(Tj), a, lower=lower, trans=trans, rightside=rightside, alpha=0.75, out=a))
    assert np.array_equal(out, out2)


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("lower,trans,rightside", FLAGS)
@pytest.mark.parametrize("n,m", [(1, 2), (6, 3), (64, 5), (70, 64), (150, 150), (260, 9)])
def test_trmm_parity(la, orc, dtype, lower, trans, rightside, n, m):
    batch = 3
    T = tri(n + 2 * m, batch, n, lower, dtype)
    other = np.triu_indices(n, 1) if lower else np.tril_indices(n, -1)
    Tj = T.copy()
    Tj[:, other[0], other[1]] = np.nan
    rng = np.random.default_rng(n * m + 1)
    A = rng.standard_normal((batch, m, n) if rightside else (batch, n, m)).astype(npdt(dtype))
    alpha = -2.0 if (n + m) % 2 else 1.0
    ref = orc.trmm(T, A, lower=lower, trans=trans, rightside=rightside, alpha=alpha)
    out = host(la.trmm(dev(Tj), dev(A), lower=lower, trans=trans, rightside=rightside, alpha=alpha))
    assert relerr(out, ref) <= TOL[dtype]
    a = dev(A)
    out2 = host(la.trmm(dev(Tj), a, lower=lower, trans=trans, rightside=rightside, alpha=alpha, out=a))
    assert np.array_equal(out, out2)


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("lower,trans,rightside", [(True, False, False), (True, True, False), (False, False, True),
                                                   (True, True, True)])
@pytest.mark.parametrize("n,m,batch", [(1300, 70, 1), (700, 5, 2), (300, 60, 3), (1100, 300, 1), (2100, 130, 1)])
def test_trsm_block_substitution_path(la, orc, dtype, lower, trans, rightside, n, m, batch):
    """Above the edge of the explicitly inverted diagonal blocks (256, 512 or 1024 rows, growing with
    the number of vectors) the solve is a block substitution; every size here leaves a ragged last block."""
    T = tri(n, batch, n, lower, dtype)
    rng = np.random.default_rng(n + m)
    A = rng.standard_normal((batch, m, n) if rightside else (batch, n, m)).astype(npdt(dtype))
    ref = orc.trsm(T, A, lower=lower, trans=trans, rightside=rightside, alpha=0.5)
    a = dev(A)
    out = host(la.trsm(dev(T), a, lower=lower, trans=trans, rightside=rightside, alpha=0.5, out=a))  # in place
    assert relerr(out, ref) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("lower,trans,rightside", FLAGS)
@pytest.mark.parametrize("n,m,batch", [(130, 17, 70), (260, 40, 300), (384, 16, 9), (500, 100, 5), (512, 530, 2)])
def test_trsm_streamed_factor_path(la, orc, dtype, lower, trans, rightside, n, m, batch):
    """128 < n <= 512: one launch, one workgroup per item and slab of 16 vectors.  Two, three and four tile rows
    per wavefront, ragged last tiles and slabs, more workgroups than the chip holds at once, both triangles
    (an upper factor is read through 8-byte loads, a lower one through 16-byte loads), forward and backward
    substitution, out of place (the other triangle holds NaN) and in place; each item judged on its own."""
    T = tri(n * 7 + m, batch, n, lower, dtype)
    other = np.triu_indices(n, 1) if lower else np.tril_indices(n, -1)
    Tj = T.copy()
    Tj[:, other[0], other[1]] = np.nan  # never read
    rng = np.random.default_rng(n * 1000 + m)
    A = rng.standard_normal((batch, m, n) if rightside else (batch, n, m)).astype(npdt(dtype))
    ref = orc.trsm(T, A, lower=lower, trans=trans, rightside=rightside, alpha=0.75)
    out = host(la.trsm(dev(Tj), dev(A), lower=lower, trans=trans, rightside=rightside, alpha=0.75))
    per = np.linalg.norm((out - ref).reshape(batch, -1), axis=1) / np.linalg.norm(ref.reshape(batch, -1), axis=1)
    assert per.max() <= TOL[dtype]
    a = dev(A)
    out2 = host(la.trsm(dev(Tj), a, lower=lower, trans=trans, rightside=rightside, alpha=0.75, out=a))  # in place
    assert np.array_equal(out, out2)


@pytest.mark.parametrize("dtype", ["f64", "f32"])
def test_potrf_backward_ragged_large(la, orc, dtype):
    """A size that is no multiple of 64 above every small-matrix shortcut."""
    n, batch = 1100, 1
    A = spd(n, batch, n, dtype)
    L = la.potrf(dev(A))
    Lh = host(L)
    assert relerr(Lh, orc.potrf(A)) <= TOL[dtype]
    G = np.tril(np.random.default_rng(n).standard_normal((batch, n, n))).astype(npdt(dtype))
    g = dev(G)
    out = host(la.potrf_backward(L, g, out=g))
    assert np.array_equal(out, out.transpose(0, 2, 1))
    assert relerr(out, orc.potrf_backward(Lh, G)) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("lower", [True, False])
@pytest.mark.parametrize("batch,n", [(40, 600), (3, 1300), (160, 300)])
def test_potrf_backward_blocked_sweep(la, orc, dtype, lower, batch, n):
    """Sizes above the largest block of the inverse-based expression for their batch (256 rows for
    40 and more matrices, 1024 for 3): the reverse sweep over the blocked factorisation, two levels
    deep for n = 600, with a trailing block small enough for the one-workgroup kernel for n = 300;
    once into a separate output, once over Lbar itself."""
    rng = np.random.default_rng(batch * n)
    F = np.tril(rng.standard_normal((batch, n, n))) / np.sqrt(n) + np.eye(n)
    G = np.tril(rng.standard_normal((batch, n, n)))
    if not lower:
        F, G = F.transpose(0, 2, 1), G.transpose(0, 2, 1)
    F, G = np.ascontiguousarray(F).astype(npdt(dtype)), np.ascontiguousarray(G).astype(npdt(dtype))
    ref = orc.potrf_backward(F, G, lower=lower)
    f, g = dev(F), dev(G)
    o = dev(np.full(G.shape, np.nan, dtype=npdt(dtype)))  # every entry of the output has to be written
    out = host(la.potrf_backward(f, g, lower=lower, out=o))
    assert np.array_equal(host(g), G)  # the input is left alone
    assert np.array_equal(out, out.transpose(0, 2, 1))
    assert relerr(out, ref) <= TOL[dtype]
    again = host(la.potrf_backward(f, g, lower=lower, out=g))
    assert np.array_equal(again, out)


# ----------------------------------------------------------------------------
# syrk / sumlogdiag / GP glue
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("n,k", [(2048, 64), (2880, 32), (4096, 48), (4096, 2064)])
def test_syrk_large_lower_triangle_tile_counts(la, orc, dtype, n, k):
    """Outputs whose lower-triangle tile count is a few tiles over whole rounds of workgroup slots
    (32 or 45 tile rows): the launcher issues the tiles below the diagonal and the diagonal blocks
    separately."""
    rng = np.random.default_rng(n + k)
    A = rng.standard_normal((1, n, k)).astype(npdt(dtype))
    ref = orc.syrk(A, alpha=0.25)
    out = host(la.syrk(dev(A), alpha=0.25))
    assert np.array_equal(out, out.transpose(0, 2, 1))
    assert relerr(out, ref) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("trans", [False, True])
@pytest.mark.parametrize("n,k,batch", [(33, 8, 70), (48, 32, 1030), (40, 50, 64), (64, 64, 65), (100, 17, 64), (128, 48, 64),
                                       (128, 128, 64), (57, 1, 1100)])
def test_syrk_one_workgroup_per_matrix(la, orc, dtype, trans, n, k, batch):
    """From 64 matrices of 32 < n <= 128 on, syrk keeps its operand in LDS, one workgroup per matrix (four wavefronts
    above 1024 matrices of at most four tile rows), and writes every tile with its mirror image; 128 x 128 operands
    in fp64 do not fit and take the tiled product."""
    import torch

    rng = np.random.default_rng(n * k + batch)
    A = rng.standard_normal((batch, k, n) if trans else (batch, n, k)).astype(npdt(dtype))
    ref = orc.syrk(A, trans=trans, alpha=-0.75)
    out = torch.full((batch, n, n), float("nan"), dtype=dev(A).dtype, device="cuda")
    la.syrk(dev(A), trans=trans, alpha=-0.75, out=out)
    o = host(out)
    assert np.array_equal(o, o.transpose(0, 2, 1))
    assert relerr(o, ref) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("trans", [False, True])
@pytest.mark.parametrize("n,k,batch", [(16, 32, 4099), (16, 1, 70001), (13, 31, 1030), (8, 16, 4101), (7, 5, 259), (4, 8, 4111),
                                       (3, 32, 1037), (2, 2, 19), (1, 7, 5), (16, 33, 7),
                                       (32, 32, 1027), (29, 9, 4098), (24, 32, 515), (20, 1, 130), (17, 31, 5), (32, 33, 6)])
def test_small_syrk_with_many_matrices(la, orc, dtype, trans, n, k, batch):
    """n <= 16 with an inner dimension up to 32 runs in 16, 8 or 4 lanes per matrix, 16 < n <= 32 in 16 lanes with
    two rows per lane (k = 33 does not)."""
    rng = np.random.default_rng(n * 50 + k)
    A = rng.standard_normal((batch, k, n) if trans else (batch, n, k)).astype(npdt(dtype))
    ref = orc.syrk(A, trans=trans, alpha=0.5)
    out = host(la.syrk(dev(A), trans=trans, alpha=0.5))
    assert np.array_equal(out, out.transpose(0, 2, 1))
    assert relerr(out, ref) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("trans", [False, True])
@pytest.mark.parametrize("n,k", [(1, 1), (4, 9), (16, 32), (32, 64), (65, 17), (130, 200), (64, 0), (50, 9568), (200, 2064),
                                 (64, 4096)])
def test_syrk_parity(la, orc, dtype, trans, n, k):
    batch = 3
    rng = np.random.default_rng(n + k)
    A = rng.standard_normal((batch, k, n) if trans else (batch, n, k)).astype(npdt(dtype))
    ref = orc.syrk(A, trans=trans, alpha=0.25)
    out = host(la.syrk(dev(A), trans=trans, alpha=0.25))
    assert np.array_equal(out, out.transpose(0, 2, 1))
    if k == 0:
        assert np.all(out == 0)
    else:
        assert relerr(out, ref) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("ta", [False, True])
@pytest.mark.parametrize("tb", [False, True])
@pytest.mark.parametrize("m,n,k", [(1, 1, 1), (5, 7, 3), (64, 64, 64), (130, 70, 96), (256, 384, 128), (200, 64, 0),
                                   (96, 64, 4112), (3, 200, 2048), (200, 5, 2500)])
def test_gemm2_parity(la, orc, dtype, ta, tb, m, n, k):
    batch = 3
    rng = np.random.default_rng(m + 3 * n + 7 * k)
    A = rng.standard_normal((batch, k, m) if ta else (batch, m, k)).astype(npdt(dtype))
    B = rng.standard_normal((batch, n, k) if tb else (batch, k, n)).astype(npdt(dtype))
    ref = orc.gemm2(A, B, ta=ta, tb=tb, alpha=1.5)
    out = host(la.gemm2(dev(A), dev(B), ta=ta, tb=tb, alpha=1.5))
    if k == 0:
        assert np.all(out == 0)
    else:
        assert relerr(out, ref) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("ta", [False, True])
@pytest.mark.parametrize("tb", [False, True])
@pytest.mark.parametrize("m,n,k,batch", [(16, 16, 16, 4099), (16, 1, 16, 70001), (3, 16, 9, 1030), (8, 8, 8, 4101),
                                         (2, 13, 7, 259), (4, 4, 4, 4111), (4, 16, 3, 1037), (9, 2, 4, 19), (1, 1, 1, 70),
                                         (16, 16, 17, 5), (16, 17, 16, 5), (17, 16, 16, 5),
                                         (32, 32, 32, 1027), (24, 16, 32, 4098), (3, 32, 9, 515), (32, 1, 17, 130),
                                         (20, 27, 5, 66), (1, 1, 32, 7), (33, 32, 32, 3), (32, 32, 33, 3)])
def test_small_gemm2_with_many_matrices(la, orc, dtype, ta, tb, m, n, k, batch):
    """m, n, k <= 16 run in lane groups of 4, 8 or 16 per item, up to 32 in 16 lanes with two rows per lane (the
    last two shapes do not)."""
    rng = np.random.default_rng(m + 3 * n + 7 * k)
    A = rng.standard_normal((batch, k, m) if ta else (batch, m, k)).astype(npdt(dtype))
    B = rng.standard_normal((batch, n, k) if tb else (batch, k, n)).astype(npdt(dtype))
    ref = orc.gemm2(A, B, ta=ta, tb=tb, alpha=-0.5)
    out = host(la.gemm2(dev(A), dev(B), ta=ta, tb=tb, alpha=-0.5))
    assert out.shape == (batch, m, n)
    assert relerr(out, ref) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("n", [1, 16, 32, 100, 1000])
def test_sumlogdiag_parity(la, orc, dtype, n):
    batch = 9
    T = tri(n, batch, n, True, dtype)
    ref = orc.sumlogdiag(T)
    out = host(la.sumlogdiag(dev(T))).astype(np.float64)
    assert np.max(np.abs(out - ref) / np.maximum(np.abs(ref), 1.0)) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("n,batch", [(1, 300), (2, 70001), (3, 1001), (4, 4099), (7, 513), (16, 70001), (17, 99), (32, 1027),
                                     (33, 70)])
def test_sumlogdiag_small_sizes_with_many_matrices(la, orc, dtype, n, batch):
    """Up to n = 32 several matrices share a wavefront (lane groups of 1 .. 32); 33 takes a wavefront each."""
    T = tri(n + batch, batch, n, True, dtype)
    ref = orc.sumlogdiag(T)
    out = host(la.sumlogdiag(dev(T))).astype(np.float64)
    assert out.shape == (batch,)
    assert np.max(np.abs(out - ref) / np.maximum(np.abs(ref), 1.0)) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("n", [3, 32, 128, 150])
def test_gp_glue_parity(la, orc, dtype, n):
    batch = 4
    T = tri(n + 5, batch, n, True, dtype)
    rng = np.random.default_rng(n)
    y, z, a = (rng.standard_normal((batch, n)).astype(npdt(dtype)) for _ in range(3))
    ref_loss, ref_G = orc.gp_glue(T, y, z, a)
    loss, G = la.gp_glue(dev(T), dev(y), dev(z), dev(a))
    loss, G = host(loss).astype(np.float64), host(G)
    assert np.all(np.triu(G, 1) == 0.0)
    assert relerr(G, ref_G) <= TOL[dtype]
    assert np.max(np.abs(loss - ref_loss) / np.maximum(np.abs(ref_loss), 1.0)) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f64", "f32"])
def test_blocked_paths_at_condition_1e3(la, orc, dtype):
    """The blocked paths lean on explicit inverses of (blocks of) the factor; the tolerances are
    stated for condition numbers up to 1e3, so here is a matrix with exactly that spectrum
    (eigenvalues spread evenly in the logarithm from 1 to 1000) at a size where potrf goes panel
    by panel with merged inverses, the backward pass sweeps the blocked factorisation and trsm
    substitutes block by block."""
    rng = np.random.default_rng(1003)
    batch, n = 3, 1400
    Q, _ = np.linalg.qr(rng.standard_normal((batch, n, n)))
    A = (Q * np.logspace(0, 3, n)[None, None, :]) @ Q.transpose(0, 2, 1)
    A = (0.5 * (A + A.transpose(0, 2, 1))).astype(npdt(dtype))
    assert 900 <= np.linalg.cond(A[0].astype(np.float64)) <= 1100
    G = np.tril(rng.standard_normal((batch, n, n))).astype(npdt(dtype))
    R = rng.standard_normal((batch, n, 70)).astype(npdt(dtype))
    L = la.potrf(dev(A))
    Lh = host(L)
    assert relerr(Lh, orc.potrf(A)) <= TOL[dtype]
    assert relerr(host(la.potrf_backward(L, dev(G))), orc.potrf_backward(Lh, G)) <= TOL[dtype]
    assert relerr(host(la.trsm(L, dev(R))), orc.trsm(Lh, R)) <= TOL[dtype]
