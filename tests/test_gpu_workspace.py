"""The workspace contract of the blocked paths on the GPU: a call runs entirely on the workspace it is
given (two calls on two streams with two workspaces may overlap), a workspace that is too small is
refused before anything is launched, and the bytes la_workspace_bytes names are enough for every flag."""
import ctypes
import sys

import numpy as np
import pytest

import workloads

pytestmark = pytest.mark.gpu


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


def _spd(rng, batch, n):
    X = rng.standard_normal((batch, n, 2 * n))
    return X @ X.transpose(0, 2, 1) / (2 * n) + np.eye(n)


def test_two_streams_two_workspaces_overlap_safely(la, orc):
    import torch

    from paper_1710_08717_amd import binding

    rng = np.random.default_rng(11)
    n, batch = 640, 3
    A1, A2 = _spd(rng, batch, n), _spd(rng, batch, n)
    G1, G2 = np.tril(rng.standard_normal((batch, n, n))), np.tril(rng.standard_normal((batch, n, n)))
    d = lambda a: torch.from_numpy(a).cuda()
    dA1, dA2, dG1, dG2 = d(A1), d(A2), d(G1), d(G2)
    need = max(la.workspace_bytes(binding.OP_POTRF, dA1, batch, n), la.workspace_bytes(binding.OP_POTRF_BACKWARD, dA1, batch, n))
    assert need > 0
    ws1 = torch.empty(need, dtype=torch.uint8, device="cuda")
    ws2 = torch.empty(need, dtype=torch.uint8, device="cuda")
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    for rep in range(3):  # interleaved enqueues: the two chains run side by side on the device
        with torch.cuda.stream(s1):
            L1 = la.potrf(dA1, workspace=ws1)
        with torch.cuda.stream(s2):
            L2 = la.potrf(dA2, workspace=ws2)
        with torch.cuda.stream(s1):
            B1 = la.potrf_backward(L1, dG1, workspace=ws1)
        with torch.cuda.stream(s2):
            B2 = la.potrf_backward(L2, dG2, workspace=ws2)
    torch.cuda.synchronize()
    for (L, B, A, G) in ((L1, B1, A1, G1), (L2, B2, A2, G2)):
        Lr = orc.potrf(A)
        Br = orc.potrf_backward(Lr, G)
        for x, r in ((L, Lr), (B, Br)):
            x = x.cpu().numpy().reshape(batch, -1)
            r = r.reshape(batch, -1)
            assert np.max(np.linalg.norm(x - r, axis=1) / np.linalg.norm(r, axis=1)) <= 1e-10


def test_too_small_workspace_launches_nothing(la):
    import torch

    from paper_1710_08717_amd import binding

    lib = binding.load()
    vp = ctypes.c_void_p
    n, batch = 512, 2
    A = torch.from_numpy(_spd(np.random.default_rng(3), batch, n)).cuda()
    L = torch.full_like(A, 7.0)
    need = la.workspace_bytes(binding.OP_POTRF, A, batch, n)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    st = vp(torch.cuda.current_stream().cuda_stream)
    assert lib.la_potrf_batched_ws(1, 1, batch, n, vp(A.data_ptr()), vp(L.data_ptr()), vp(0), vp(ws.data_ptr()), need - 256, st) == 4
    assert lib.la_potrf_batched(1, 1, batch, n, vp(A.data_ptr()), vp(L.data_ptr()), vp(0), st) == 4
    torch.cuda.synchronize()
    assert (L == 7.0).all()
    with pytest.raises(la.LaError):
        la.potrf(A, workspace=ws[: need - 256])
    assert lib.la_potrf_batched_ws(1, 1, batch, n, vp(A.data_ptr()), vp(L.data_ptr()), vp(0), vp(ws.data_ptr()), need, st) == 0
    torch.cuda.synchronize()
    Lh = L.cpu().numpy()
    assert np.allclose(Lh @ Lh.transpose(0, 2, 1), A.cpu().numpy(), rtol=0, atol=1e-12)


@pytest.mark.parametrize("dtype", ["f64", "f32"])
def test_exact_workspace_suffices_for_every_flag_with_a_guard_band(la, orc, dtype):
    """Each operator on exactly la_workspace_bytes bytes, with a canary after the workspace that must survive."""
    import torch

    from paper_1710_08717_amd import binding

    rng = np.random.default_rng(5)
    npd = workloads.np_dtype(dtype)
    tol = {"f32": 2e-4, "f64": 1e-10}[dtype]
    n, m, batch = 384, 80, 2
    A = _spd(rng, batch, n).astype(npd)
    Lr = orc.potrf(A.astype(np.float64))
    R = rng.standard_normal((batch, n, m)).astype(npd)
    dL = torch.from_numpy(np.ascontiguousarray(Lr.astype(npd))).cuda()
    dLt = torch.from_numpy(np.ascontiguousarray(Lr.transpose(0, 2, 1).astype(npd))).cuda()

    def guarded(op, *sizes):
        need = la.workspace_bytes(op, dL, batch, *sizes)
        buf = torch.zeros(need + 4096, dtype=torch.uint8, device="cuda")
        buf[need:] = 0xA5
        return buf, need

    def rel(x, r):
        x = x.cpu().numpy().astype(np.float64).reshape(batch, -1)
        r = r.reshape(batch, -1)
        return np.max(np.linalg.norm(x - r, axis=1) / np.linalg.norm(r, axis=1))

    for lower in (True, False):
        F = dL if lower else dLt
        Fh = Lr if lower else Lr.transpose(0, 2, 1)
        for trans in (False, True):
            for right in (False, True):
                Rh = R.transpose(0, 2, 1).copy() if right else R
                dR = torch.from_numpy(np.ascontiguousarray(Rh)).cuda()
                for name, op, fn, ofn in (("trsm", binding.OP_TRSM, la.trsm, orc.trsm), ("trmm", binding.OP_TRMM, la.trmm, orc.trmm)):
                    buf, need = guarded(op, n, m)
                    X = fn(F, dR, lower=lower, trans=trans, rightside=right, alpha=0.5, workspace=buf[:need])
                    ref = ofn(np.ascontiguousarray(Fh), Rh.astype(np.float64), lower=lower, trans=trans, rightside=right, alpha=0.5)
                    assert rel(X, ref) <= tol, (name, lower, trans, right)
                    assert (buf[need:] == 0xA5).all(), (name, lower, trans, right)
        buf, need = guarded(binding.OP_POTRF, n)
        dA = torch.from_numpy(A).cuda()
        Lg = la.potrf(dA, lower=lower, workspace=buf[:need])
        assert rel(Lg, Fh) <= tol
        assert (buf[need:] == 0xA5).all()
        G = np.tril(rng.standard_normal((batch, n, n))).astype(npd)
        Gh = G if lower else G.transpose(0, 2, 1).copy()
        buf, need = guarded(binding.OP_POTRF_BACKWARD, n)
        Bg = la.potrf_backward(F, torch.from_numpy(np.ascontiguousarray(Gh)).cuda(), lower=lower, workspace=buf[:need])
        ref = orc.potrf_backward(np.ascontiguousarray(Fh), Gh.astype(np.float64), lower=lower)
        assert rel(Bg, ref) <= tol
        assert (buf[need:] == 0xA5).all()


@pytest.mark.parametrize("batch,n,m,dtype", [(16, 32, 8, "f64"), (3, 300, 40, "f64"), (2, 700, 24, "f32")])
def test_calls_with_a_workspace_can_be_captured_in_a_graph(la, batch, n, m, dtype):
    """With a workspace an entry point allocates nothing and only enqueues kernels on the caller's stream, so a chain
    of calls can be recorded into a HIP graph.  Every replay -- with eager work of the same library and
    synchronisations between the replays -- must reproduce the eager results bit for bit."""
    import torch

    from paper_1710_08717_amd import binding

    dt = torch.float64 if dtype == "f64" else torch.float32
    gen = torch.Generator(device="cuda").manual_seed(5 + n)
    X = torch.randn(batch, n, n, dtype=dt, device="cuda", generator=gen)
    A = (X @ X.transpose(1, 2) / n + torch.eye(n, dtype=dt, device="cuda")).contiguous()
    rhs = torch.randn(batch, n, m, dtype=dt, device="cuda", generator=gen)
    G = torch.tril(torch.randn(batch, n, n, dtype=dt, device="cuda", generator=gen))
    L, Xo, Y, Ab = torch.empty_like(A), torch.empty_like(rhs), torch.empty_like(rhs), torch.empty_like(A)
    info = torch.zeros(batch, dtype=torch.int32, device="cuda")
    need = max(la.workspace_bytes(o, A, batch, n, m) for o in (binding.OP_POTRF, binding.OP_POTRF_BACKWARD, binding.OP_TRSM,
                                                               binding.OP_TRMM))
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")

    def chain():
        la.potrf(A, out=L, info=info, workspace=ws)
        la.trsm(L, rhs, out=Xo, workspace=ws)
        la.trmm(L, Xo, out=Y, trans=True, workspace=ws)
        la.potrf_backward(L, G, out=Ab, workspace=ws)

    chain()  # eager: also sets the kernels' attributes once, outside the capture
    torch.cuda.synchronize()
    ref = [t.clone() for t in (L, Xo, Y, Ab)]
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(s):
        with torch.cuda.graph(g, stream=s):
            chain()
    torch.cuda.synchronize()
    for rep in range(3):
        for t in (L, Xo, Y, Ab):
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for got, want in zip((L, Xo, Y, Ab), ref):
            assert torch.equal(got, want), rep
        assert int(info.abs().sum()) == 0
        # eager work of the library between the replays (other sizes, its own scratch use)
        other = la.potrf(A[:, : n // 2, : n // 2].contiguous())
        torch.cuda.synchronize()
        assert torch.isfinite(other).all()
