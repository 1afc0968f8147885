#!/usr/bin/env python3
"""Throughput benchmark of the batched Cholesky hot path on one MI355X.

Default workload (the one the headline metric is quoted on): 65536 SPD matrices of
size 16 in fp32, potrf forward + potrf backward per step ("C2").  Other configurations
can be timed with --config C1|C3|C4|C5 (C5 also with --dtype f32).

One JSON line is printed on stdout; progress goes to stderr.

Timed region 1 (headline): W warm-up steps, then exactly K steps between
torch.cuda.synchronize() calls, wall clock.  Inputs are resident in HBM before it starts.
Steps rotate over several distinct buffer sets so that the 256 MB Infinity Cache cannot
serve repeats of the HBM-bound configurations.
Timed region 2 (roofline): the same K steps again with a HIP event pair around every
library call, on the stream the kernels run on, which gives the average duration of each
entry point's launch(es).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
PEAK_TFLOPS = {"f64": 78.6, "f32": 157.3}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def backward_flops(n, batch, elem_size):
    """Flops per matrix of the backward pass as the library runs it.  Up to a block size that
    depends on the batch it evaluates the closed expression, counted as 2 n^3 (lower triangle of
    L^T Lbar, L^-T applied to n columns, lower triangle of the product with L^-1).  Above it, it
    sweeps the blocked factorisation in reverse, which needs fewer flops: a level that splits n
    into n1 + n2 costs 2 n2^2 n1 (symmetric block times panel) + n1^2 n2 (panel solve) +
    n1^2 n2 (lower triangle of the panel product) = 2 n1 n2 n, and the blocks at the bottom cost
    2 n0^3 each.  The rule for the block size and the split mirror the library's."""
    budget = (16.0 if elem_size == 4 else 8.0) * 1048576.0
    base = 2048
    while base > 256 and float(base) * base * batch > budget:
        base //= 2

    def rec(k):
        if k <= base:
            return 2.0 * k ** 3
        q = k // 2048
        halves_fit = k % 2048 == 0 and q & (q - 1) == 0
        k1 = 2048 if (k > 4096 and not halves_fit) else (k // 2 + 127) // 128 * 128
        k2 = k - k1
        return 2.0 * k1 * k2 * k + rec(k1) + rec(k2)

    return rec(n)


def flops_model(name, n, m, batch=1, elem_size=8):
    """Useful flops per matrix: potrf n^3/3, backward see backward_flops, trsm/trmm n^2 m each."""
    f = {"potrf": n ** 3 / 3.0, "backward": backward_flops(n, batch, elem_size)}
    if name == "C1":
        f["trsm"] = float(n * n * m)
        f["sumlogdiag"] = float(n)
    elif name == "C3":
        f["trsm"] = 2.0 * n * n
        f["sumlogdiag"] = float(n)
    elif name == "C4":
        f["trsm"] = float(n * n * m)
        f["trmm"] = float(n * n * m)
    elif name == "C5":
        f["trsm"] = float(n * n * m)
    return f


def bytes_model(n, s):
    """Algorithmic HBM bytes per matrix: triangular inputs count n(n+1)/2, outputs are full squares."""
    tri = n * (n + 1) // 2
    return {"potrf": (tri + n * n) * s, "backward": (2 * tri + n * n) * s}


def bench_sgp(args, la, torch, np, workloads):
    """Second workload (section 3.2; the paper times it on n = 9568 cases with U inducing points):
    one step = the sparse-GP criterion and its full gradient, one call of la_sgp_criterion."""
    U, n = args.inducing, (args.n or 9568)
    dtype = args.dtype or "f64"
    steps = args.steps if args.steps is not None else 5
    warmup = args.warmup if args.warmup is not None else 1
    w = workloads.make_sgp(U, n, dtype=dtype)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    Kuu, Kuf, kff, y = dev(w["Kuu"]), dev(w["Kuf"]), dev(w["Kff_diag"]), dev(w["y"])
    ws = torch.empty(int(la.load().la_sgp_workspace_bytes(0 if dtype == "f32" else 1, U, n)), dtype=torch.uint8,
                     device="cuda")
    run = lambda: la.sgp_criterion(Kuu, Kuf, kff, y, w["noise_var"], workspace=ws)
    for _ in range(warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        out = run()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    # useful flops: two potrf (U^3 / 3 each), two potrf backward (2 U^3 each), trsm and its backward solve
    # (U^2 n each), syrk (U^2 n), its backward product (2 U^2 n), the triangular outer product (U^2 n)
    flops = (2.0 / 3.0 + 4.0) * U ** 3 + 6.0 * U * U * n
    log(f"[bench] SGP U={U} n={n} {dtype}: {ms:.3f} ms per criterion+gradient, phi = {float(out['phi'][0]):.6f}")
    cpu = None
    if not args.no_cpu_baseline:
        import oracle

        Us, ns = max(1, U // 8), max(1, n // 8)
        ws_ = workloads.make_sgp(Us, ns, dtype=dtype)
        t0, passes = time.perf_counter(), 0
        while True:
            oracle.sgp_criterion(ws_["Kuu"], ws_["Kuf"], ws_["Kff_diag"], ws_["y"], ws_["noise_var"])
            passes += 1
            dt_cpu = time.perf_counter() - t0
            if dt_cpu >= 10.0 or passes >= 50:
                break
        cpu = {"value": passes / dt_cpu, "unit": "evaluations/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"U={Us}, n={ns} (one eighth of each dimension, about 1/512 of the work), {passes} passes, "
                         f"{dt_cpu:.2f} s in total"}
    peak = PEAK_TFLOPS[dtype]
    print(json.dumps({
        "metric": "sparse-GP criterion+gradient evaluations/s", "value": 1e3 / ms, "unit": "evaluations/s", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": {"workload": f"SGP: U={U} n={n} {dtype} (shape of the paper's 'power' experiment)"},
        "gflops": flops / (ms * 1e-3) / 1e9, "useful_flops_per_step": flops,
        "roofline": {"bound": "mfma", "kernel": "la_sgp_criterion (all launches)", "achieved": flops / (ms * 1e-3) / 1e12,
                     "peak": peak, "unit": "TFLOP/s", "frac": flops / (ms * 1e-3) / 1e12 / peak, "traffic": None},
        "cpu_baseline": cpu}), flush=True)


def bench_kalman(args, la, torch, np, workloads):
    """Third workload (section 3.4): one step = one call of la_kalman_filter over a batch of
    sequences: likelihood, filtered means and covariances of every time step."""
    dh, dv = (int(x) for x in args.kf_dims.split(","))
    T = args.kf_steps
    batch = args.batch or 65536
    dtype = args.dtype or "f32"
    steps = args.steps if args.steps is not None else 10
    warmup = args.warmup if args.warmup is not None else 2
    w = workloads.make_kalman(batch, T, dh, dv, dtype=dtype, shared=True)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    ops = [dev(w[k]) for k in ("A", "B", "Sh", "Sv", "mu0", "S0", "v")]
    run = lambda: la.kalman_filter(*ops)
    for _ in range(warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        out = run()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for a, b in ev:
        a.record()
        run()
        b.record()
    torch.cuda.synchronize()
    kms = float(np.mean([a.elapsed_time(b) for a, b in ev]))
    # dense flop counts of the step's products and solves (the prediction is skipped at t = 0)
    predict = 2.0 * dh * dh + 4.0 * dh ** 3
    update = (2.0 * dv * dh + 2.0 * dh * dh * dv + 2.0 * dv * dv * dh + dv ** 3 / 3.0 + 2.0 * dh * dv * dv + 2.0 * dh * dv
              + dv * dv + 2.0 * dh * dh * dv + 4.0 * dh ** 3 + 2.0 * dv * dv * dh + 2.0 * dh * dh * dv)
    flops = batch * (T * update + (T - 1) * predict)
    s = 4 if dtype == "f32" else 8
    alg_bytes = batch * T * (dv + dh + dh * dh) * s
    seqsteps = batch * T
    log(f"[bench] KF batch={batch} T={T} dh={dh} dv={dv} {dtype}: {ms:.3f} ms per call (kernel {kms:.3f} ms), "
        f"mean nll = {float(out[0].double().mean()):.6f}")
    cpu = None
    if not args.no_cpu_baseline:
        import oracle

        sb = min(batch, 4096)
        ws_ = {k: (w[k][:sb] if k == "v" else w[k]) for k in ("A", "B", "Sh", "Sv", "mu0", "S0", "v")}
        t0, passes = time.perf_counter(), 0
        while True:
            oracle.kalman_filter(ws_["A"], ws_["B"], ws_["Sh"], ws_["Sv"], ws_["mu0"], ws_["S0"], ws_["v"])
            passes += 1
            dt_cpu = time.perf_counter() - t0
            if dt_cpu >= 10.0 or passes >= 50:
                break
        cpu = {"value": passes * sb * T / dt_cpu, "unit": "sequence-steps/s", "cores": oracle.num_threads(),
               "kind": "oracle", "sample": f"the first {sb} sequences, {passes} passes, {dt_cpu:.2f} s in total"}
    # vector FMA rate: 256 CUs x 4 SIMDs x 16 lanes x 2 flops x 2.4 GHz = 78.6 TFLOP/s for fp64 and for
    # one-per-lane fp32 multiply-adds; the published fp32 figure (157.3) counts two per lane (packed), a
    # form the lane-broadcast multiply-adds of this kernel do not have
    peak = PEAK_TFLOPS[dtype]
    ach = flops / (kms * 1e-3) / 1e12
    print(json.dumps({
        "metric": "Kalman filter sequence-steps/s", "value": seqsteps / (ms * 1e-3), "unit": "sequence-steps/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": {"workload": f"KF: batch={batch} T={T} dh={dh} dv={dv} {dtype}, one parameter set for all sequences"},
        "gflops": flops / (ms * 1e-3) / 1e9, "useful_flops_per_step": flops,
        "roofline": {"bound": "alu", "kernel": "k_kalman", "achieved": ach, "peak": peak, "unit": "TFLOP/s",
                     "frac": ach / peak, "traffic": None, "avg_launch_ms": kms,
                     "frac_of_unpacked_fma_rate": ach / 78.6,
                     "hbm_frac_on_algorithmic_bytes": alg_bytes / (kms * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "cpu_baseline": cpu}), flush=True)


def bench_small(args, la, torch, np, workloads):
    """Operators of the path on many small matrices (batch mode, section 4.1): one step = potrf, trsm, trmm,
    syrk, sumlogdiag, potrf backward, gemm2, potri and the trsm / trmm / syrk backward rules, each once
    over the whole batch.  Inputs are seeded like the C2 workload (A = X X^T / 2n + I / 2)."""
    n = args.n or 16
    dtype = args.dtype or "f32"
    batch = args.batch or 65536 * 256 // (n * n)
    m, k = min(n, 16), min(2 * n, 32)
    steps = args.steps if args.steps is not None else 20
    warmup = args.warmup if args.warmup is not None else 3
    s = 4 if dtype == "f32" else 8
    rng = np.random.default_rng(171008717 + 9000 + n)
    dt = workloads.np_dtype(dtype)
    X = rng.standard_normal((batch, n, k)).astype(dt)
    A = torch.from_numpy(X).cuda()
    Aspd = (A @ A.transpose(1, 2) / k + 0.5 * torch.eye(n, dtype=A.dtype, device="cuda")).contiguous()
    B = torch.from_numpy(rng.standard_normal((batch, n, m)).astype(dt)).cuda()
    Gb = torch.from_numpy(rng.standard_normal((batch, n, m)).astype(dt)).cuda()
    Lbar = torch.tril(torch.from_numpy(rng.standard_normal((batch, n, n)).astype(dt)).cuda())
    Gs = torch.from_numpy(rng.standard_normal((batch, n, n)).astype(dt)).cuda()
    L = la.potrf(Aspd)
    o_nn = [torch.empty_like(Aspd) for _ in range(4)]
    o_nm = [torch.empty_like(B) for _ in range(4)]
    o_nk = torch.empty_like(A)
    o_b = torch.empty(batch, dtype=A.dtype, device="cuda")
    nn, nm, nk = n * n * s * batch, n * m * s * batch, n * k * s * batch
    ops = {  # name -> (call, bytes of its operands and results as full rectangles)
        "potrf": (lambda: la.potrf(Aspd, out=o_nn[0]), 2 * nn),
        "backward": (lambda: la.potrf_backward(L, Lbar, out=o_nn[1]), 3 * nn),
        "trsm": (lambda: la.trsm(L, B, out=o_nm[0]), nn + 2 * nm),
        "trmm": (lambda: la.trmm(L, B, out=o_nm[1]), nn + 2 * nm),
        "syrk": (lambda: la.syrk(A, out=o_nn[2]), nk + nn),
        "sumlogdiag": (lambda: la.sumlogdiag(L, out=o_b), nn),
        "gemm2": (lambda: la.gemm2(L, B, out=o_nm[2]), nn + 2 * nm),
        "potri": (lambda: la.potri(L, out=o_nn[3]), 2 * nn),
        "trsm_backward": (lambda: la.trsm_backward(L, o_nm[0], Gb, out_a=o_nm[3], out_l=o_nn[2]), 2 * nn + 3 * nm),
        "trmm_backward": (lambda: la.trmm_backward(L, B, Gb, out_a=o_nm[3], out_l=o_nn[2]), 2 * nn + 3 * nm),
        "syrk_backward": (lambda: la.syrk_backward(A, Gs, out=o_nk), nn + 2 * nk),
    }

    def step():
        for f, _ in ops.values():
            f()

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    kernel_ms = {}
    for name, (f, _) in ops.items():
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        for a, b in ev:
            a.record()
            f()
            b.record()
        torch.cuda.synchronize()
        kernel_ms[name] = float(np.mean([a.elapsed_time(b) for a, b in ev]))
    tbs = {name: ops[name][1] / (kernel_ms[name] * 1e-3) / 1e12 for name in ops}
    log(f"[bench] SMALL batch={batch} n={n} m={m} k={k} {dtype}: {ms:.3f} ms per step; per operator (us, TB/s): "
        + ", ".join(f"{nm_} {kernel_ms[nm_] * 1e3:.0f} {tbs[nm_]:.2f}" for nm_ in ops))
    cpu = None
    if not args.no_cpu_baseline:
        import oracle

        sb = min(batch, 4096)
        Lh, Bh, lb_h = L[:sb].cpu().numpy(), B[:sb].cpu().numpy(), Lbar[:sb].cpu().numpy()
        t0, passes = time.perf_counter(), 0
        while True:
            oracle.trsm(Lh, Bh)
            oracle.potrf_backward(Lh, lb_h)
            passes += 1
            dt_cpu = time.perf_counter() - t0
            if dt_cpu >= 10.0 or passes >= 200:
                break
        cpu = {"value": passes * sb / dt_cpu, "unit": "matrices/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"trsm + potrf backward on the first {sb} matrices, {passes} passes, {dt_cpu:.2f} s in total"}
    dom = "backward"
    ach = ops[dom][1] / (kernel_ms[dom] * 1e-3) / 1e9
    print(json.dumps({
        "metric": "small-matrix operator set, matrices/s", "value": batch / (ms * 1e-3), "unit": "matrices/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": {"workload": f"SMALL: batch={batch} n={n} vectors={m} inner={k} {dtype}", "ops": list(ops)},
        "kernel_ms": kernel_ms, "tb_per_s_full_rectangles": tbs,
        "roofline": {"bound": "hbm", "kernel": "la_potrf_backward", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": ach / HBM_PEAK_GBS, "traffic": None, "byte_model": "operands and results as full squares"},
        "cpu_baseline": cpu}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--config", default="C2", choices=["C1", "C2", "C3", "C4", "C5", "SGP", "KF", "SMALL"])
    ap.add_argument("--kf-dims", default="16,16", help="KF only: state and observation dimension, dh,dv (each <= 16)")
    ap.add_argument("--kf-steps", type=int, default=32, help="KF only: time steps per sequence")
    ap.add_argument("--inducing", type=int, default=3200, help="SGP only: number of inducing points U")
    ap.add_argument("--unfused", action="store_true",
                    help="C3 only: the operator chain potrf, 2 x trsm, glue, backward instead of the one-launch la_gp_criterion")
    ap.add_argument("--with-backward-ops", action="store_true",
                    help="C4 only: also run trmm / trsm / syrk backward on the step's operands")
    ap.add_argument("--dtype", default=None, choices=["f32", "f64"])
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--n", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-secondary", action="store_true",
                    help="default (C2) run only: skip the blocked configurations C4 and C5-fp64 reported under `secondary`")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run plain device copies of 256 MiB (reference rows for rocprofv3 --pmc byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1")
        sys.exit(2)

    import numpy as np
    import torch

    import paper_1710_08717_amd as la
    import workloads

    la.load()  # raises if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    name = args.config
    if name == "SGP":
        return bench_sgp(args, la, torch, np, workloads)
    if name == "KF":
        return bench_kalman(args, la, torch, np, workloads)
    if name == "SMALL":
        return bench_small(args, la, torch, np, workloads)
    out = run_config(name, args, la, torch, np, workloads)
    if name == "C2" and not args.no_secondary and args.batch is None and args.n is None and args.dtype is None:
        # The metric has a second half, "n >= 512 potrf + backward against the fp64 matrix-core peak": the two
        # blocked configurations run in the same process, same steps and warm-up, and ride along under `secondary`.
        out["secondary"] = {}
        for key, cfg, dt in (("C4", "C4", None), ("C5_f64", "C5", "f64")):
            sub = argparse.Namespace(**vars(args))
            sub.config, sub.dtype = cfg, dt
            r = run_config(cfg, sub, la, torch, np, workloads)
            out["secondary"][key] = {
                "workload": r["config"]["workload"], "ops": r["config"]["ops"], "dtype": r["dtype"],
                "steps": r["steps"], "warmup": r["warmup"], "ms_per_step": r["ms_per_step"],
                "value": r["value"], "unit": r["unit"], "gflops": r["gflops"],
                "useful_flops_per_step": r["useful_flops_per_step"], "kernel_ms": r["kernel_ms"],
                "roofline": r["roofline"], "cpu_baseline": r["cpu_baseline"]}
            torch.cuda.empty_cache()
    print(json.dumps(out), flush=True)


def run_config(name, args, la, torch, np, workloads):
    """One of the five configurations: returns the JSON record of its run."""
    w = workloads.make(name, batch=args.batch, n=args.n, dtype=args.dtype)
    batch, n, dtype, m = w["batch"], w["n"], w["dtype"], w["m"]
    s = 4 if dtype == "f32" else 8
    steps = args.steps if args.steps is not None else {"C1": 200, "C2": 200, "C3": 100, "C4": 20, "C5": 3}[name]
    warmup = args.warmup if args.warmup is not None else {"C1": 20, "C2": 20, "C3": 10, "C4": 3, "C5": 1}[name]
    log(f"[bench] {name}: batch={batch} n={n} dtype={dtype} m={m} steps={steps} warmup={warmup}")

    extra = bool(args.with_backward_ops) and name == "C4"
    fused_gp = name == "C3" and not args.unfused
    # ---- resident inputs, several rotating buffer sets -----------------------------
    set_bytes = 4 * batch * n * n * s
    nsets = int(max(1, min(8, (1 << 31) // max(set_bytes, 1)))) if name != "C5" else 1
    A0 = torch.from_numpy(w["A"]).cuda()
    G0 = torch.from_numpy(w["Lbar"]).cuda()
    sets = []
    for i in range(nsets):
        d = {"A": A0.clone() if i else A0, "G": G0.clone() if i else G0,
             "L": torch.empty_like(A0), "Abar": torch.empty_like(A0)}
        if "rhs" in w:
            d["rhs"] = torch.from_numpy(w["rhs"]).cuda()
            d["X"] = torch.empty_like(d["rhs"])
            d["Y"] = torch.empty_like(d["rhs"])
        if name == "C3":
            d["y"] = torch.from_numpy(w["y"]).cuda().contiguous()
            d["z"] = torch.empty_like(d["y"])
            d["alpha"] = torch.empty_like(d["y"])
            d["loss"] = torch.empty(batch, dtype=A0.dtype, device="cuda")
        if name == "C1":
            d["sld"] = torch.empty(batch, dtype=A0.dtype, device="cuda")
        if extra:
            d["Ybar"] = torch.from_numpy(w["rhs"][:, ::-1, :].copy()).cuda()  # any fixed upstream gradient
            for k_ in ("Xbar", "Rbar", "Sbar"):
                d[k_] = torch.empty_like(d["rhs"])
            d["Lb1"] = torch.empty_like(A0)
            d["Lb2"] = torch.empty_like(A0)
        sets.append(d)
    # one workspace for every call of the step (the calls run one after the other on one stream)
    from paper_1710_08717_amd import binding as B_

    need = max([la.workspace_bytes(B_.OP_POTRF, A0, batch, n), la.workspace_bytes(B_.OP_POTRF_BACKWARD, A0, batch, n)]
               + ([la.workspace_bytes(o, A0, batch, n, m) for o in (B_.OP_TRSM, B_.OP_TRMM, B_.OP_TRSM_BACKWARD,
                                                                    B_.OP_TRMM_BACKWARD)] if m else [])
               + ([la.workspace_bytes(B_.OP_SYRK_BACKWARD, A0, batch, n, 0, m)] if extra else []))
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
    log(f"[bench] workspace for the step's calls: {need / 2 ** 20:.1f} MiB")
    torch.cuda.synchronize()

    timers = {}
    # the events of the second region exist before it starts (an event is created at its first record; growing
    # the runtime's event pool in the middle of the region showed up as one 38 ms gap inside a bracketed call)
    pool = [torch.cuda.Event(enable_timing=True) for _ in range(2 * 8 * steps)]
    for e in pool:
        e.record()
    torch.cuda.synchronize()

    def call(tag, fn, timed):
        if not timed:
            fn()
            return
        e0 = pool.pop() if pool else torch.cuda.Event(enable_timing=True)
        e1 = pool.pop() if pool else torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        timers.setdefault(tag, []).append((e0, e1))

    def step(i, timed=False):
        d = sets[i % nsets]
        if fused_gp:  # C3: the whole criterion + gradient is one launch
            call("gp_criterion", lambda: la.gp_criterion(d["A"], d["y"], out=d["Abar"], loss=d["loss"]), timed)
            return
        call("potrf", lambda: la.potrf(d["A"], out=d["L"], workspace=ws), timed)
        if name == "C1":
            call("trsm", lambda: la.trsm(d["L"], d["rhs"], out=d["X"], workspace=ws), timed)
            call("sumlogdiag", lambda: la.sumlogdiag(d["L"], out=d["sld"]), timed)
        elif name == "C3":
            yv, zv, av = d["y"].view(batch, n, 1), d["z"].view(batch, n, 1), d["alpha"].view(batch, n, 1)
            call("trsm", lambda: (la.trsm(d["L"], yv, out=zv, workspace=ws), la.trsm(d["L"], zv, trans=True, out=av, workspace=ws)), timed)
            call("gp_glue", lambda: la.gp_glue(d["L"], d["y"], d["z"], d["alpha"], loss=d["loss"], Lbar=d["G"]), timed)
        elif name == "C4":
            call("trsm", lambda: la.trsm(d["L"], d["rhs"], out=d["X"], workspace=ws), timed)
            call("trmm", lambda: la.trmm(d["L"], d["X"], out=d["Y"], workspace=ws), timed)
            if extra:
                call("trmm_backward", lambda: la.trmm_backward(d["L"], d["X"], d["Ybar"], out_a=d["Xbar"], out_l=d["Lb1"],
                                                                  workspace=ws),
                     timed)
                call("trsm_backward", lambda: la.trsm_backward(d["L"], d["X"], d["Xbar"], out_a=d["Rbar"], out_l=d["Lb2"],
                                                                  workspace=ws),
                     timed)
                call("syrk_backward", lambda: la.syrk_backward(d["rhs"], d["G"], out=d["Sbar"], workspace=ws), timed)
        elif name == "C5":
            call("trsm", lambda: la.trsm(d["L"], d["rhs"], out=d["X"], workspace=ws), timed)
        call("backward", lambda: la.potrf_backward(d["L"], d["G"], out=d["Abar"], workspace=ws), timed)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / steps
    log(f"[bench] region 1: {ms_per_step:.4f} ms/step")

    for i in range(steps):
        step(i, timed=True)
    torch.cuda.synchronize()
    kern_ms = {k: float(np.mean([a.elapsed_time(b) for a, b in v])) for k, v in timers.items()}
    log(f"[bench] region 2 (per entry point, ms): {kern_ms}")

    if args.calib_copy:
        src = torch.empty(1 << 26, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)  # plain elementwise copy kernel: reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()

    fm = flops_model(name, n, m, batch, s)
    if extra:  # product with the triangle + kept triangle of an n x n outer product; two n x n x m products
        fm.update({"trmm_backward": 2.0 * n * n * m, "trsm_backward": 2.0 * n * n * m, "syrk_backward": 4.0 * n * n * m})
    total_flops = batch * sum(fm.values())
    mats_per_s = batch / (ms_per_step * 1e-3)
    gflops = total_flops / (ms_per_step * 1e-3) / 1e9

    # ---- roofline of the dominant kernel -------------------------------------------
    if fused_gp:
        alg_bytes = (n * (n + 1) // 2 + n + n * n + 1) * s * batch  # lower triangle of A, y; Abar in full, loss
        achieved = alg_bytes / (kern_ms["gp_criterion"] * 1e-3) / 1e9
        roof = {"bound": "hbm", "kernel": "k_gp_leaf16 (la_gp_criterion)", "achieved": achieved, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                "algorithmic_bytes_per_launch": alg_bytes, "avg_launch_ms": kern_ms["gp_criterion"],
                "note": "latency bound: one workgroup per matrix walks the 8 tile columns of the factorisation in turn"}
    elif name in ("C1", "C2", "C3"):
        bm = bytes_model(n, s)
        dom = "backward"
        alg_bytes = bm[dom] * batch
        achieved = alg_bytes / (kern_ms[dom] * 1e-3) / 1e9
        roof = {"bound": "hbm", "kernel": "la_potrf_backward", "achieved": achieved, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                "algorithmic_bytes_per_launch": alg_bytes, "avg_launch_ms": kern_ms[dom],
                "duration_source": "HIP event pair around each launch on the launch stream, averaged over the timed "
                                   "steps (an event pair adds about 1-2.5 us to a bracketed launch; the rocprofv3 kernel "
                                   "trace under profiles/ gives the kernel alone)",
                "potrf_forward": {"achieved": bm["potrf"] * batch / (kern_ms["potrf"] * 1e-3) / 1e9,
                                  "avg_launch_ms": kern_ms["potrf"],
                                  "frac": bm["potrf"] * batch / (kern_ms["potrf"] * 1e-3) / 1e9 / HBM_PEAK_GBS}}
        tf = os.path.join(ROOT, "profiles", f"traffic_{name.lower()}.json")
        if os.path.exists(tf):
            with open(tf) as f:
                roof["traffic"] = json.load(f).get("backward_bytes_per_launch")
    else:
        dom = "backward"
        fl = fm[dom] * batch
        achieved = fl / (kern_ms[dom] * 1e-3) / 1e12
        roof = {"bound": "mfma", "kernel": "la_potrf_backward (GEMM phases)", "achieved": achieved,
                "peak": PEAK_TFLOPS[dtype], "unit": "TFLOP/s", "frac": achieved / PEAK_TFLOPS[dtype], "traffic": None,
                "useful_flops_per_call": fl, "avg_call_ms": kern_ms[dom],
                "flop_model": "as executed: 2 n^3 per matrix for the closed expression"
                              + ("" if fl == 2.0 * n ** 3 * batch else "; reverse sweep over the blocked factorisation "
                                 "above the base block (2 n1 n2 n per level, 2 n0^3 per base block), "
                                 f"{fl / (2.0 * n ** 3 * batch):.3f} of the closed expression's count"),
                "duration_source": "HIP event pair around each library call on the launch stream (a call is many "
                                   "launches), averaged over the timed steps",
                "per_call": {k_: {"ms": kern_ms[k_], "tflops": fm[k_] * batch / (kern_ms[k_] * 1e-3) / 1e12,
                                  "frac": fm[k_] * batch / (kern_ms[k_] * 1e-3) / 1e12 / PEAK_TFLOPS[dtype]}
                             for k_ in kern_ms if k_ in fm},
                "whole_step_frac": gflops / 1e3 / PEAK_TFLOPS[dtype]}

    # ---- CPU baseline: the oracle, as it stands, on this machine's host cores ------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle

        sb = batch
        # bounded sample: shrink the batch until a pass is a few seconds of CPU work
        est = sb * (n ** 3) * 2.0  # rough oracle flops (fwd + composite backward)
        while sb > 1 and est > 6e10:
            sb //= 2
            est /= 2
        if name == "C5":
            # one matrix of the full size takes the oracle minutes: time the leading ns x ns problem (an SPD matrix
            # of the same recipe) and scale by the cubic flop count
            ns, ms_ = 4096, 256
            As = np.ascontiguousarray(w["A"][:, :ns, :ns], dtype=np.float64)
            Gs = np.ascontiguousarray(w["Lbar"][:, :ns, :ns], dtype=np.float64)
            Rs = np.ascontiguousarray(w["rhs"][:, :ns, :ms_], dtype=np.float64)
            t0 = time.perf_counter()
            Lr = oracle.potrf(As)
            oracle.potrf_backward(Lr, Gs)
            oracle.trsm(Lr, Rs)
            dt_cpu = time.perf_counter() - t0
            scale = (ns / n) ** 3
            cpu = {"value": scale / dt_cpu, "unit": "matrices/s", "cores": oracle.num_threads(), "kind": "oracle",
                   "sample": f"leading {ns} x {ns} block of the C5 matrix with {ms_} right-hand sides, one pass, "
                             f"{dt_cpu:.2f} s; value = (1 / time) x ({ns}/{n})^3, the cubic flop ratio",
                   "gflops": sum(flops_model(name, ns, ms_).values()) / dt_cpu / 1e9}
        else:
            As = np.ascontiguousarray(w["A"][:sb], dtype=np.float64)
            Gs = np.ascontiguousarray(w["Lbar"][:sb], dtype=np.float64)
            Rs = np.ascontiguousarray(w["rhs"][:sb], dtype=np.float64) if "rhs" in w else None
            passes, t0 = 0, time.perf_counter()
            while True:  # whole passes of the same ops until about 10 s of CPU work are spent
                Lr = oracle.potrf(As)
                oracle.potrf_backward(Lr, Gs)
                if Rs is not None:
                    X = oracle.trsm(Lr, Rs)
                    if name == "C4":
                        oracle.trmm(Lr, X)
                    if extra:
                        xb, _ = oracle.trmm_backward(Lr, X, Rs[:, ::-1, :])
                        oracle.trsm_backward(Lr, X, xb)
                        oracle.syrk_backward(Rs, Gs)
                passes += 1
                dt_cpu = time.perf_counter() - t0
                if dt_cpu >= 10.0 or passes >= 200:
                    break
            cpu = {"value": sb * passes / dt_cpu, "unit": "matrices/s", "cores": oracle.num_threads(),
                   "kind": "oracle",
                   "sample": f"first {sb} of {batch} matrices of {name}, {passes} passes of the same ops "
                             f"(fp64 oracle on the fp32-rounded inputs), {dt_cpu:.2f} s in total",
                   "gflops": sb * passes * sum(fm.values()) / dt_cpu / 1e9}
        log(f"[bench] cpu baseline: {cpu}")

    out = {
        "metric": "batched potrf fwd+bwd matrices/s",
        "value": mats_per_s,
        "unit": "matrices/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": dtype,
        "data": "synthetic",
        "config": {"workload": f"{name}: batch={batch} n={n} {dtype}" + (f" rhs={m}" if m else ""),
                   "ops": (["gp_criterion (potrf, 2 x trsm, sumlogdiag, glue, backward in one launch)"] if fused_gp
                           else list(fm.keys()) + (["gp_glue"] if name == "C3" else [])), "buffer_sets": nsets},
        "gflops": gflops,
        "useful_flops_per_step": total_flops,
        "kernel_ms": kern_ms,
        "roofline": roof,
        "cpu_baseline": cpu,
    }
    del sets, A0, G0
    return out


if __name__ == "__main__":
    main()
