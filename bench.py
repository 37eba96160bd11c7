"""Benchmark of the collapsed Taylor-mode hot path on one MI355X.

One step = one operator call over the whole batch: seed the coefficient block, the stacked
GEMM + jet rule of every hidden layer, and the last layer.  Inputs are resident in HBM before
the timed region.  Prints one JSON line:
  value / unit        operator evaluations per second (N / time per step), whole job
  roofline            the stacked-GEMM launches of a step: algorithmic flops / their HIP-event-timed duration
                      against the dense MFMA peak of the arithmetic type; `traffic` = HBM bytes per launch from
                      the committed rocprofv3 FETCH_SIZE / WRITE_SIZE summary of the workload and variant (profiles/layer_kernel_<tag>.txt; null if none)
  cpu_baseline        the fp64 numpy oracle timed on the host cores for a bounded sample of the same workload
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "Laplacian evals/sec (50-D 768-768-512-512 tanh MLP, N=4096); % MFMA peak"
PEAK_TFLOPS = {"f32": 157.3, "f64": 78.6, "bf16": 2500.0, "bf16x3": 2500.0}  # MI355X dense MFMA peaks


def gemm_flops(dims, N, rho, R, per_point_dirs):
    """Algorithmic flops of the stacked-GEMM launches of one call.  Hidden layers 2..L-1 multiply all
    N*rho coefficient rows: 2 * N * rho * d_in * d_out (un-padded widths, collapsed row count).  The first
    layer goes through the GEMM kernel only when directions differ per point in more than 16 input dimensions
    (or the input is wider than 64), and then only its 1 + R non-zero rows per point count.  The width-1 last
    layer is not a GEMM."""
    f = sum(2.0 * N * rho * dims[l] * dims[l + 1] for l in range(1, len(dims) - 2))
    if (per_point_dirs and dims[0] > 16) or dims[0] > 64:
        f += 2.0 * N * (1 + R) * dims[0] * dims[1]
    return f


def recorded_traffic(tag):
    """HBM bytes per stacked-GEMM launch from the committed rocprofv3 FETCH_SIZE / WRITE_SIZE summary of this
    workload and variant (counters cannot be read from inside this process); None if there is no such summary.
    tag: the workload name, plus _bf16 / _bf16x3 / _f64 / _backward for the variants."""
    path = os.path.join(ROOT, "profiles", f"layer_kernel_{tag}.txt")
    try:
        with open(path) as fh:
            for line in fh:
                if line.startswith("traffic_bytes_per_launch:"):
                    return float(line.split(":")[1])
    except OSError:
        pass
    return None


def cpu_baseline(w, arrs, budget_s):
    """The oracle as it stands (full Hessian per point, then the trace or contraction / 4th directional
    derivatives), timed on the host cores for a bounded sample of the same workload."""
    import numpy as np
    from threadpoolctl import threadpool_info

    from oracle import operators as orc

    def run(P):
        sub = dict(arrs, x=arrs["x"][:P])
        V = arrs.get("V")
        if V is not None and V.ndim == 3:
            sub["V"] = V[:P]
        t0 = time.perf_counter()
        if w.op == "laplacian":
            orc.laplacian(sub["Ws"], sub["bs"], sub["x"], sub.get("V"), sub.get("scale", 1.0), mode="hessian")
        elif w.op == "weighted_laplacian":
            orc.weighted_laplacian(sub["Ws"], sub["bs"], sub["x"], sub["sigma"], mode="hessian")
        elif w.op == "biharmonic_exact":
            orc.biharmonic_exact(sub["Ws"], sub["bs"], sub["x"])
        else:
            orc.biharmonic_rand(sub["Ws"], sub["bs"], sub["x"], sub["V"])
        return time.perf_counter() - t0

    p0 = min(8, w.N)
    t_probe = run(p0)
    P = int(max(p0, min(w.N, budget_s / max(t_probe / p0, 1e-9))))
    t = run(P)
    kind = {"biharmonic_rand": "4-level duals per direction", "biharmonic_exact": "4-level duals per index pair (i,i,j,j)"}.get(
        w.op, "full Hessian per point")
    info = threadpool_info()
    cores = max([i.get("num_threads", 1) for i in info] or [1])
    return {"value": P / t, "unit": "evals/s", "cores": cores, "kind": "oracle",
            "sample": f"first {P} of {w.N} points of {w.name}, fp64 numpy nested-dual oracle "
                      f"({kind}), {t:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c2", help="c1..c5 (c2 is the configuration the metric is quoted on)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="budget of the oracle baseline; 0 skips it")
    ap.add_argument("--mfma", choices=["native", "bf16x3", "bf16"], default="native",
                    help="matrix cores used by the GEMMs of an fp32 workload: native fp32 (default), split bf16 or plain bf16")
    ap.add_argument("--taylor", choices=["collapsed", "standard"], default="collapsed",
                    help="standard = the un-collapsed comparison path (1 + K*R rows per point); c1..c5 only")
    ap.add_argument("--backward", action="store_true",
                    help="time forward-with-tape plus the reverse pass to all weights (laplacian and biharmonic_rand workloads, collapsed, native MFMA)")
    ap.add_argument("--fp64", action="store_true", help="run an fp32 workload with every array widened to fp64 (fp64 MFMA kernels)")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="also launch one plain device copy of this many MiB (calibrates rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (points are independent, nothing is exchanged); use --gpus 1")

    import numpy as np
    import torch

    import paper_2505_13644_amd as ctm
    from paper_2505_13644_amd import synth

    w = synth.WORKLOADS[args.workload]
    arrs = w.build()
    if args.fp64:
        if args.mfma != "native":
            sys.exit("bench.py: --fp64 and --mfma exclude each other")
        wide = lambda v: [a.astype(np.float64) for a in v] if isinstance(v, list) else (v.astype(np.float64) if isinstance(v, np.ndarray) else v)
        arrs = {k: wide(v) for k, v in arrs.items()}
    dev = torch.device("cuda:0")
    t = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    mfma = {"native": None, "bf16x3": ctm.CTM_F32_BF16X3, "bf16": ctm.CTM_F32_BF16}[args.mfma]
    mlp = ctm.ctm_create_mlp([t(W) for W in arrs["Ws"]], [t(b) for b in arrs["bs"]], mfma=mfma)
    x, V, sigma = t(arrs["x"]), t(arrs.get("V")), t(arrs.get("sigma"))
    K = 4 if w.op.startswith("biharmonic") else 2
    R = w.dims[0] if w.directions == "basis" else w.R
    u = torch.empty(w.N, dtype=x.dtype, device=dev)
    op = torch.empty(w.N, dtype=x.dtype, device=dev)
    if w.op == "biharmonic_exact":
        ws_bytes = ctm.binding.lib().ctm_biharmonic_exact_workspace_bytes(mlp.handle, w.N)
    else:
        ws_bytes = ctm.ctm_workspace_bytes(mlp, K, w.N, R)
    std = args.taylor == "standard"
    if std:
        if w.op not in ("laplacian", "biharmonic_rand", "weighted_laplacian"):
            sys.exit("bench.py: --taylor standard covers the laplacian / weighted_laplacian / biharmonic_rand workloads")
        ws_bytes = ctm.binding.lib().ctm_workspace_bytes_standard(mlp.handle, K, w.N, R)
        Vstd = sigma.t().contiguous() if w.op == "weighted_laplacian" else V
        std_scale = 1.0 / (3.0 * R) if K == 4 else arrs.get("scale", 1.0)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)

    bwd = args.backward
    if bwd:
        if w.op not in ("laplacian", "biharmonic_rand") or std or args.mfma != "native":
            sys.exit("bench.py: --backward covers the laplacian and biharmonic_rand workloads with collapsed Taylor mode and native MFMA")
        if K == 4:
            tape = torch.empty(ctm.ctm_biharmonic_tape_bytes(mlp, w.N, R), dtype=torch.uint8, device=dev)
            ws = torch.empty(ctm.ctm_biharmonic_backward_workspace_bytes(mlp, w.N, R), dtype=torch.uint8, device=dev)
        else:
            tape = torch.empty(ctm.ctm_tape_bytes(mlp, w.N, R), dtype=torch.uint8, device=dev)
            ws = torch.empty(ctm.ctm_backward_workspace_bytes(mlp, w.N, R), dtype=torch.uint8, device=dev)
        gu = torch.ones(w.N, dtype=x.dtype, device=dev)
        gop = torch.ones(w.N, dtype=x.dtype, device=dev)
        nl = len(w.dims) - 1
        gW = [torch.empty(w.dims[l + 1], w.dims[l], dtype=x.dtype, device=dev) for l in range(nl)]
        gb = [torch.empty(w.dims[l + 1], dtype=x.dtype, device=dev) for l in range(nl)]

    def step():
        if bwd and K == 4:
            ctm.ctm_biharmonic_rand_fwd(mlp, x, V, u, op, tape)
            ctm.ctm_biharmonic_rand_bwd(mlp, w.N, R, tape, gu, gop, gW, gb, ws)
        elif bwd:
            ctm.ctm_laplacian_fwd(mlp, x, V, arrs.get("scale", 1.0), u, op, tape)
            ctm.ctm_laplacian_bwd(mlp, w.N, R, arrs.get("scale", 1.0), tape, gu, gop, gW, gb, ws)
        elif std:
            ctm.ctm_taylor_standard(mlp, K, x, Vstd, std_scale, u, op, ws)
        elif w.op == "laplacian":
            ctm.ctm_laplacian(mlp, x, V, arrs.get("scale", 1.0), u, op, ws)
        elif w.op == "weighted_laplacian":
            ctm.ctm_weighted_laplacian(mlp, x, sigma, u, op, ws)
        elif w.op == "biharmonic_exact":
            ctm.ctm_biharmonic_exact(mlp, x, u, op, ws)
        else:
            ctm.ctm_biharmonic_rand(mlp, x, V, u, op, ws)

    if args.copy_probe_mib > 0:
        src = torch.ones(args.copy_probe_mib << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3

    # per-kernel durations, measured live with HIP events on the launch stream (a second pass,
    # so the events do not sit inside the timed region above)
    ctm.ctm_profile_begin()
    for _ in range(args.steps):
        step()
    ms, launches = ctm.ctm_profile_end()

    # per-step times (the paper reports the minimum of 50 repetitions, Sec. 4): one event pair per step
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for e0, e1 in evs:
        e0.record()
        step()
        e1.record()
    torch.cuda.synchronize()
    per_step = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
    rho = 1 + K * R if std else ctm.ctm_rows_per_point(K, R)
    if w.op == "biharmonic_exact":
        D = w.dims[0]
        fams = [D, D * (D - 1), D * (D - 1) // 2]
        flops = sum(gemm_flops(w.dims, w.N, ctm.ctm_rows_per_point(4, r), r, False) for r in fams if r)
        rho = sum(ctm.ctm_rows_per_point(4, r) for r in fams if r)
    elif bwd:
        # forward GEMMs over all rows (the recording forward always builds the input block), and per hidden layer
        # one weight-gradient GEMM plus, except for the first layer, one cotangent GEMM
        fwd = sum(2.0 * w.N * rho * w.dims[l] * w.dims[l + 1] for l in range(len(w.dims) - 2))
        dgrad = sum(2.0 * w.N * rho * w.dims[l] * w.dims[l + 1] for l in range(1, len(w.dims) - 2))
        flops = fwd + fwd + dgrad
    else:
        flops = gemm_flops(w.dims, w.N, rho, R, w.directions in ("rademacher", "gaussian"))
    layer_ms_per_step = (ms["layer"] + (ms["final"] if bwd else 0.0)) / args.steps   # reverse pass: class "final" holds the weight-gradient GEMMs
    dt = "f64" if (w.dtype == np.float64 or args.fp64) else "f32"
    if args.mfma != "native":
        dt = args.mfma
        # executed matrix-core flops: 3 bf16 MFMAs per product for the split variant
        flops *= 3 if args.mfma == "bf16x3" else 1
    achieved = flops / (layer_ms_per_step * 1e-3) / 1e12
    roofline = {
        "bound": "mfma", "achieved": achieved, "peak": PEAK_TFLOPS[dt], "unit": "TFLOP/s",
        "frac": achieved / PEAK_TFLOPS[dt],
        "traffic": recorded_traffic(w.name + ("" if args.mfma == "native" else "_" + args.mfma) + ("_f64" if args.fp64 else "")
                                    + ("_backward" if bwd else "") + ("_standard" if std else "")),
        "kernel": "layer_kernel (stacked GEMM + fused jet rule)",
        "flops_per_step": flops, "launches_per_step": launches["layer"] / args.steps,
        "avg_launch_ms": ms["layer"] / max(1, launches["layer"]),
        "stage_ms_per_step": {{"seed": "first_layer_or_seed"}.get(k, k): v / args.steps for k, v in ms.items()},
    }
    # the elementwise first layer (shared directions) is bound by writing the [N*rho, d_1] block once
    es = 8 if dt == "f64" else 4
    shared_first = w.directions in ("basis", "sigma") and w.dims[0] <= 64 and w.op != "biharmonic_exact" and not bwd
    if args.mfma == "bf16":
        es = 2   # plain-bf16 handles keep the block between the layers as one bf16 plane
    if shared_first and ms["seed"] > 0:   # (the one-launch path of tiny calls has no separate first-layer kernel)
        first_bytes = (w.N * rho * w.dims[1] + w.N * w.dims[0]) * es
        first_ms = ms["seed"] / args.steps
        roofline["first_layer"] = {"bound": "hbm", "achieved": first_bytes / (first_ms * 1e-3) / 1e9, "peak": 8000.0,
                                   "unit": "GB/s", "frac": first_bytes / (first_ms * 1e-3) / 1e9 / 8000.0,
                                   "bytes_per_step": first_bytes, "ms_per_step": first_ms}
    out = {
        "metric": METRIC, "value": w.N / (ms_per_step * 1e-3), "unit": "evals/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "ms_per_step_min": per_step[0], "ms_per_step_median": per_step[len(per_step) // 2], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": dt, "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.op}, tanh MLP {'-'.join(map(str, w.dims))}, N={w.N}, "
                               f"{w.directions} directions R={R}, {args.taylor} order-{K} Taylor mode, {rho} rows/point"
                               + (", forward with tape + reverse pass to all weights" if bwd else "")},
        "roofline": roofline,
    }
    if args.fp64:
        out["config"]["workload"] += ", arrays widened to fp64"
    if args.cpu_seconds > 0:
        out["cpu_baseline"] = cpu_baseline(w, arrs, args.cpu_seconds)
    mlp.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
