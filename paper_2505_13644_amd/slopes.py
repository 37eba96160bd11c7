"""Time and memory slopes in the measurement protocol of the paper's benchmark (Sec. 4, Table 1), on this GPU.

    python -m paper_2505_13644_amd.slopes [--reps 50] [--out FILE]

For every operator the run time is the minimum over `reps` repetitions (HIP events around one call), measured for
several batch sizes N ("exact" rows: cost per added datum) or several sample counts S at a fixed batch ("stochastic"
rows: cost per added Monte-Carlo sample), and a straight line is fitted; the slope is reported.  Collapsed Taylor
mode (the library's operator calls) is timed beside standard, un-collapsed Taylor mode (ctm_taylor_standard) on the
same inputs, which gives the ratio that collapsing buys on this hardware.  Memory is what the caller must provide:
the workspace of the call ("non-differentiable") and, for collapsed mode, tape + reverse-pass workspace
("differentiable"), again as slopes.  Network: tanh MLP D-768-768-512-512-1 (Sec. 4); D = 50 for the Laplacians,
D = 5 for the biharmonic; synthetic seeded inputs.  Only the HIP library is used.
"""
from __future__ import annotations

import argparse
import sys

import numpy as np


def _fit(xs, ys):
    A = np.stack([np.asarray(xs, dtype=np.float64), np.ones(len(xs))], axis=1)
    (slope, icpt), *_ = np.linalg.lstsq(A, np.asarray(ys, dtype=np.float64), rcond=None)
    return float(slope), float(icpt)


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--reps", type=int, default=50)
    ap.add_argument("--out", default=None, help="also write the table to this file")
    args = ap.parse_args()

    import torch

    import paper_2505_13644_amd as ctm
    from paper_2505_13644_amd import synth

    dev = torch.device("cuda:0")
    t = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    hidden = (768, 768, 512, 512)
    lines = []

    def emit(s=""):
        print(s, flush=True)
        lines.append(s)

    def min_ms(fn):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        best = float("inf")
        for _ in range(args.reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            e1.synchronize()
            best = min(best, e0.elapsed_time(e1))
        return best

    def make(D):
        dims = (D,) + hidden + (1,)
        Ws, bs = synth.make_mlp(dims, 0, 0.01, np.float32)
        return ctm.ctm_create_mlp([t(W) for W in Ws], [t(b) for b in bs]), dims

    def biharm_families(D):
        E = np.eye(D, dtype=np.float32)
        f0 = 4 * E
        f1 = np.stack([3 * E[a] + E[b] for a in range(D) for b in range(D) if a != b])
        f2 = np.stack([2 * E[a] + 2 * E[b] for a in range(D) for b in range(a + 1, D)])
        return [t(f0), t(f1), t(f2)]

    lib = ctm.binding.lib()
    MiB = 1024.0 * 1024.0
    emit("operator, varied, collapsed ms/unit, standard ms/unit, time ratio, collapsed MiB/unit, standard MiB/unit, memory ratio, "
         "collapsed differentiable MiB/unit")

    # ---- exact operators: vary the batch size ------------------------------------------------------
    Ns = [1024, 2048, 4096, 8192]
    mlp50, _ = make(50)
    mlp5, _ = make(5)
    sig_diag = np.diag(synth._rng(0, "diag").uniform(0.5, 1.5, 50)).astype(np.float32)  # full-rank diagonal sigma
    fams = biharm_families(5)

    def exact_row(name, mlp, D, K, R_col, col_fn, std_fn, std_ws, diff_bytes):
        tc, ts, mc, ms_, md = [], [], [], [], []
        for N in Ns:
            x = t(synth.make_points(N, D, 0, np.float32))
            u = torch.empty(N, dtype=torch.float32, device=dev)
            op = torch.empty(N, dtype=torch.float32, device=dev)
            wc_ = torch.empty(R_col(N), dtype=torch.uint8, device=dev)
            tc.append(min_ms(lambda: col_fn(mlp, x, u, op, wc_)))
            del wc_
            ws_ = torch.empty(std_ws(N), dtype=torch.uint8, device=dev)
            ts.append(min_ms(lambda: std_fn(mlp, x, u, op, ws_)))
            del ws_
            mc.append(R_col(N) / MiB)
            ms_.append(std_ws(N) / MiB)
            md.append(diff_bytes(N) / MiB if diff_bytes else float("nan"))
        sc, ss = _fit(Ns, tc)[0], _fit(Ns, ts)[0]
        wc, wsd = _fit(Ns, mc)[0], _fit(Ns, ms_)[0]
        wd = _fit(Ns, md)[0] if diff_bytes else float("nan")
        emit(f"{name}, N in {Ns}, {sc:.6f}, {ss:.6f}, {sc / ss:.3f}, {wc:.4f}, {wsd:.4f}, {wc / wsd:.3f}, {wd:.4f}")

    exact_row("exact Laplacian (D=50)", mlp50, 50, 2,
              lambda N: ctm.ctm_workspace_bytes(mlp50, 2, N, 50),
              lambda m, x, u, op, w: ctm.ctm_laplacian(m, x, None, 1.0, u, op, w),
              lambda m, x, u, op, w: ctm.ctm_taylor_standard(m, 2, x, None, 1.0, u, op, w),
              lambda N: lib.ctm_workspace_bytes_standard(mlp50.handle, 2, N, 50),
              lambda N: ctm.ctm_tape_bytes(mlp50, N, 50) + ctm.ctm_backward_workspace_bytes(mlp50, N, 50))
    sg = t(sig_diag)
    sgT = t(sig_diag.T.copy())
    exact_row("exact weighted Laplacian (D=50, full-rank diagonal sigma)", mlp50, 50, 2,
              lambda N: ctm.ctm_workspace_bytes(mlp50, 2, N, 50),
              lambda m, x, u, op, w: ctm.ctm_weighted_laplacian(m, x, sg, u, op, w),
              lambda m, x, u, op, w: ctm.ctm_taylor_standard(m, 2, x, sgT, 1.0, u, op, w),
              lambda N: lib.ctm_workspace_bytes_standard(mlp50.handle, 2, N, 50),
              lambda N: ctm.ctm_tape_bytes(mlp50, N, 50) + ctm.ctm_backward_workspace_bytes(mlp50, N, 50))

    def std_biharm(m, x, u, op, w):
        for V in fams:  # the three direction families of the interpolation formula, un-collapsed
            ctm.ctm_taylor_standard(m, 4, x, V, 1.0, u, op, w)

    exact_row("exact biharmonic (D=5, interpolation)", mlp5, 5, 4,
              lambda N: lib.ctm_biharmonic_exact_workspace_bytes(mlp5.handle, N),
              lambda m, x, u, op, w: ctm.ctm_biharmonic_exact(m, x, u, op, w),
              std_biharm,
              lambda N: lib.ctm_workspace_bytes_standard(mlp5.handle, 4, N, 20),
              lambda N: ctm.ctm_biharmonic_exact_tape_bytes(mlp5, N) + ctm.ctm_biharmonic_exact_backward_workspace_bytes(mlp5, N))

    # ---- stochastic operators: vary the number of samples at a fixed batch ---------------------------
    def stoch_row(name, mlp, D, K, N, Ss, col_fn, std_fn, diff_bytes, col_bytes=None):
        x = t(synth.make_points(N, D, 0, np.float32))
        u = torch.empty(N, dtype=torch.float32, device=dev)
        op = torch.empty(N, dtype=torch.float32, device=dev)
        tc, ts, mc, ms_, md = [], [], [], [], []
        for S in Ss:
            V = t(synth.make_directions("gaussian", (N, S, D), 0, np.float32))
            nb = col_bytes(N, S) if col_bytes else ctm.ctm_workspace_bytes(mlp, K, N, S)
            wc_ = torch.empty(nb, dtype=torch.uint8, device=dev)
            tc.append(min_ms(lambda: col_fn(mlp, x, V, S, u, op, wc_)))
            del wc_
            ws_ = torch.empty(lib.ctm_workspace_bytes_standard(mlp.handle, K, N, S), dtype=torch.uint8, device=dev)
            ts.append(min_ms(lambda: std_fn(mlp, x, V, S, u, op, ws_)))
            del ws_
            mc.append(nb / MiB)
            ms_.append(lib.ctm_workspace_bytes_standard(mlp.handle, K, N, S) / MiB)
            md.append(diff_bytes(N, S) / MiB)
        sc, ss = _fit(Ss, tc)[0], _fit(Ss, ts)[0]
        wc, wsd, wd = _fit(Ss, mc)[0], _fit(Ss, ms_)[0], _fit(Ss, md)[0]
        emit(f"{name}, S in {Ss} at N={N}, {sc:.6f}, {ss:.6f}, {sc / ss:.3f}, {wc:.4f}, {wsd:.4f}, {wc / wsd:.3f}, {wd:.4f}")

    lap_diff = lambda N, S: ctm.ctm_tape_bytes(mlp50, N, S) + ctm.ctm_backward_workspace_bytes(mlp50, N, S)
    stoch_row("stochastic Laplacian (D=50)", mlp50, 50, 2, 2048, [8, 16, 24, 32, 40],
              lambda m, x, V, S, u, op, w: ctm.ctm_laplacian(m, x, V, 1.0 / S, u, op, w),
              lambda m, x, V, S, u, op, w: ctm.ctm_taylor_standard(m, 2, x, V, 1.0 / S, u, op, w),
              lap_diff)

    def col_wrand(m, x, V, S, u, op, w):
        ctm.ctm_weighted_laplacian_rand(m, x, sg, V, u, op, w)

    def std_wrand(m, x, V, S, u, op, w):
        dirs = torch.matmul(V, sgT)  # sigma v per point and sample (the library forms these itself in the collapsed call)
        ctm.ctm_taylor_standard(m, 2, x, dirs, 1.0 / S, u, op, w)

    stoch_row("stochastic weighted Laplacian (D=50, diagonal sigma)", mlp50, 50, 2, 2048, [8, 16, 24, 32, 40], col_wrand, std_wrand, lap_diff,
              col_bytes=lambda N, S: lib.ctm_weighted_laplacian_rand_workspace_bytes(mlp50.handle, N, 50, S, 0, S * 50))
    stoch_row("stochastic biharmonic (D=5)", mlp5, 5, 4, 256, [8, 16, 32, 48],
              lambda m, x, V, S, u, op, w: ctm.ctm_biharmonic_rand(m, x, V, u, op, w),
              lambda m, x, V, S, u, op, w: ctm.ctm_taylor_standard(m, 4, x, V, 1.0 / (3.0 * S), u, op, w),
              lambda N, S: ctm.ctm_biharmonic_tape_bytes(mlp5, N, S) + ctm.ctm_biharmonic_backward_workspace_bytes(mlp5, N, S))
    mlp50.close()
    mlp5.close()
    if args.out:
        with open(args.out, "w") as f:
            f.write("\n".join(lines) + "\n")


if __name__ == "__main__":
    sys.exit(main())
