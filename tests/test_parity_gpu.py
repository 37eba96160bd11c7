"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle, element by
element on identical seeded inputs.  Error metric (pass/fail): max_n |gpu_n - ref_n| / max_n |ref_n|.
Bars: fp64 <= 1e-5 (tightened here to 1e-10, the arithmetic allows it), fp32 <= 2e-4.
"""
import ctypes

import numpy as np
import pytest

from paper_2505_13644_amd import synth
from helpers import gpu_run, oracle_run

pytestmark = pytest.mark.gpu

TOL32 = 2e-4
TOL64 = 1e-10


def err(got, ref):
    from oracle.operators import scaled_max_err
    return scaled_max_err(got, ref)


def check(got, ref, tol, what):
    gu, go = got
    ru, ro = ref
    eu, eo = err(gu, ru), err(go, ro)
    print(f"[{what}] scaled max err: u {eu:.3e}  op {eo:.3e}  (tol {tol:g}; max|op| {np.max(np.abs(ro)):.3e})", flush=True)
    assert np.all(np.isfinite(gu)) and np.all(np.isfinite(go))
    assert eu <= tol, f"{what}: u error {eu}"
    assert eo <= tol, f"{what}: op error {eo}"


def tol_of(dtype):
    return TOL64 if dtype == np.float64 else TOL32


# Regression guards: what the arithmetic actually delivers, with a small margin -- far inside the bars above, so that a
# kernel change that loses a decimal digit or two fails here although it would still pass the bar.  fp32 native: one
# rounding per product / accumulate, dot products of at most 768 terms, four layers: observed 1e-6.  Split bf16 keeps
# about 16 bits per operand: observed 1e-5.
GUARD = {"f32": 2e-5, "bf16x3": 1e-4, "bf16": 2e-2}


def check_every_point(got, ref, tol, guard, what):
    """Per-point mixed tolerance and a relative l2 error beside the scaled max-norm: |d_n| <= tol |ref_n| + guard max|ref|
    for every point n (an absolute floor is needed because the operator is a sum of signed terms that can cancel to
    ~0 at a point while the rounding error stays at the scale of the terms), ||d||_2 <= tol ||ref||_2, and the scaled
    max-norm itself inside the guard."""
    for name, g, r in (("u", got[0], ref[0]), ("op", got[1], ref[1])):
        g, r = np.asarray(g, dtype=np.float64), np.asarray(r, dtype=np.float64)
        d = np.abs(g - r)
        scale = np.max(np.abs(r))
        bound = tol * np.abs(r) + guard * scale
        worst = int(np.argmax(d - bound))
        l2 = np.linalg.norm(g - r) / max(np.linalg.norm(r), 1e-300)
        print(f"[{what}] {name}: scaled max {np.max(d) / scale:.3e} (guard {guard:g}), rel l2 {l2:.3e}, "
              f"worst point {worst}: |d| {d[worst]:.3e} vs bound {bound[worst]:.3e}", flush=True)
        assert np.all(d <= bound), f"{what}: {name}[{worst}] off by {d[worst]:.3e}, allowed {bound[worst]:.3e}"
        assert l2 <= tol, f"{what}: relative l2 error of {name} {l2:.3e}"
        assert np.max(d) <= guard * scale, f"{what}: {name} scaled max error {np.max(d) / scale:.3e} above the regression guard {guard:g}"


# ---------------------------------------------------------------------------
# the five named workloads
# ---------------------------------------------------------------------------
def test_c1_exact_laplacian_fp64_full():
    w = synth.WORKLOADS["c1"]
    arrs = w.build()
    print("case c1 N=8 fp64", flush=True)
    got = gpu_run(arrs, w.op)
    check(got, oracle_run(arrs, w.op, mode="hessian"), TOL64, "c1 hessian")
    check(got, oracle_run(arrs, w.op, mode="directional"), TOL64, "c1 directional")
    assert TOL64 <= w.tol


@pytest.mark.parametrize("name,N", [("c2", 37), ("c3", 45), ("c4", 50), ("c5", 23)])
def test_named_workloads_reduced_batch(name, N):
    # same network, directions and dtype as the named workload, batch cut so that the oracle takes
    # seconds; N is chosen to span several tiles and leave a ragged last tile
    w = synth.WORKLOADS[name]
    arrs = w.build(N)
    print(f"case {name} N={N}", flush=True)
    got = gpu_run(arrs, w.op)
    check(got, oracle_run(arrs, w.op), w.tol, f"{name} N={N}")
    if name == "c2":
        idx = [0, 17, 36]
        ref_h = oracle_run(arrs, w.op, idx=idx, mode="hessian")
        check((got[0][idx], got[1][idx]), ref_h, w.tol, "c2 full-Hessian trace")


def test_benchmark_shape_in_fp64_every_point():
    # the benchmark's network, batch and directions with every array widened to fp64: the fp64 kernels at the tile
    # shape and launch size the fp32 benchmark uses (three workgroups per CU, two 32-column chunks per tile).  The
    # oracle widens its inputs to fp64 anyway, so its result for c2 is the reference here too.
    w = synth.WORKLOADS["c2"]
    arrs32 = w.build()
    wide = lambda v: [a.astype(np.float64) for a in v] if isinstance(v, list) else (v.astype(np.float64) if isinstance(v, np.ndarray) else v)
    arrs = {k: wide(v) for k, v in arrs32.items()}
    print(f"case c2 in fp64, full N={w.N}, every point", flush=True)
    got = gpu_run(arrs, w.op)
    ref = full_size_oracle("c2", arrs32)
    check(got, ref, TOL64, "c2 in fp64, full size")
    check_every_point(got, ref, TOL64, TOL64, "c2 in fp64, full size")


@pytest.mark.parametrize("name,n_sample", [("c2", 24), ("c3", 48), ("c4", 64), ("c5", 48), ("e1", 12)])
def test_named_workloads_full_size_sampled(name, n_sample):
    # the launch configuration the benchmark times; the oracle checks a seeded sample of points
    w = synth.WORKLOADS[name]
    arrs = w.build()
    print(f"case {name} full N={w.N}", flush=True)
    gu, go, mlp = gpu_run(arrs, w.op, return_mlp=True)
    idx = np.sort(np.random.default_rng(123).choice(w.N, n_sample, replace=False))
    idx[0], idx[-1] = 0, w.N - 1
    ru, ro = oracle_run(arrs, w.op, idx=idx)
    # the sample's scale stands in for the batch's
    check((gu[idx], go[idx]), (ru, ro), w.tol, f"{name} full-size sample")
    assert np.all(np.isfinite(go)) and np.all(np.isfinite(gu))
    # properties that hold at any size: run-to-run bitwise determinism, and every point's
    # result is independent of the rest of the batch (bitwise, since no row mixes points)
    gu2, go2 = gpu_run(arrs, w.op, mlp=mlp)
    assert np.array_equal(gu, gu2) and np.array_equal(go, go2)
    sub = dict(arrs)
    sub["x"] = arrs["x"][idx]
    if arrs.get("V") is not None and arrs["V"].ndim == 3:
        sub["V"] = arrs["V"][idx]
    su, so = gpu_run(sub, w.op, mlp=mlp)
    assert np.array_equal(su, gu[idx]) and np.array_equal(so, go[idx])
    mlp.close()


_FULL_ORACLE = {}


def full_size_oracle(name, arrs):
    """The oracle on every point of a named workload (directional mode); computed once per test session."""
    if name not in _FULL_ORACLE:
        w = synth.WORKLOADS[name]
        _FULL_ORACLE[name] = oracle_run(arrs, w.op)
    return _FULL_ORACLE[name]


def split_batch(arrs, lo, hi):
    sub = dict(arrs)
    sub["x"] = arrs["x"][lo:hi]
    if arrs.get("V") is not None and arrs["V"].ndim == 3:
        sub["V"] = arrs["V"][lo:hi]
    return sub


@pytest.mark.parametrize("name", ["c2", "c3", "c4", "c5", "e1"])
def test_named_workloads_full_size_every_point(name):
    # the launch configuration the benchmark times, compared with the oracle (directional mode: R second / fourth
    # directional derivatives per point) on EVERY point, and bitwise batch independence for every point: the batch
    # cut at a point that is no multiple of any tile height gives the same bits as the full batch
    w = synth.WORKLOADS[name]
    arrs = w.build()
    print(f"case {name} full N={w.N}, every point", flush=True)
    gu, go, mlp = gpu_run(arrs, w.op, return_mlp=True)
    ru, ro = full_size_oracle(name, arrs)
    check((gu, go), (ru, ro), w.tol, f"{name} full size, all {w.N} points")
    check_every_point((gu, go), (ru, ro), w.tol, GUARD["f32"], f"{name} full size")
    if name == "c2":   # the other oracle mode (full Hessian, then its trace) on three points
        idx = [0, 2049, w.N - 1]
        ref_h = oracle_run(arrs, w.op, idx=idx, mode="hessian")
        assert err(ref_h[1], ro[idx]) <= 1e-10
    cut = w.N // 2 + 3
    parts = [gpu_run(split_batch(arrs, lo, hi), w.op, mlp=mlp) for lo, hi in ((0, cut), (cut, w.N))]
    assert np.array_equal(np.concatenate([p[0] for p in parts]), gu)
    assert np.array_equal(np.concatenate([p[1] for p in parts]), go)
    # a cut that keeps the launch shapes of the full batch (16-point workgroups in the first-layer kernel) and ends in a
    # ragged chunk and a ragged tile
    big = (3 * w.N) // 4 - 71
    pu, po = gpu_run(split_batch(arrs, 0, big), w.op, mlp=mlp)
    assert np.array_equal(pu, gu[:big]) and np.array_equal(po, go[:big])
    mlp.close()


# ---------------------------------------------------------------------------
# bf16 matrix-core variants of the fp32 path (bar for these: 2e-2)
# ---------------------------------------------------------------------------
def mfma_modes():
    import paper_2505_13644_amd as ctm
    # split bf16 (3 MFMAs per product) keeps about 16 bits per operand: held to the fp32 bar as well
    return {"bf16x3": (ctm.CTM_F32_BF16X3, 2e-4), "bf16": (ctm.CTM_F32_BF16, 2e-2)}


@pytest.mark.parametrize("mode", ["bf16x3", "bf16"])
@pytest.mark.parametrize("name,N", [("c2", 37), ("c3", 45), ("c4", 50), ("c5", 23)])
def test_bf16_mfma_variants_reduced_batch(mode, name, N):
    code, tol = mfma_modes()[mode]
    w = synth.WORKLOADS[name]
    arrs = w.build(N)
    print(f"case {name} N={N} {mode}", flush=True)
    check(gpu_run(arrs, w.op, mfma=code), oracle_run(arrs, w.op), tol, f"{name} N={N} {mode}")


@pytest.mark.parametrize("mode", ["bf16x3", "bf16"])
@pytest.mark.parametrize("name", ["c2", "c3", "c4", "c5"])
def test_bf16_mfma_variants_full_size_every_point(mode, name):
    code, tol = mfma_modes()[mode]
    w = synth.WORKLOADS[name]
    arrs = w.build()
    print(f"case {name} full N={w.N} {mode}, every point", flush=True)
    gu, go, mlp = gpu_run(arrs, w.op, return_mlp=True, mfma=code)
    ref = full_size_oracle(name, arrs)
    check((gu, go), ref, tol, f"{name} full size {mode}")
    check_every_point((gu, go), ref, tol, GUARD[mode], f"{name} full size {mode}")
    gu2, go2 = gpu_run(arrs, w.op, mlp=mlp)
    assert np.array_equal(gu, gu2) and np.array_equal(go, go2)
    mlp.close()


@pytest.mark.parametrize("dims,N,R,K", [
    ((6, 256, 448, 1), 4100, 10, 2),     # 12 row blocks (16 points of 12 rows), two column tiles, the second 192 columns wide, ragged batch
    ((5, 64, 256, 1), 1027, 32, 4),      # order 4: two points of 98 rows per tile, two wavefronts per point, last tile one point
    ((9, 256, 480, 224, 1), 2050, 16, 2),  # 9 row blocks; 256 -> 480 takes the 256-column tiles, 480 -> 224 the 128-column ones
])
def test_plain_bf16_256_column_tiles(dims, N, R, K):
    # batches that give every compute unit at least two 256-column tiles take the wide plain-bf16 kernel (every tile height
    # it is built for, both ways of sharing a tile's points among the wavefronts); compared with the oracle on every point
    import paper_2505_13644_amd as ctm
    arrs = small_case(dims, N, np.float32, seed=N, R=R, per_point=True)
    op_name = "laplacian" if K == 2 else "biharmonic_rand"
    print(f"case bf16 256-column tiles dims={dims} N={N} R={R} K={K}", flush=True)
    got = gpu_run(arrs, op_name, mfma=ctm.CTM_F32_BF16)
    ref = oracle_run(arrs, op_name)
    check(got, ref, 2e-2, f"bf16 wide {dims}")
    again = gpu_run(arrs, op_name, mfma=ctm.CTM_F32_BF16)
    assert np.array_equal(got[0], again[0]) and np.array_equal(got[1], again[1])
    # the same points in a batch too small for the wide tiles take the 128-column kernel: same result up to the order of the k sum
    sub = split_batch(arrs, 0, 40)
    small = gpu_run(sub, op_name, mfma=ctm.CTM_F32_BF16)
    scale = max(np.max(np.abs(ref[1])), 1e-30)
    assert np.max(np.abs(small[1] - got[1][:40])) <= 2e-2 * scale


@pytest.mark.parametrize("mode", ["bf16x3", "bf16"])
@pytest.mark.parametrize("dims,N,R,per_point", [((7, 33, 65, 1), 19, None, False), ((3, 100, 1), 130, None, False),
                                                ((4, 48, 48, 48, 1), 33, 21, True), ((6, 24, 16, 1), 21, 300, False)])
def test_bf16_mfma_variants_shapes(mode, dims, N, R, per_point):
    code, tol = mfma_modes()[mode]
    arrs = small_case(dims, N, np.float32, seed=N, R=R, per_point=per_point)
    print(f"case bf16 shapes dims={dims} N={N} R={R} {mode}", flush=True)
    check(gpu_run(arrs, "laplacian", mfma=code), oracle_run(arrs, "laplacian"), tol, f"laplacian {dims} {mode}")
    if R is not None and R <= 60:
        check(gpu_run(arrs, "biharmonic_rand", mfma=code), oracle_run(arrs, "biharmonic_rand"), tol, f"biharmonic {dims} {mode}")


# ---------------------------------------------------------------------------
# shapes that stress tiling: odd widths, one hidden layer, N = 1, R = 1, many directions
# ---------------------------------------------------------------------------
def small_case(dims, N, dtype, seed, R=None, kind="gaussian", per_point=True, bias=0.1):
    Ws, bs = synth.make_mlp(dims, seed, bias, dtype)
    arrs = {"Ws": Ws, "bs": bs, "x": synth.make_points(N, dims[0], seed, dtype)}
    if R is None:
        arrs["V"], arrs["scale"] = None, 1.0
    else:
        shape = (N, R, dims[0]) if per_point else (R, dims[0])
        arrs["V"], arrs["scale"] = synth.make_directions(kind, shape, seed, dtype), 1.0 / R
    return arrs


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("dims,N,R,per_point", [
    ((7, 33, 65, 1), 19, None, False),     # widths that are no multiple of anything
    ((3, 100, 1), 130, None, False),       # one hidden layer
    ((5, 16, 16, 1), 1, None, False),      # a single point
    ((6, 40, 24, 1), 11, 1, True),         # a single direction
    ((6, 40, 24, 1), 70, 9, False),        # shared directions [R, D]
    ((4, 48, 48, 48, 1), 33, 21, True),    # per-point directions
    ((50, 96, 1), 9, 150, False),          # more rows per point than half a tile
    ((50, 160, 96, 1), 41, None, False),   # the benchmark's 52 rows per point: tallest tile, four points each, several column tiles
])
def test_laplacian_shapes(dtype, dims, N, R, per_point):
    arrs = small_case(dims, N, dtype, seed=len(dims) + N, R=R, per_point=per_point)
    print(f"case laplacian dims={dims} N={N} R={R} per_point={per_point} {dtype.__name__}", flush=True)
    check(gpu_run(arrs, "laplacian"), oracle_run(arrs, "laplacian"), tol_of(dtype), f"laplacian {dims}")


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("R", [300, 255, 509])
def test_laplacian_direction_set_split_over_passes(dtype, R):
    # more directions than fit one tile: several passes whose partial sums are added
    dims, N = (6, 24, 16, 1), 21
    arrs = small_case(dims, N, dtype, seed=R, R=R, per_point=False)
    print(f"case multi-pass R={R} {dtype.__name__}", flush=True)
    check(gpu_run(arrs, "laplacian"), oracle_run(arrs, "laplacian"), tol_of(dtype), f"multi-pass R={R}")


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("dims,N,K", [((9, 50, 30, 1), 40, 4), ((50, 64, 64, 1), 17, 50), ((5, 16, 1), 3, 1)])
def test_weighted_laplacian_shapes(dtype, dims, N, K):
    Ws, bs = synth.make_mlp(dims, 3, 0.1, dtype)
    arrs = {"Ws": Ws, "bs": bs, "x": synth.make_points(N, dims[0], 3, dtype), "sigma": synth.make_sigma(dims[0], K, 3, dtype)}
    print(f"case weighted dims={dims} N={N} K={K} {dtype.__name__}", flush=True)
    got = gpu_run(arrs, "weighted_laplacian")
    check(got, oracle_run(arrs, "weighted_laplacian", mode="hessian"), tol_of(dtype), f"weighted {dims} K={K}")


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("dims,N,S,per_point", [
    ((10, 64, 32, 1), 37, 5, True),
    ((3, 20, 1), 9, 1, True),
    ((4, 32, 32, 32, 1), 50, 12, False),
    ((5, 24, 16, 1), 6, 100, False),       # S above the per-tile limit of 84: two passes
])
def test_biharmonic_shapes(dtype, dims, N, S, per_point):
    arrs = small_case(dims, N, dtype, seed=S, R=S, per_point=per_point, bias=0.05)
    print(f"case biharmonic dims={dims} N={N} S={S} {dtype.__name__}", flush=True)
    check(gpu_run(arrs, "biharmonic_rand"), oracle_run(arrs, "biharmonic_rand"), tol_of(dtype), f"biharmonic {dims} S={S}")


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("dims,N,R,per_point", [
    ((5, 16, 16, 1), 8, None, False),       # c1's shape, standard basis
    ((6, 40, 24, 1), 37, 9, False),         # shared directions
    ((4, 48, 48, 48, 1), 33, 21, True),     # per-point directions
    ((3, 100, 1), 20, 5, True),             # one hidden layer
    ((6, 24, 16, 1), 11, 200, False),       # 1 + 2R rows exceed one tile: two passes
])
def test_standard_taylor_mode_equals_collapsed_and_oracle(dtype, dims, N, R, per_point):
    # Sec. 3.1: propagating then summing (1 + K R rows) and propagating the sum (1 + (K-1) R + 1 rows) agree
    arrs = small_case(dims, N, dtype, seed=N + len(dims), R=R, per_point=per_point)
    print(f"case standard taylor dims={dims} N={N} R={R} {dtype.__name__}", flush=True)
    std2 = gpu_run(arrs, "laplacian_standard")
    check(std2, oracle_run(arrs, "laplacian"), tol_of(dtype), f"standard K=2 {dims}")
    col2 = gpu_run(arrs, "laplacian")
    assert err(std2[1], col2[1]) <= (1e-12 if dtype == np.float64 else 2e-5)
    if R is not None and R <= 60:
        std4 = gpu_run(arrs, "biharmonic_rand_standard")
        check(std4, oracle_run(arrs, "biharmonic_rand"), tol_of(dtype), f"standard K=4 {dims}")
        col4 = gpu_run(arrs, "biharmonic_rand")
        assert err(std4[1], col4[1]) <= (1e-12 if dtype == np.float64 else 2e-5)


def test_standard_taylor_mode_many_order4_directions():
    arrs = small_case((5, 24, 16, 1), 6, np.float64, seed=100, R=100, per_point=False, bias=0.05)   # 401 rows: two passes
    check(gpu_run(arrs, "biharmonic_rand_standard"), oracle_run(arrs, "biharmonic_rand"), TOL64, "standard K=4 S=100")


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("sigma_per_point,v_mode", [(False, "shared"), (False, "per_point"), (True, "shared"), (True, "per_point"),
                                                    (True, None), (False, None)])
def test_stochastic_and_point_dependent_weighted_laplacian(dtype, sigma_per_point, v_mode):
    # Eq. 8 stochastic case: directions sigma_n v_{n,s}; v_mode None = exact operator with the columns of sigma_n
    dims, N, K, S = (9, 40, 24, 1), 27, 3, 7
    rng = np.random.default_rng(5)
    arrs = small_case(dims, N, dtype, seed=K)
    arrs["sigma"] = (rng.standard_normal((N, 9, K) if sigma_per_point else (9, K)) / 3).astype(dtype)
    arrs["Vk"] = None if v_mode is None else rng.standard_normal((N, S, K) if v_mode == "per_point" else (S, K)).astype(dtype)
    print(f"case weighted rand sigma_per_point={sigma_per_point} v={v_mode} {dtype.__name__}", flush=True)
    check(gpu_run(arrs, "weighted_laplacian_rand"), oracle_run(arrs, "weighted_laplacian_rand"), tol_of(dtype),
          f"weighted rand {sigma_per_point} {v_mode}")


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("dims,N", [((1, 12, 1), 9), ((2, 16, 16, 1), 21), ((5, 32, 24, 1), 13), ((7, 20, 1), 5)])
def test_exact_biharmonic_by_interpolation(dtype, dims, N):
    # three collapsed 4-jet families combined with gamma_{(2,2),j} (Sec. 3.3, App. E.1) against the full
    # tensor sum_{ij} d^4 u / dx_i^2 dx_j^2 of the oracle; D = 5 is the paper's benchmark dimension
    arrs = small_case(dims, N, dtype, seed=dims[0], bias=0.1)
    print(f"case exact biharmonic dims={dims} N={N} {dtype.__name__}", flush=True)
    check(gpu_run(arrs, "biharmonic_exact"), oracle_run(arrs, "biharmonic_exact"), tol_of(dtype) if dtype == np.float64 else 2e-4,
          f"exact biharmonic {dims}")


def test_exact_biharmonic_many_directions_and_stochastic_estimate():
    # D = 12: the 132-direction family needs two passes; a 4096-sample Gaussian estimate must agree statistically
    dims, N = (12, 24, 1), 4
    arrs = small_case(dims, N, np.float64, seed=12)
    gu, go = gpu_run(arrs, "biharmonic_exact")
    ru, ro = oracle_run(arrs, "biharmonic_exact")
    check((gu, go), (ru, ro), TOL64, "exact biharmonic D=12")
    S = 4096
    V = synth.make_directions("gaussian", (N, S, 12), 1, np.float64)
    _, est = gpu_run(dict(arrs, V=V), "biharmonic_rand")
    from oracle.operators import directional_derivative
    d4 = directional_derivative(arrs["Ws"], arrs["bs"], arrs["x"], V, 4) / 3.0
    np.testing.assert_allclose(est, d4.mean(axis=1), rtol=1e-9, atol=1e-12)
    assert np.all(np.abs(est - go) <= 6 * d4.std(axis=1) / np.sqrt(S))


# ---------------------------------------------------------------------------
# properties and special cases
# ---------------------------------------------------------------------------
def test_one_hidden_layer_closed_form_on_gpu():
    # u = sum_j a_j tanh(w_j.x + b_j) + c  =>  Lap u = sum_j a_j |w_j|^2 tanh''(z_j),
    # <d^4 u, v^4> = sum_j a_j (w_j.v)^4 tanh''''(z_j)   (special case of the App. H scheme)
    dims, N, S = (6, 40, 1), 25, 3
    arrs = small_case(dims, N, np.float64, 77, R=S, per_point=True)
    W1, a = arrs["Ws"]
    b1, c = arrs["bs"]
    x, V = arrs["x"], arrs["V"]
    z = x @ W1.T + b1
    t = np.tanh(z)
    s = 1 - t * t
    d2, d4 = -2 * t * s, 16 * t * s * s - 8 * t ** 3 * s
    lap = dict(arrs, V=None, scale=1.0)
    gu, go = gpu_run(lap, "laplacian")
    np.testing.assert_allclose(gu, t @ a[0] + c[0], rtol=1e-12)
    np.testing.assert_allclose(go, (d2 * (W1 ** 2).sum(1)) @ a[0], rtol=1e-10, atol=1e-13)
    _, gb = gpu_run(arrs, "biharmonic_rand")
    wv = np.einsum("id,nsd->nsi", W1, V)
    np.testing.assert_allclose(gb, np.einsum("nsi,ni,i->n", wv ** 4, d4, a[0]) / (3 * S), rtol=1e-10, atol=1e-13)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_identity_activation_gives_exactly_zero(dtype):
    import paper_2505_13644_amd as ctm
    arrs = small_case((5, 16, 16, 1), 13, dtype, 5, R=4, per_point=True)
    gu, go = gpu_run(arrs, "laplacian", act=ctm.CTM_ACT_IDENTITY)
    ru, ro = oracle_run(arrs, "laplacian", act="identity")
    assert np.all(go == 0.0) and np.all(ro == 0.0)
    assert err(gu, ru) <= (1e-12 if dtype == np.float64 else 1e-5)
    _, gb = gpu_run(arrs, "biharmonic_rand", act=ctm.CTM_ACT_IDENTITY)
    assert np.all(gb == 0.0)


def test_collapsed_sum_equals_sum_of_single_direction_calls():
    # Sec. 3.1: propagating the sum equals summing R separately propagated jets
    arrs = small_case((6, 32, 32, 1), 20, np.float64, 9, R=5, per_point=True)
    _, full = gpu_run(dict(arrs, scale=1.0), "laplacian")
    parts = sum(gpu_run(dict(arrs, V=np.ascontiguousarray(arrs["V"][:, r:r + 1]), scale=1.0), "laplacian")[1] for r in range(5))
    np.testing.assert_allclose(full, parts, rtol=1e-11, atol=1e-13)
    _, full4 = gpu_run(arrs, "biharmonic_rand")
    parts4 = sum(gpu_run(dict(arrs, V=np.ascontiguousarray(arrs["V"][:, r:r + 1])), "biharmonic_rand")[1] for r in range(5)) / 5
    np.testing.assert_allclose(full4, parts4, rtol=1e-10, atol=1e-13)


def test_basis_and_sigma_special_cases_agree():
    dims, N = (8, 40, 24, 1), 15
    arrs = small_case(dims, N, np.float64, 4)
    _, exact = gpu_run(arrs, "laplacian")
    eye = np.eye(8)
    _, via_v = gpu_run(dict(arrs, V=eye, scale=1.0), "laplacian")
    _, via_sigma = gpu_run(dict(arrs, sigma=eye), "weighted_laplacian")
    Q, _ = np.linalg.qr(np.random.default_rng(0).standard_normal((8, 8)))
    _, rotated = gpu_run(dict(arrs, V=np.ascontiguousarray(Q.T), scale=1.0), "laplacian")
    np.testing.assert_array_equal(exact, via_v)
    np.testing.assert_array_equal(exact, via_sigma)
    np.testing.assert_allclose(rotated, exact, rtol=1e-10, atol=1e-12)


def test_errors_from_the_library_with_a_live_handle():
    import torch
    import paper_2505_13644_amd as ctm
    from paper_2505_13644_amd import binding as B
    arrs = small_case((5, 16, 16, 1), 8, np.float32, 1)
    dev = torch.device("cuda:0")
    mlp = ctm.ctm_create_mlp([torch.from_numpy(W).to(dev) for W in arrs["Ws"]], None)
    x = torch.from_numpy(arrs["x"]).to(dev)
    u = torch.empty(8, device=dev)
    need = ctm.ctm_workspace_bytes(mlp, 2, 8, 5)
    ws = torch.empty(need + 256, dtype=torch.uint8, device=dev)
    L = B.lib()
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    assert L.ctm_laplacian(mlp.handle, p(x), 8, None, 4, 0, 1.0, p(u), p(u), p(ws), need, st) == -2   # basis needs R = D
    assert L.ctm_laplacian(mlp.handle, p(x), 8, p(x), 5, 7, 1.0, p(u), p(u), p(ws), need, st) == -2   # bad stride
    assert L.ctm_laplacian(mlp.handle, p(x), 0, None, 5, 0, 1.0, p(u), p(u), p(ws), need, st) == -2
    assert L.ctm_laplacian(mlp.handle, p(x), 8, None, 5, 0, 1.0, p(u), p(u), p(ws), need - 1, st) == -5
    assert "workspace" in ctm.ctm_last_error()
    assert L.ctm_laplacian(mlp.handle, p(x), 8, None, 5, 0, 1.0, p(u), p(u), ctypes.c_void_p(ws.data_ptr() + 4), need, st) == -6
    assert L.ctm_laplacian(mlp.handle, None, 8, None, 5, 0, 1.0, p(u), p(u), p(ws), need, st) == -1
    assert L.ctm_biharmonic_rand(mlp.handle, p(x), 8, None, 5, 0, p(u), p(u), p(ws), need, st) == -1
    assert L.ctm_weighted_laplacian(mlp.handle, p(x), 8, None, 5, p(u), p(u), p(ws), need, st) == -1
    # u or op may be left out
    op = torch.full((8,), 7.0, device=dev)
    assert L.ctm_laplacian(mlp.handle, p(x), 8, None, 5, 0, 1.0, None, p(op), p(ws), need, st) == 0
    torch.cuda.synchronize()
    ref = oracle_run({"Ws": arrs["Ws"], "bs": [np.zeros_like(b) for b in arrs["bs"]], "x": arrs["x"], "V": None}, "laplacian")
    assert err(op.double().cpu().numpy(), ref[1]) <= TOL32
    with pytest.raises(ValueError):
        ctm.ctm_laplacian(mlp, x[:, :4].contiguous())
    # recording forward / reverse pass: tape and workspace sizes, direction limits, missing directions
    V = torch.randn(8, 3, 5, device=dev)
    tape = torch.empty(ctm.ctm_biharmonic_tape_bytes(mlp, 8, 3), dtype=torch.uint8, device=dev)
    assert L.ctm_biharmonic_rand_fwd(mlp.handle, p(x), 8, p(V), 3, 15, p(u), p(op), p(tape), tape.numel() - 1, st) == -5
    assert L.ctm_biharmonic_rand_fwd(mlp.handle, p(x), 8, None, 3, 15, p(u), p(op), p(tape), tape.numel(), st) == -1
    assert L.ctm_biharmonic_rand_fwd(mlp.handle, p(x), 8, p(V), 3, 14, p(u), p(op), p(tape), tape.numel(), st) == -2
    # 85 directions take two passes and two tapes: the tape of a 3-direction call is too small for them
    assert L.ctm_biharmonic_rand_fwd(mlp.handle, p(x), 8, p(V), 85, 85 * 5, p(u), p(op), p(tape), tape.numel(), st) == -5
    assert L.ctm_biharmonic_rand_fwd(mlp.handle, p(x), 8, p(V), 3, 15, p(u), p(op), p(tape), tape.numel(), st) == 0
    bws = torch.empty(ctm.ctm_biharmonic_backward_workspace_bytes(mlp, 8, 3), dtype=torch.uint8, device=dev)
    assert L.ctm_biharmonic_rand_bwd(mlp.handle, 8, 3, p(tape), tape.numel(), p(u), p(op), None, None, p(bws), bws.numel() - 1, st) == -5
    assert L.ctm_biharmonic_rand_bwd(mlp.handle, 8, 3, p(tape), tape.numel() - 1, p(u), p(op), None, None, p(bws), bws.numel(), st) == -5
    assert L.ctm_biharmonic_rand_bwd(mlp.handle, 8, 3, p(tape), tape.numel(), p(u), p(op), None, None, p(bws), bws.numel(), st) == 0  # no gradient wanted
    assert L.ctm_laplacian_fwd(mlp.handle, p(x), 8, None, 5, 0, 1.0, p(u), p(op), p(tape), 16, st) == -5
    assert L.ctm_laplacian_fwd(mlp.handle, p(x), 8, None, 300, 0, 1.0, p(u), p(op), p(tape), tape.numel(), st) == -2   # basis needs R = D
    torch.cuda.synchronize()
    # the bf16 variants have no recording forward
    m16 = ctm.ctm_create_mlp([torch.from_numpy(W).to(dev) for W in arrs["Ws"]], None, mfma=ctm.CTM_F32_BF16X3)
    assert L.ctm_tape_bytes(m16.handle, 8, 5) == 0 and "CTM_F32 and CTM_F64" in ctm.ctm_last_error()
    m16.close()
    mlp.close()


def test_operator_call_can_be_captured_in_a_hip_graph_and_replayed():
    # serving loops replay captured graphs: the calls launch kernels only (no allocation, no sync, no memset node)
    import torch
    import paper_2505_13644_amd as ctm
    w = synth.WORKLOADS["c3"]
    N = 64
    arrs = w.build(N)
    dev = torch.device("cuda:0")
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    mlp = ctm.ctm_create_mlp([t(W) for W in arrs["Ws"]], [t(b) for b in arrs["bs"]])
    x, V = t(arrs["x"]), t(arrs["V"])
    u, op = torch.empty(N, device=dev), torch.empty(N, device=dev)
    ws = torch.empty(ctm.ctm_workspace_bytes(mlp, 2, N, w.R), dtype=torch.uint8, device=dev)
    ctm.ctm_laplacian(mlp, x, V, arrs["scale"], u, op, ws)          # warm-up outside the capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        ctm.ctm_laplacian(mlp, x, V, arrs["scale"], u, op, ws)
    for rep in range(4):
        xr = synth.make_points(N, 50, seed=100 + rep)
        x.copy_(t(xr))
        u.zero_(); op.zero_()
        g.replay()
        torch.cuda.synchronize()
        gu, go = u.cpu().numpy().copy(), op.cpu().numpy().copy()
        eu, eo = ctm.ctm_laplacian(mlp, x, V, arrs["scale"])          # eager, fresh outputs and workspace
        torch.cuda.synchronize()
        assert np.array_equal(gu, eu.cpu().numpy()) and np.array_equal(go, eo.cpu().numpy()), f"replay {rep}"
        assert np.any(go != 0)
    del g
    mlp.close()


def test_concurrent_calls_on_two_streams_with_their_own_workspaces():
    # a handle is read-only in operator calls: calls that overlap on two streams with distinct workspaces and outputs
    # must give the results of the same calls made one after the other
    import torch
    import paper_2505_13644_amd as ctm
    dev = torch.device("cuda:0")
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    w = synth.WORKLOADS["c3"]
    arrs = w.build(1500)
    mlp = ctm.ctm_create_mlp([t(W) for W in arrs["Ws"]], [t(b) for b in arrs["bs"]])
    halves = [split_batch(arrs, 0, 700), split_batch(arrs, 700, 1500)]
    xs = [t(h["x"]) for h in halves]
    Vs = [t(h["V"]) for h in halves]
    ref = [ctm.ctm_laplacian(mlp, x, V, arrs["scale"]) for x, V in zip(xs, Vs)]
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    outs = [(torch.empty_like(r[0]), torch.empty_like(r[1])) for r in ref]
    wss = [torch.empty(ctm.ctm_workspace_bytes(mlp, 2, x.shape[0], w.R), dtype=torch.uint8, device=dev) for x in xs]
    print("case two streams, N=700 and N=800", flush=True)
    for rep in range(3):
        for i in (0, 1):
            with torch.cuda.stream(streams[i]):
                ctm.ctm_laplacian(mlp, xs[i], Vs[i], arrs["scale"], outs[i][0], outs[i][1], wss[i])
    torch.cuda.synchronize()
    for i in (0, 1):
        assert torch.equal(outs[i][0], ref[i][0]) and torch.equal(outs[i][1], ref[i][1])
    mlp.close()


@pytest.mark.parametrize("op_name,N", [("laplacian", 37), ("biharmonic_rand", 23), ("biharmonic_exact", 9)])
def test_calls_stay_inside_their_buffers(op_name, N):
    # guard words before and after u, op and the workspace must survive a call untouched
    import torch
    import paper_2505_13644_amd as ctm
    dims = (6, 40, 24, 1)
    arrs = small_case(dims, N, np.float32, seed=N, R=5, per_point=True)
    dev = torch.device("cuda:0")
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    mlp = ctm.ctm_create_mlp([t(W) for W in arrs["Ws"]], [t(b) for b in arrs["bs"]])
    x, V = t(arrs["x"]), t(arrs["V"])
    G = 64                                           # guard elements
    ubuf = torch.full((N + 2 * G,), 7.25, device=dev)
    obuf = torch.full((N + 2 * G,), -3.5, device=dev)
    if op_name == "laplacian":
        need = ctm.ctm_workspace_bytes(mlp, 2, N, 5)
    elif op_name == "biharmonic_rand":
        need = ctm.ctm_workspace_bytes(mlp, 4, N, 5)
    else:
        need = ctm.binding.lib().ctm_biharmonic_exact_workspace_bytes(mlp.handle, N)
    wbuf = torch.full((need + 512,), 0x5A, dtype=torch.uint8, device=dev)
    off = (-wbuf.data_ptr()) % 256 + 256             # 256-byte aligned start with at least 256 guard bytes in front
    ws = wbuf[off:off + need]
    u, op = ubuf[G:G + N], obuf[G:G + N]
    if op_name == "laplacian":
        ctm.ctm_laplacian(mlp, x, V, 0.2, u, op, ws)
    elif op_name == "biharmonic_rand":
        ctm.ctm_biharmonic_rand(mlp, x, V, u, op, ws)
    else:
        ctm.ctm_biharmonic_exact(mlp, x, u, op, ws)
    torch.cuda.synchronize()
    assert torch.all(ubuf[:G] == 7.25) and torch.all(ubuf[G + N:] == 7.25)
    assert torch.all(obuf[:G] == -3.5) and torch.all(obuf[G + N:] == -3.5)
    assert torch.all(wbuf[:off] == 0x5A) and torch.all(wbuf[off + need:] == 0x5A)
    assert torch.all(torch.isfinite(u)) and torch.all(torch.isfinite(op)) and not torch.any(u == 7.25)
    mlp.close()


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("dims,N,R,per_point", [((5, 24, 24, 1), 19, None, False), ((6, 40, 1), 33, 4, True), ((4, 32, 32, 32, 1), 9, 6, False)])
def test_sin_activation_all_operators(dtype, dims, N, R, per_point):
    # the paper's graph-rewrite appendix uses sin as its elementwise example; same operators, sin networks
    import paper_2505_13644_amd as ctm
    arrs = small_case(dims, N, dtype, seed=N, R=R, per_point=per_point)
    tol = tol_of(dtype)
    print(f"case sin dims={dims} N={N} R={R} {dtype.__name__}", flush=True)
    check(gpu_run(arrs, "laplacian", act=ctm.CTM_ACT_SIN), oracle_run(arrs, "laplacian", act="sin"), tol, f"sin laplacian {dims}")
    check(gpu_run(arrs, "laplacian_standard", act=ctm.CTM_ACT_SIN), oracle_run(arrs, "laplacian", act="sin"), tol, f"sin standard {dims}")
    if R is not None:
        check(gpu_run(arrs, "biharmonic_rand", act=ctm.CTM_ACT_SIN), oracle_run(arrs, "biharmonic_rand", act="sin"), tol, f"sin biharmonic {dims}")
    else:
        check(gpu_run(arrs, "biharmonic_exact", act=ctm.CTM_ACT_SIN), oracle_run(arrs, "biharmonic_exact", act="sin"),
              tol if dtype == np.float64 else 2e-4, f"sin exact biharmonic {dims}")


def test_sin_network_closed_form():
    # u = sum_j a_j sin(w_j.x + b_j):  Lap u = -sum_j a_j |w_j|^2 sin(z_j),  Lap^2 u = sum_j a_j |w_j|^4 sin(z_j)
    import paper_2505_13644_amd as ctm
    arrs = small_case((4, 30, 1), 12, np.float64, 8)
    W1, a = arrs["Ws"]
    b1, c = arrs["bs"]
    z = arrs["x"] @ W1.T + b1
    n2 = (W1 ** 2).sum(1)
    gu, gl = gpu_run(arrs, "laplacian", act=ctm.CTM_ACT_SIN)
    np.testing.assert_allclose(gu, np.sin(z) @ a[0] + c[0], rtol=1e-12)
    np.testing.assert_allclose(gl, -(np.sin(z) * n2) @ a[0], rtol=1e-10, atol=1e-13)
    _, gb = gpu_run(arrs, "biharmonic_exact", act=ctm.CTM_ACT_SIN)
    np.testing.assert_allclose(gb, (np.sin(z) * n2 ** 2) @ a[0], rtol=1e-9, atol=1e-12)


def test_coefficient_blocks_beyond_two_to_the_31_elements():
    # Maximum sizes: N * rho * ld exceeds 2^31 elements, so every kernel's indexing must be 64-bit.  A small network
    # keeps the arithmetic negligible; inputs are drawn on the device from a seeded generator, a sample of points
    # (first, last and spread) is checked against the oracle, and a sub-batch must reproduce its points bit for bit.
    import torch
    import paper_2505_13644_amd as ctm
    from oracle import operators as orc
    dev = torch.device("cuda:0")
    dims = (5, 16, 16, 1)
    Ws, bs = synth.make_mlp(dims, 3, 0.1, np.float32)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    mlp = ctm.ctm_create_mlp([t(W) for W in Ws], [t(b) for b in bs])
    g = torch.Generator(device=dev)
    g.manual_seed(7)
    for R, N in ((None, 9_700_000), (2, 16_900_000)):
        rho = 2 + (5 if R is None else R)
        assert N * rho * 32 > 2 ** 31
        print(f"case huge batch N={N} rho={rho}", flush=True)
        x = torch.rand(N, 5, generator=g, device=dev)
        V = None if R is None else torch.randn(N, R, 5, generator=g, device=dev)
        u, op = ctm.ctm_laplacian(mlp, x, V, 0.5)
        idx = np.unique(np.concatenate([np.arange(4), np.arange(N - 4, N), np.linspace(0, N - 1, 40).astype(np.int64)]))
        ti = torch.from_numpy(idx).to(dev)
        xs = x[ti].cpu().numpy()
        Vs = None if V is None else V[ti].cpu().numpy()
        ru, rop = orc.laplacian(Ws, bs, xs, Vs, 0.5)
        eu, eo = orc.scaled_max_err(u[ti].cpu().numpy(), ru), orc.scaled_max_err(op[ti].cpu().numpy(), rop)
        print(f"  sampled errors: u {eu:.2e} op {eo:.2e}", flush=True)
        assert eu <= 2e-4 and eo <= 2e-4
        tail = slice(N - 1000, N)
        u2, op2 = ctm.ctm_laplacian(mlp, x[tail].contiguous(), None if V is None else V[tail].contiguous(), 0.5)
        assert torch.equal(u2, u[tail]) and torch.equal(op2, op[tail])
        del x, V, u, op
        torch.cuda.empty_cache()
    mlp.close()


@pytest.mark.parametrize("op_name", ["laplacian", "biharmonic_rand"])
def test_results_do_not_depend_on_the_tile_shape(op_name):
    # rho = 62 rows per point: a large batch runs tiles of 4 points (a wavefront per point in the rule), a small one
    # tiles of 1 point whose directions are shared out over 4 wavefronts.  The direction sum is grouped the same
    # way in both, so a point's result is the same bit pattern in either batch.
    import torch
    import paper_2505_13644_amd as ctm
    from oracle import operators as orc
    dev = torch.device("cuda:0")
    D = 60 if op_name == "laplacian" else 6
    dims = (D, 128, 128, 1)
    Ws, bs = synth.make_mlp(dims, 4, 0.1, np.float32)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    mlp = ctm.ctm_create_mlp([t(W) for W in Ws], [t(b) for b in bs])
    N = 4096
    x = synth.make_points(N, D, 4, np.float32)
    if op_name == "laplacian":
        V = None
        call = lambda xs, Vs: ctm.ctm_laplacian(mlp, xs, None)
    else:
        V = synth.make_directions("gaussian", (N, 20, D), 4, np.float32)   # 2 + 3 * 20 = 62 rows
        call = lambda xs, Vs: ctm.ctm_biharmonic_rand(mlp, xs, Vs)
    xt, Vt = t(x), None if V is None else t(V)
    u, op = call(xt, Vt)
    for n_small in (1, 64, 700):
        u2, op2 = call(xt[:n_small].contiguous(), None if Vt is None else Vt[:n_small].contiguous())
        assert torch.equal(u2, u[:n_small]) and torch.equal(op2, op[:n_small]), n_small
    idx = np.arange(0, N, 173)
    if op_name == "laplacian":
        ru, rop = orc.laplacian(Ws, bs, x[idx], None, 1.0, mode="directional")
    else:
        ru, rop = orc.biharmonic_rand(Ws, bs, x[idx], V[idx])
    assert orc.scaled_max_err(u.cpu().numpy()[idx], ru) <= 2e-4
    assert orc.scaled_max_err(op.cpu().numpy()[idx], rop) <= 2e-4
    mlp.close()


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("dims,N,R,per_point,K", [
    ((5, 16, 16, 1), 8, None, False, 2),       # c1: 56 rows
    ((5, 16, 16, 1), 36, None, False, 2),      # 252 rows: the largest batch of that network on the one-launch path
    ((7, 33, 20, 3), 12, 6, True, 2),          # odd widths, three outputs, per-point directions
    ((4, 24, 24, 24, 1), 9, 5, False, 4),      # order 4, shared directions, 17 rows per point
    ((3, 40, 1), 30, 2, True, 4),              # one hidden layer, order 4
])
def test_one_launch_path_agrees_with_the_tiled_path(dtype, dims, N, R, per_point, K):
    # calls of at most 256 coefficient rows run in one workgroup with the coefficients resident in LDS; the same points
    # inside a batch too large for that take the tiled kernels: both must match the oracle, and each other to rounding
    # (they sum the dot products in different orders)
    import torch
    import paper_2505_13644_amd as ctm
    tol = tol_of(dtype)
    big = 300
    arrs = small_case(dims, big, dtype, seed=N + K, R=R, per_point=per_point)
    op_name = "laplacian" if K == 2 else "biharmonic_rand"
    rho = ctm.ctm_rows_per_point(K, dims[0] if R is None else R)
    assert N * rho <= 256 < big * rho
    sub = split_batch(arrs, 0, N)
    print(f"case one-launch dims={dims} N={N} R={R} K={K} {np.dtype(dtype).name}", flush=True)
    if dims[-1] == 1:
        ref = oracle_run(sub, op_name)
    else:
        from oracle import operators as orc
        fn = orc.laplacian if K == 2 else orc.biharmonic_rand
        args = (sub["x"], sub["V"], sub["scale"]) if K == 2 else (sub["x"], sub["V"])
        ref = orc.per_output(fn, sub["Ws"], sub["bs"], *args)
    small = gpu_run(sub, op_name)
    tiled = gpu_run(arrs, op_name)
    check(small, ref, tol, "one launch")
    check((tiled[0][:N], tiled[1][:N]), ref, tol, "tiled")
    close = 1e-12 if dtype == np.float64 else 2e-5
    assert err(small[0], tiled[0][:N]) <= close and err(small[1], tiled[1][:N]) <= close
    again = gpu_run(sub, op_name)
    assert np.array_equal(small[0], again[0]) and np.array_equal(small[1], again[1])


@pytest.mark.parametrize("gain", [4.0, 8.0])
def test_saturating_activations_stay_inside_the_fp32_bar(gain):
    # weights scaled up and points spread over [-2, 2): most tanh units saturate, so 1 - t^2 is a difference of nearly
    # equal numbers and the operator values grow by orders of magnitude; the scaled max-norm error must still hold
    import torch
    import paper_2505_13644_amd as ctm
    from oracle import operators as orc
    dev = torch.device("cuda:0")
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    dims = (10, 128, 128, 128, 1)
    Ws, bs = synth.make_mlp(dims, 0, 0.1, np.float32)
    Ws = [(W * gain).astype(np.float32) for W in Ws[:-1]] + [Ws[-1]]
    x = (synth.make_points(120, 10, 0, np.float32) * 4 - 2).astype(np.float32)
    V = synth.make_directions("gaussian", (120, 6, 10), 0, np.float32)
    mlp = ctm.ctm_create_mlp([t(W) for W in Ws], [t(b) for b in bs])
    u, op = ctm.ctm_laplacian(mlp, t(x))
    u4, op4 = ctm.ctm_biharmonic_rand(mlp, t(x), t(V))
    ru, rop = orc.laplacian(Ws, bs, x, None, 1.0, mode="directional")
    _, rop4 = orc.biharmonic_rand(Ws, bs, x, V)
    errs = (err(u.cpu().numpy(), ru), err(op.cpu().numpy(), rop), err(op4.cpu().numpy(), rop4))
    print(f"case saturation gain={gain}: u {errs[0]:.2e} laplacian {errs[1]:.2e} biharmonic {errs[2]:.2e}", flush=True)
    assert max(errs) <= TOL32
    mlp.close()


@pytest.mark.parametrize("dims,N", [((3, 4096, 2048, 1), 24), ((4,) + (32,) * 18 + (1,), 50), ((64, 96, 1), 40), ((65, 96, 80, 1), 33)])
def test_very_wide_very_deep_and_wide_input_networks(dims, N):
    # 32 column tiles in one layer; 19 linear layers; an input as wide as the register-resident first layer takes (64)
    # and one just beyond it (65: seed block + stacked GEMM for the first layer even with shared directions)
    arrs = small_case(dims, N, np.float32, 3)
    print(f"case network shape dims={dims[:3]}..x{len(dims) - 1} N={N}", flush=True)
    u, op = gpu_run(arrs, "laplacian")
    ru, rop = oracle_run(arrs, "laplacian")
    eu, eo = err(u, ru), err(op, rop)
    print(f"  u {eu:.2e} op {eo:.2e}", flush=True)
    assert eu <= TOL32 and eo <= TOL32
