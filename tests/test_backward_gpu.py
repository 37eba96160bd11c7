"""GPU parity of the reverse pass: dL/dW_l and dL/db_l of L = sum_n gu_n u_n + gop_n op_n from the HIP path against
the nested-autograd fp64 oracle, on identical seeded inputs.  Metric: per tensor, max |got - ref| / max |ref|."""
import numpy as np
import pytest

from paper_2505_13644_amd import synth

pytestmark = pytest.mark.gpu


def run_gpu(arrs, scale, gu, gop, dtype):
    import torch
    import paper_2505_13644_amd as ctm
    dev = torch.device("cuda:0")
    t = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    mlp = ctm.ctm_create_mlp([t(W) for W in arrs["Ws"]], [t(b) for b in arrs["bs"]])
    x, V = t(arrs["x"]), t(arrs.get("V"))
    N = x.shape[0]
    R = x.shape[1] if V is None else V.shape[-2]
    u, op, tape = ctm.ctm_laplacian_fwd(mlp, x, V, scale)
    u2, op2 = ctm.ctm_laplacian(mlp, x, V, scale)
    gW, gb = ctm.ctm_laplacian_bwd(mlp, N, R, scale, tape, t(gu.astype(dtype)), t(gop.astype(dtype)))
    torch.cuda.synchronize()
    # the plain call takes the GEMM-free first layer for shared directions, so the two differ by rounding only
    tol = 1e-12 if dtype == np.float64 else 2e-5
    den_u, den_o = u2.abs().max().item(), op2.abs().max().item()
    same = (u - u2).abs().max().item() <= tol * den_u and (op - op2).abs().max().item() <= tol * den_o
    out = ([g.double().cpu().numpy() for g in gW], [g.double().cpu().numpy() for g in gb], same)
    mlp.close()
    return out


def rel(got, ref):
    den = np.max(np.abs(ref))
    return np.max(np.abs(got - ref)) / (den if den > 0 else 1.0)


def case(dims, N, dtype, seed, R, per_point, bias=0.1):
    Ws, bs = synth.make_mlp(dims, seed, bias, dtype)
    arrs = {"Ws": Ws, "bs": bs, "x": synth.make_points(N, dims[0], seed, dtype)}
    arrs["V"] = None if R is None else synth.make_directions("gaussian", (N, R, dims[0]) if per_point else (R, dims[0]), seed, dtype)
    return arrs


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("dims,N,R,per_point", [
    ((5, 16, 16, 1), 8, None, False),        # c1's network
    ((6, 40, 24, 1), 37, 9, False),          # shared directions, ragged tiles
    ((4, 48, 48, 48, 1), 33, 7, True),       # three hidden layers, per-point directions
    ((3, 100, 1), 130, None, False),         # one hidden layer
    ((7, 33, 65, 1), 19, 3, True),           # odd widths
    ((50, 160, 144, 1), 300, None, False),   # widths over one 128-column tile, many row ranges in the weight gradient
])
def test_weight_gradients_against_the_autograd_oracle(dtype, dims, N, R, per_point):
    from oracle import gradients as og
    arrs = case(dims, N, dtype, seed=N + len(dims), R=R, per_point=per_point)
    rng = np.random.default_rng(N)
    gu, gop = rng.standard_normal(N), rng.standard_normal(N)
    scale = 0.37
    print(f"case backward dims={dims} N={N} R={R} {dtype.__name__}", flush=True)
    gW, gb, same = run_gpu(arrs, scale, gu, gop, dtype)
    assert same, "the recording forward must agree with ctm_laplacian"
    _, rW, rb = og.laplacian_loss_grads(arrs["Ws"], arrs["bs"], arrs["x"], arrs["V"], scale,
                                        gu.astype(dtype).astype(np.float64), gop.astype(dtype).astype(np.float64))
    tol = 1e-9 if dtype == np.float64 else 2e-4
    for l in range(len(dims) - 1):
        eW, eb = rel(gW[l], rW[l]), rel(gb[l], rb[l])
        print(f"  layer {l}: dW err {eW:.2e}  db err {eb:.2e}", flush=True)
        assert eW <= tol and eb <= tol, (l, eW, eb)


def test_backward_on_the_benchmark_network_and_determinism():
    from oracle import gradients as og
    w = synth.WORKLOADS["c2"]
    N = 24
    arrs = w.build(N)
    rng = np.random.default_rng(3)
    gu, gop = rng.standard_normal(N), rng.standard_normal(N)
    gW, gb, same = run_gpu(arrs, 1.0, gu, gop, np.float32)
    gW2, gb2, _ = run_gpu(arrs, 1.0, gu, gop, np.float32)
    assert same
    for a, b in zip(gW + gb, gW2 + gb2):
        assert np.array_equal(a, b)
    _, rW, rb = og.laplacian_loss_grads(arrs["Ws"], arrs["bs"], arrs["x"], None, 1.0, gu.astype(np.float32).astype(np.float64),
                                        gop.astype(np.float32).astype(np.float64))
    for l in range(5):
        eW, eb = rel(gW[l], rW[l]), rel(gb[l], rb[l])
        print(f"  c2 net layer {l}: dW err {eW:.2e}  db err {eb:.2e}", flush=True)
        assert eW <= 2e-4 and eb <= 2e-4


def test_only_some_gradients_and_missing_cotangents():
    import torch
    import paper_2505_13644_amd as ctm
    from oracle import gradients as og
    arrs = case((6, 40, 24, 1), 21, np.float64, 5, 4, True)
    dev = torch.device("cuda:0")
    t = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    mlp = ctm.ctm_create_mlp([t(W) for W in arrs["Ws"]], [t(b) for b in arrs["bs"]])
    x, V = t(arrs["x"]), t(arrs["V"])
    u, op, tape = ctm.ctm_laplacian_fwd(mlp, x, V, 0.25)
    gop = np.random.default_rng(1).standard_normal(21)
    gW = [None, torch.full((24, 40), 9.0, dtype=torch.float64, device=dev), None]
    gb = [torch.full((40,), 9.0, dtype=torch.float64, device=dev), None, None]
    ctm.ctm_laplacian_bwd(mlp, 21, 4, 0.25, tape, None, t(gop), gW, gb)       # gu = NULL: zeros
    torch.cuda.synchronize()
    _, rW, rb = og.laplacian_loss_grads(arrs["Ws"], arrs["bs"], arrs["x"], arrs["V"], 0.25, np.zeros(21), gop)
    assert rel(gW[1].cpu().numpy(), rW[1]) <= 1e-9 and rel(gb[0].cpu().numpy(), rb[0]) <= 1e-9
    # new weights through ctm_update_mlp give the gradients of the new network
    Ws2, bs2 = synth.make_mlp((6, 40, 24, 1), 77, 0.1, np.float64)
    ctm.ctm_update_mlp(mlp, [t(W) for W in Ws2], [t(b) for b in bs2])
    u, op, tape = ctm.ctm_laplacian_fwd(mlp, x, V, 0.25)
    gWn, gbn = ctm.ctm_laplacian_bwd(mlp, 21, 4, 0.25, tape, None, t(gop))
    torch.cuda.synchronize()
    _, rW2, rb2 = og.laplacian_loss_grads(Ws2, bs2, arrs["x"], arrs["V"], 0.25, np.zeros(21), gop)
    for l in range(3):
        assert rel(gWn[l].cpu().numpy(), rW2[l]) <= 1e-9 and rel(gbn[l].cpu().numpy(), rb2[l]) <= 1e-9
    # ... and so does every copy of the weights the handle keeps: the plain forward with shared directions reads a
    # transposed copy of the first layer's
    from oracle import operators as orc
    xx = np.random.default_rng(5).random((64, 6))           # 512 coefficient rows: the tiled path, not the one-launch one
    gu, gl = ctm.ctm_laplacian(mlp, t(xx))                  # standard basis
    ru, rl = orc.laplacian(Ws2, bs2, xx)
    torch.cuda.synchronize()
    assert orc.scaled_max_err(gu.cpu().numpy(), ru) <= 1e-10 and orc.scaled_max_err(gl.cpu().numpy(), rl) <= 1e-10
    mlp.close()


def test_backward_refuses_a_tape_recorded_before_a_weight_update():
    # the reverse pass reads the weights from the handle: after ctm_update_mlp an older tape must be refused, not
    # silently differentiated against the new weights; two forwards on unchanged weights keep both tapes valid
    import torch
    import paper_2505_13644_amd as ctm
    from paper_2505_13644_amd.autograd import laplacian
    from oracle import gradients as og
    arrs = case((6, 40, 24, 1), 21, np.float64, 5, 4, True)
    dev = torch.device("cuda:0")
    t = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    mlp = ctm.ctm_create_mlp([t(W) for W in arrs["Ws"]], [t(b) for b in arrs["bs"]])
    x, V = t(arrs["x"]), t(arrs["V"])
    gop = t(np.random.default_rng(1).standard_normal(21))
    _, _, tape_a = ctm.ctm_laplacian_fwd(mlp, x, V, 0.25)
    _, _, tape_b = ctm.ctm_laplacian_fwd(mlp, x[:9].contiguous(), V[:9].contiguous(), 0.25)
    ctm.ctm_laplacian_bwd(mlp, 9, 4, 0.25, tape_b, None, gop[:9].contiguous())      # both tapes are current
    ctm.ctm_laplacian_bwd(mlp, 21, 4, 0.25, tape_a, None, gop)
    Ws2, bs2 = synth.make_mlp((6, 40, 24, 1), 77, 0.1, np.float64)
    ctm.ctm_update_mlp(mlp, [t(W) for W in Ws2], [t(b) for b in bs2])
    with pytest.raises(ctm.CtmError) as ei:
        ctm.ctm_laplacian_bwd(mlp, 21, 4, 0.25, tape_a, None, gop)
    assert ei.value.status == -4 and "ctm_update_mlp" in str(ei.value)
    _, _, tape_c = ctm.ctm_laplacian_fwd(mlp, x, V, 0.25)
    ctm.ctm_laplacian_bwd(mlp, 21, 4, 0.25, tape_c, None, gop)
    # the autograd glue: two forwards on the same parameters, then one backward through both
    Ws = [t(W).requires_grad_() for W in arrs["Ws"]]
    bs = [t(b).requires_grad_() for b in arrs["bs"]]
    u1, op1 = laplacian(mlp, Ws, bs, x, V, 0.25)
    u2, op2 = laplacian(mlp, Ws, bs, x[:9].contiguous(), V[:9].contiguous(), 0.25)
    ((op1 * gop).sum() + (op2 * gop[:9]).sum()).backward()
    torch.cuda.synchronize()
    g = gop.cpu().numpy()
    _, rW1, rb1 = og.laplacian_loss_grads(arrs["Ws"], arrs["bs"], arrs["x"], arrs["V"], 0.25, np.zeros(21), g)
    _, rW2, rb2 = og.laplacian_loss_grads(arrs["Ws"], arrs["bs"], arrs["x"][:9], arrs["V"][:9], 0.25, np.zeros(9), g[:9])
    for l in range(3):
        assert rel(Ws[l].grad.cpu().numpy(), rW1[l] + rW2[l]) <= 1e-9 and rel(bs[l].grad.cpu().numpy(), rb1[l] + rb2[l]) <= 1e-9
    # an in-place parameter update between forward and backward is refused as well
    u1, op1 = laplacian(mlp, Ws, bs, x, V, 0.25)
    with torch.no_grad():
        Ws[0].mul_(1.5)
    u2, op2 = laplacian(mlp, Ws, bs, x, V, 0.25)
    with pytest.raises(ctm.CtmError):
        op1.sum().backward()
    op2.sum().backward()
    mlp.close()


def test_autograd_wrapper_trains_a_small_pinn():
    # Poisson problem  Lap u = f  on [0,1]^3 with the manufactured solution u* = sum_i sin(pi x_i):
    # f = -pi^2 u*.  A few Adam steps on residual + boundary-free value loss must reduce the loss, and the
    # gradients autograd receives must equal the oracle's.
    import torch
    import paper_2505_13644_amd as ctm
    from paper_2505_13644_amd.autograd import laplacian
    from oracle import gradients as og
    dev = torch.device("cuda:0")
    dims, N = (3, 32, 32, 1), 256
    Wn, bn = synth.make_mlp(dims, 11, 0.05, np.float64)
    Ws = [torch.tensor(W, device=dev, requires_grad=True) for W in Wn]
    bs = [torch.tensor(b, device=dev, requires_grad=True) for b in bn]
    xn = synth.make_points(N, 3, 11, np.float64)
    x = torch.tensor(xn, device=dev)
    ustar = torch.sin(np.pi * x).sum(1)
    f = -np.pi ** 2 * ustar
    mlp = ctm.ctm_create_mlp([W.detach() for W in Ws], [b.detach() for b in bs])

    def loss_fn():
        u, lap = laplacian(mlp, Ws, bs, x)
        return ((lap - f) ** 2).mean() + ((u - ustar) ** 2).mean()

    # gradient check against the oracle at the initial weights: dL/du = 2 (u - u*) / N, dL/dop = 2 (lap - f) / N
    loss = loss_fn()
    loss.backward()
    with torch.no_grad():
        u0, lap0 = ctm.ctm_laplacian(mlp, x)
        gu = (2 * (u0 - ustar) / N).cpu().numpy()
        gop = (2 * (lap0 - f) / N).cpu().numpy()
    _, rW, rb = og.laplacian_loss_grads(Wn, bn, xn, None, 1.0, gu, gop)
    for l in range(3):
        assert rel(Ws[l].grad.cpu().numpy(), rW[l]) <= 1e-8 and rel(bs[l].grad.cpu().numpy(), rb[l]) <= 1e-8
    opt = torch.optim.Adam(Ws + bs, lr=3e-3)
    first = loss.item()
    for _ in range(60):
        opt.zero_grad()
        loss = loss_fn()
        loss.backward()
        opt.step()
    last = loss_fn().item()
    print(f"  pinn loss {first:.4f} -> {last:.4f}", flush=True)
    assert last < 0.5 * first
    mlp.close()


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_weight_gradients_sin_activation(dtype):
    import torch
    import paper_2505_13644_amd as ctm
    from oracle import gradients as og
    arrs = case((5, 24, 16, 1), 21, dtype, 9, 3, True)
    dev = torch.device("cuda:0")
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    mlp = ctm.ctm_create_mlp([t(W) for W in arrs["Ws"]], [t(b) for b in arrs["bs"]], act=ctm.CTM_ACT_SIN)
    rng = np.random.default_rng(2)
    gu, gop = rng.standard_normal(21).astype(dtype), rng.standard_normal(21).astype(dtype)
    u, op, tape = ctm.ctm_laplacian_fwd(mlp, t(arrs["x"]), t(arrs["V"]), 0.5)
    gW, gb = ctm.ctm_laplacian_bwd(mlp, 21, 3, 0.5, tape, t(gu), t(gop))
    torch.cuda.synchronize()
    _, rW, rb = og.laplacian_loss_grads(arrs["Ws"], arrs["bs"], arrs["x"], arrs["V"], 0.5, gu.astype(np.float64), gop.astype(np.float64), act="sin")
    tol = 1e-9 if dtype == np.float64 else 2e-4
    for l in range(3):
        assert rel(gW[l].double().cpu().numpy(), rW[l]) <= tol and rel(gb[l].double().cpu().numpy(), rb[l]) <= tol
    mlp.close()


# ---- randomized biharmonic: reverse of the order-4 rule (Sec. 3.3, Eq. 9; "differentiable" evaluation, Sec. 4) ----

def run_gpu_biharmonic(arrs, gu, gop, dtype, act=None):
    import torch
    import paper_2505_13644_amd as ctm
    dev = torch.device("cuda:0")
    t = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    mlp = ctm.ctm_create_mlp([t(W) for W in arrs["Ws"]], [t(b) for b in arrs["bs"]], ctm.CTM_ACT_TANH if act is None else act)
    x, V = t(arrs["x"]), t(arrs["V"])
    N, S = x.shape[0], V.shape[-2]
    u, op, tape = ctm.ctm_biharmonic_rand_fwd(mlp, x, V)
    u2, op2 = ctm.ctm_biharmonic_rand(mlp, x, V)
    gW, gb = ctm.ctm_biharmonic_rand_bwd(mlp, N, S, tape, t(gu.astype(dtype)), t(gop.astype(dtype)))
    torch.cuda.synchronize()
    tol = 1e-12 if dtype == np.float64 else 2e-5
    same = (u - u2).abs().max().item() <= tol * u2.abs().max().item() and (op - op2).abs().max().item() <= tol * op2.abs().max().item()
    out = ([g.double().cpu().numpy() for g in gW], [g.double().cpu().numpy() for g in gb], same)
    mlp.close()
    return out


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("dims,N,S,per_point", [
    ((5, 16, 16, 1), 8, 3, True),            # c1's network
    ((3, 40, 24, 1), 37, 5, False),          # shared directions, ragged tiles
    ((4, 48, 48, 48, 2), 21, 4, True),       # three hidden layers, two outputs
    ((2, 100, 1), 70, 2, False),             # one hidden layer
    ((10, 160, 144, 1), 60, 6, True),        # widths over one 128-column tile
])
def test_biharmonic_weight_gradients_against_the_autograd_oracle(dtype, dims, N, S, per_point):
    from oracle import gradients as og
    arrs = case(dims, N, dtype, seed=N + len(dims), R=S, per_point=per_point)
    C = dims[-1]
    rng = np.random.default_rng(N)
    shape = (N,) if C == 1 else (N, C)
    gu, gop = rng.standard_normal(shape), rng.standard_normal(shape)
    print(f"case biharmonic backward dims={dims} N={N} S={S} {dtype.__name__}", flush=True)
    gW, gb, same = run_gpu_biharmonic(arrs, gu, gop, dtype)
    assert same, "the recording forward must agree with ctm_biharmonic_rand"
    _, rW, rb = og.biharmonic_loss_grads(arrs["Ws"], arrs["bs"], arrs["x"], arrs["V"],
                                         gu.astype(dtype).astype(np.float64), gop.astype(dtype).astype(np.float64))
    tol = 1e-9 if dtype == np.float64 else 2e-4
    for l in range(len(dims) - 1):
        eW, eb = rel(gW[l], rW[l]), rel(gb[l], rb[l])
        print(f"  layer {l}: dW err {eW:.2e}  db err {eb:.2e}", flush=True)
        assert eW <= tol and eb <= tol, (l, eW, eb)


def test_biharmonic_backward_on_its_benchmark_network_and_sin_activation():
    import torch
    import paper_2505_13644_amd as ctm
    from oracle import gradients as og
    # the order-4 workload's network and direction count at a reduced batch
    w = synth.WORKLOADS["c5"]
    N = 12
    arrs = w.build(N)
    rng = np.random.default_rng(8)
    gu, gop = rng.standard_normal(N), rng.standard_normal(N)
    gW, gb, same = run_gpu_biharmonic(arrs, gu, gop, np.float32)
    gW2, gb2, _ = run_gpu_biharmonic(arrs, gu, gop, np.float32)
    assert same
    for a, b in zip(gW + gb, gW2 + gb2):
        assert np.array_equal(a, b)  # fixed partitions and orders: bitwise reproducible
    _, rW, rb = og.biharmonic_loss_grads(arrs["Ws"], arrs["bs"], arrs["x"], arrs["V"], gu.astype(np.float32).astype(np.float64),
                                         gop.astype(np.float32).astype(np.float64))
    for l in range(len(rW)):
        eW, eb = rel(gW[l], rW[l]), rel(gb[l], rb[l])
        print(f"  c5 net layer {l}: dW err {eW:.2e}  db err {eb:.2e}", flush=True)
        assert eW <= 2e-4 and eb <= 2e-4
    # sin activation: its fifth derivative is cos
    arrs = case((4, 24, 16, 1), 15, np.float64, 3, 3, True)
    gu, gop = rng.standard_normal(15), rng.standard_normal(15)
    gW, gb, _ = run_gpu_biharmonic(arrs, gu, gop, np.float64, act=ctm.CTM_ACT_SIN)
    _, rW, rb = og.biharmonic_loss_grads(arrs["Ws"], arrs["bs"], arrs["x"], arrs["V"], gu, gop, act="sin")
    for l in range(3):
        assert rel(gW[l], rW[l]) <= 1e-9 and rel(gb[l], rb[l]) <= 1e-9
    # more than 84 directions: one tape per pass, the size query counts them all
    dev = torch.device("cuda:0")
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    mlp = ctm.ctm_create_mlp([t(W) for W in arrs["Ws"]], [t(b) for b in arrs["bs"]])
    one = ctm.ctm_biharmonic_tape_bytes(mlp, 10, 84)
    assert ctm.ctm_biharmonic_tape_bytes(mlp, 10, 85) > one > 0
    mlp.close()


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_gradients_of_direction_sets_split_over_several_passes(dtype):
    # more rows per point than one tile holds: the recording forward keeps a tape per pass and the reverse pass adds
    # the passes' gradients in pass order -- order 2 with R = 300 (two passes) and R = 520 (three), order 4 with S = 100
    from oracle import gradients as og
    tol = 1e-9 if dtype == np.float64 else 2e-4
    rng = np.random.default_rng(17)
    for R, per_point in ((300, False), (520, True)):
        arrs = case((6, 24, 16, 1), 11, dtype, R, R, per_point)
        gu, gop = rng.standard_normal(11), rng.standard_normal(11)
        print(f"case split reverse order 2 R={R} per_point={per_point} {np.dtype(dtype).name}", flush=True)
        gW, gb, same = run_gpu(arrs, 1.0 / R, gu, gop, dtype)
        assert same
        _, rW, rb = og.laplacian_loss_grads(arrs["Ws"], arrs["bs"], arrs["x"], arrs["V"], 1.0 / R, gu.astype(dtype).astype(np.float64),
                                            gop.astype(dtype).astype(np.float64))
        for l in range(len(rW)):
            assert rel(gW[l], rW[l]) <= tol and rel(gb[l], rb[l]) <= tol, (R, l)
    arrs = case((5, 24, 16, 1), 7, dtype, 4, 100, True)
    gu, gop = rng.standard_normal(7), rng.standard_normal(7)
    print(f"case split reverse order 4 S=100 {np.dtype(dtype).name}", flush=True)
    gW, gb, same = run_gpu_biharmonic(arrs, gu, gop, dtype)
    assert same
    _, rW, rb = og.biharmonic_loss_grads(arrs["Ws"], arrs["bs"], arrs["x"], arrs["V"], gu.astype(dtype).astype(np.float64),
                                         gop.astype(dtype).astype(np.float64))
    for l in range(len(rW)):
        assert rel(gW[l], rW[l]) <= tol and rel(gb[l], rb[l]) <= tol, l


def test_autograd_wrapper_biharmonic():
    import torch
    import paper_2505_13644_amd as ctm
    from paper_2505_13644_amd.autograd import biharmonic_rand
    from oracle import gradients as og
    dev = torch.device("cuda:0")
    dims, N, S = (3, 24, 24, 1), 40, 4
    Wn, bn = synth.make_mlp(dims, 13, 0.05, np.float64)
    Ws = [torch.tensor(W, device=dev, requires_grad=True) for W in Wn]
    bs = [torch.tensor(b, device=dev, requires_grad=True) for b in bn]
    xn = synth.make_points(N, 3, 13, np.float64)
    Vn = synth.make_directions("gaussian", (N, S, 3), 13, np.float64)
    mlp = ctm.ctm_create_mlp([W.detach() for W in Ws], [b.detach() for b in bs])
    u, op = biharmonic_rand(mlp, Ws, bs, torch.tensor(xn, device=dev), torch.tensor(Vn, device=dev))
    loss = (op ** 2).mean() + (u ** 2).mean()
    loss.backward()
    gu, gop = (2 * u / N).detach().cpu().numpy(), (2 * op / N).detach().cpu().numpy()
    _, rW, rb = og.biharmonic_loss_grads(Wn, bn, xn, Vn, gu, gop)
    for l in range(3):
        assert rel(Ws[l].grad.cpu().numpy(), rW[l]) <= 1e-8 and rel(bs[l].grad.cpu().numpy(), rb[l]) <= 1e-8
    mlp.close()


# ---- exact biharmonic: three order-4 tapes, three reverse passes added in a fixed order (Sec. 3.3, Eq. 12) ----

@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("dims,N", [((1, 12, 1), 9), ((2, 16, 16, 1), 21), ((3, 24, 16, 2), 17), ((5, 32, 24, 1), 13)])
def test_exact_biharmonic_weight_gradients_against_the_autograd_oracle(dtype, dims, N):
    import torch
    import paper_2505_13644_amd as ctm
    from oracle import gradients as og
    Ws, bs = synth.make_mlp(dims, N, 0.1, dtype)
    x = synth.make_points(N, dims[0], N, dtype)
    C = dims[-1]
    rng = np.random.default_rng(N)
    shape = (N,) if C == 1 else (N, C)
    gu, gop = rng.standard_normal(shape).astype(dtype), rng.standard_normal(shape).astype(dtype)
    dev = torch.device("cuda:0")
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    print(f"case exact biharmonic backward dims={dims} N={N} {dtype.__name__}", flush=True)
    mlp = ctm.ctm_create_mlp([t(W) for W in Ws], [t(b) for b in bs])
    u, op, tape = ctm.ctm_biharmonic_exact_fwd(mlp, t(x))
    u2, op2 = ctm.ctm_biharmonic_exact(mlp, t(x))
    gW, gb = ctm.ctm_biharmonic_exact_bwd(mlp, N, tape, t(gu), t(gop))
    gW2, gb2 = ctm.ctm_biharmonic_exact_bwd(mlp, N, tape, t(gu), t(gop))
    torch.cuda.synchronize()
    tolf = 1e-12 if dtype == np.float64 else 2e-5
    assert (u - u2).abs().max().item() <= tolf * u2.abs().max().item()
    assert (op - op2).abs().max().item() <= tolf * op2.abs().max().item()
    for a, b in zip(gW + gb, gW2 + gb2):
        assert torch.equal(a, b)   # accumulation over the families happens in a fixed order
    _, rW, rb = og.biharmonic_exact_loss_grads(Ws, bs, x, gu.astype(np.float64), gop.astype(np.float64))
    tol = 1e-9 if dtype == np.float64 else 2e-4
    for l in range(len(dims) - 1):
        eW, eb = rel(gW[l].double().cpu().numpy(), rW[l]), rel(gb[l].double().cpu().numpy(), rb[l])
        print(f"  layer {l}: dW err {eW:.2e}  db err {eb:.2e}", flush=True)
        assert eW <= tol and eb <= tol, (l, eW, eb)
    mlp.close()


def test_exact_biharmonic_autograd_wrapper_and_families_split_over_passes():
    import torch
    import paper_2505_13644_amd as ctm
    from paper_2505_13644_amd.autograd import biharmonic_exact
    from oracle import gradients as og
    dev = torch.device("cuda:0")
    dims, N = (2, 20, 20, 1), 30
    Wn, bn = synth.make_mlp(dims, 21, 0.05, np.float64)
    Ws = [torch.tensor(W, device=dev, requires_grad=True) for W in Wn]
    bs = [torch.tensor(b, device=dev, requires_grad=True) for b in bn]
    xn = synth.make_points(N, 2, 21, np.float64)
    mlp = ctm.ctm_create_mlp([W.detach() for W in Ws], [b.detach() for b in bs])
    u, op = biharmonic_exact(mlp, Ws, bs, torch.tensor(xn, device=dev))
    loss = ((op - 1.0) ** 2).mean() + (u ** 2).mean()
    loss.backward()
    gu, gop = (2 * u / N).detach().cpu().numpy(), (2 * (op - 1.0) / N).detach().cpu().numpy()
    _, rW, rb = og.biharmonic_exact_loss_grads(Wn, bn, xn, gu, gop)
    for l in range(3):
        assert rel(Ws[l].grad.cpu().numpy(), rW[l]) <= 1e-8 and rel(bs[l].grad.cpu().numpy(), rb[l]) <= 1e-8
    mlp.close()
    # D = 10: the family of D (D - 1) = 90 directions takes two passes
    Wn, bn = synth.make_mlp((10, 12, 1), 1, 0.05, np.float64)
    Ws = [torch.tensor(W, device=dev, requires_grad=True) for W in Wn]
    bs = [torch.tensor(b, device=dev, requires_grad=True) for b in bn]
    xn = synth.make_points(5, 10, 3, np.float64)
    m10 = ctm.ctm_create_mlp([W.detach() for W in Ws], [b.detach() for b in bs])
    u, op = biharmonic_exact(m10, Ws, bs, torch.tensor(xn, device=dev))
    loss = (op ** 2).mean() + (u ** 2).mean()
    loss.backward()
    gu, gop = (2 * u / 5).detach().cpu().numpy(), (2 * op / 5).detach().cpu().numpy()
    _, rW, rb = og.biharmonic_exact_loss_grads(Wn, bn, xn, gu, gop)
    for l in range(2):
        assert rel(Ws[l].grad.cpu().numpy(), rW[l]) <= 1e-8 and rel(bs[l].grad.cpu().numpy(), rb[l]) <= 1e-8
    m10.close()


def test_full_size_gradients_are_additive_over_the_batch():
    # At the benchmark size the oracle cannot follow (4096 Hessians of a 768-wide network), but the loss is a sum over
    # points, so the gradient of the full batch must equal the sum of the gradients of its two halves (each half takes
    # different row partitions in the weight-gradient GEMM), and a 32-point slice is checked against the oracle.
    import torch
    import paper_2505_13644_amd as ctm
    from oracle import gradients as og
    w = synth.WORKLOADS["c2"]
    arrs = w.build()
    N = w.N
    dev = torch.device("cuda:0")
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    mlp = ctm.ctm_create_mlp([t(W) for W in arrs["Ws"]], [t(b) for b in arrs["bs"]])
    rng = np.random.default_rng(11)
    gu, gop = rng.standard_normal(N).astype(np.float32), rng.standard_normal(N).astype(np.float32)
    x = t(arrs["x"])

    def grads(sl):
        n = sl.stop - sl.start
        u, op, tape = ctm.ctm_laplacian_fwd(mlp, x[sl].contiguous(), None, 1.0)
        gW, gb = ctm.ctm_laplacian_bwd(mlp, n, 50, 1.0, tape, t(gu[sl]), t(gop[sl]))
        torch.cuda.synchronize()
        return [g.double() for g in gW] + [g.double() for g in gb]

    full = grads(slice(0, N))
    a, b = grads(slice(0, N // 2)), grads(slice(N // 2, N))
    for i, (f, p, q) in enumerate(zip(full, a, b)):
        e = ((f - (p + q)).abs().max() / f.abs().max()).item()
        assert e <= 1e-4, (i, e)
    part = grads(slice(100, 132))
    _, rW, rb = og.laplacian_loss_grads(arrs["Ws"], arrs["bs"], arrs["x"][100:132], None, 1.0,
                                        gu[100:132].astype(np.float64), gop[100:132].astype(np.float64))
    for i, ref in enumerate(rW + rb):
        assert rel(part[i].cpu().numpy(), ref) <= 2e-4, i
    mlp.close()
