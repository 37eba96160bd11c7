"""Networks with C > 1 outputs: the operators act on every output component (Sec. 3.2, Eq. 7).

CPU part: pins of the oracle's per-output wrapper and of the C-output gradient oracle (closed form of a
one-hidden-layer network, finite differences).  GPU part: HIP path against the oracle, element by element."""
import numpy as np
import pytest

from oracle import gradients as og
from oracle import operators as orc
from paper_2505_13644_amd import synth


def one_hidden(rng, D, H, C):
    W1, b1 = rng.standard_normal((H, D)) * 0.6, rng.standard_normal(H) * 0.3
    A, c = rng.standard_normal((C, H)), rng.standard_normal(C)
    return W1, b1, A, c


def tanh_derivs(z):
    t = np.tanh(z)
    d1 = 1 - t * t
    return t, -2 * t * d1, 8 * t * d1 * (2 - 3 * t * t)


def test_per_output_oracle_matches_the_one_hidden_layer_closed_form():
    # u_c = sum_j A_cj tanh(z_j) + c_c :  Lap u_c = sum_j A_cj |w_j|^2 tanh''(z_j),
    # <d^4 u_c, v^4> = sum_j A_cj (w_j.v)^4 tanh''''(z_j)     (special case of the two-layer scheme, App. H)
    rng = np.random.default_rng(11)
    W1, b1, A, c = one_hidden(rng, 4, 9, 5)
    x = rng.random((6, 4))
    V = rng.standard_normal((3, 4))
    t, d2, d4 = tanh_derivs(x @ W1.T + b1)
    u, lap = orc.per_output(orc.laplacian, [W1, A], [b1, c], x)
    assert u.shape == lap.shape == (6, 5)
    np.testing.assert_allclose(u, t @ A.T + c, rtol=1e-13)
    np.testing.assert_allclose(lap, (d2 * (W1 ** 2).sum(1)) @ A.T, rtol=1e-12, atol=1e-13)
    _, bih = orc.per_output(orc.biharmonic_rand, [W1, A], [b1, c], x, V)
    want = sum(((d4 * (W1 @ v) ** 4) @ A.T) for v in V) / (3.0 * len(V))
    np.testing.assert_allclose(bih, want, rtol=1e-11, atol=1e-12)
    ex = orc.per_output(orc.biharmonic_exact, [W1, A], [b1, c], x)
    np.testing.assert_allclose(ex, (d4 * ((W1 ** 2).sum(1)) ** 2) @ A.T, rtol=1e-11, atol=1e-12)


def test_vector_output_gradient_oracle_against_finite_differences():
    rng = np.random.default_rng(17)
    dims = (3, 5, 4, 3)
    Ws = [rng.standard_normal((dims[l + 1], dims[l])) * 0.6 for l in range(3)]
    bs = [rng.standard_normal(dims[l + 1]) * 0.2 for l in range(3)]
    N, R = 4, 2
    x, V = rng.random((N, 3)), rng.standard_normal((N, R, 3))
    gu, gop = rng.standard_normal((N, 3)), rng.standard_normal((N, 3))

    def loss():
        u, op = orc.per_output(orc.laplacian, Ws, bs, x, V, 0.7)
        return float((gu * u + gop * op).sum())

    L, gW, gb = og.laplacian_loss_grads(Ws, bs, x, V, 0.7, gu, gop)
    assert L == pytest.approx(loss(), rel=1e-12)
    h = 1e-5
    for group, grads in ((Ws, gW), (bs, gb)):
        for arr, g in zip(group, grads):
            it = np.nditer(arr, flags=["multi_index"])
            for _ in it:
                i = it.multi_index
                old = arr[i]
                arr[i] = old + h
                lp = loss()
                arr[i] = old - h
                lm = loss()
                arr[i] = old
                assert g[i] == pytest.approx((lp - lm) / (2 * h), rel=2e-6, abs=2e-8), (i, g[i])


# ---------------------------------------------------------------------------------------------- GPU


def _t(a):
    import torch
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def _net(dims, seed, dtype):
    Ws, bs = synth.make_mlp(dims, seed, 0.1, dtype)
    return Ws, bs


def _err(got, ref):
    return orc.scaled_max_err(got, ref)


def _tol(dtype):
    return 1e-10 if dtype == np.float64 else 2e-4


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("dims,N,R,per_point", [((5, 24, 24, 3), 19, None, False), ((6, 40, 5), 33, 4, True),
                                                ((4, 32, 160, 9), 45, 6, False), ((3, 20, 2), 7, 300, False)])
def test_laplacian_of_every_output(dtype, dims, N, R, per_point):
    import paper_2505_13644_amd as ctm
    Ws, bs = _net(dims, N, dtype)
    x = synth.make_points(N, dims[0], N, dtype)
    V = None if R is None else synth.make_directions("gaussian", (N, R, dims[0]) if per_point else (R, dims[0]), N, dtype)
    print(f"case vector laplacian dims={dims} N={N} R={R} {dtype.__name__}", flush=True)
    mlp = ctm.ctm_create_mlp([_t(W) for W in Ws], [_t(b) for b in bs])
    u, op = ctm.ctm_laplacian(mlp, _t(x), _t(V), 0.5)
    us, ops = ctm.ctm_taylor_standard(mlp, 2, _t(x), _t(V), 0.5)
    assert tuple(u.shape) == tuple(op.shape) == (N, dims[-1])
    ru, rop = orc.per_output(orc.laplacian, Ws, bs, x, V, 0.5, mode="directional")
    for name, got, ref in (("u", u, ru), ("op", op, rop), ("u standard", us, ru), ("op standard", ops, rop)):
        e = _err(got.double().cpu().numpy(), ref)
        print(f"  {name}: {e:.2e}", flush=True)
        assert e <= _tol(dtype), (name, e)
    # every column equals, bit for bit, the scalar network built from that row of the last layer
    for c in (0, dims[-1] - 1):
        m1 = ctm.ctm_create_mlp([_t(W) for W in Ws[:-1]] + [_t(Ws[-1][c:c + 1])], [_t(b) for b in bs[:-1]] + [_t(bs[-1][c:c + 1])])
        u1, op1 = ctm.ctm_laplacian(m1, _t(x), _t(V), 0.5)
        assert (u1 == u[:, c]).all() and (op1 == op[:, c]).all()
        m1.close()
    mlp.close()


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_other_operators_of_every_output(dtype):
    import paper_2505_13644_amd as ctm
    dims, N = (4, 24, 16, 6), 21
    Ws, bs = _net(dims, 5, dtype)
    x = synth.make_points(N, 4, 5, dtype)
    V = synth.make_directions("gaussian", (N, 5, 4), 5, dtype)
    sigma = synth.make_sigma(4, 3, 5, dtype)
    mlp = ctm.ctm_create_mlp([_t(W) for W in Ws], [_t(b) for b in bs])
    checks = []
    u, op = ctm.ctm_weighted_laplacian(mlp, _t(x), _t(sigma))
    checks.append(("weighted", u, op, orc.per_output(orc.weighted_laplacian, Ws, bs, x, sigma)))
    u, op = ctm.ctm_biharmonic_rand(mlp, _t(x), _t(V))
    checks.append(("biharmonic_rand", u, op, orc.per_output(orc.biharmonic_rand, Ws, bs, x, V)))
    u, op = ctm.ctm_weighted_laplacian_rand(mlp, _t(x), _t(sigma), _t(V[:, :, :3].copy()))
    checks.append(("weighted_rand", u, op, orc.per_output(orc.weighted_laplacian_rand, Ws, bs, x, sigma, V[:, :, :3])))
    u, op = ctm.ctm_biharmonic_exact(mlp, _t(x))
    ref_ex = orc.per_output(orc.biharmonic_exact, Ws, bs, x)
    checks.append(("biharmonic_exact", u, op, (orc.per_output(orc.value, Ws, bs, x), ref_ex)))
    for name, u, op, (ru, rop) in checks:
        eu, eo = _err(u.double().cpu().numpy(), ru), _err(op.double().cpu().numpy(), rop)
        print(f"case vector {name} {dtype.__name__}: u {eu:.2e} op {eo:.2e}", flush=True)
        assert tuple(op.shape) == (N, 6)
        assert eu <= _tol(dtype) and eo <= _tol(dtype), (name, eu, eo)
    mlp.close()


@pytest.mark.gpu
def test_one_hidden_layer_closed_form_with_five_outputs_on_gpu():
    import paper_2505_13644_amd as ctm
    rng = np.random.default_rng(23)
    W1, b1, A, c = one_hidden(rng, 6, 70, 5)
    x = rng.random((50, 6))
    t, d2, _ = tanh_derivs(x @ W1.T + b1)
    mlp = ctm.ctm_create_mlp([_t(W1), _t(A)], [_t(b1), _t(c)])
    u, op = ctm.ctm_laplacian(mlp, _t(x))
    assert _err(u.cpu().numpy(), t @ A.T + c) <= 1e-12
    assert _err(op.cpu().numpy(), (d2 * (W1 ** 2).sum(1)) @ A.T) <= 1e-11
    mlp.close()


@pytest.mark.gpu
@pytest.mark.parametrize("mode", ["bf16x3", "bf16"])
def test_bf16_variants_with_several_outputs(mode):
    import paper_2505_13644_amd as ctm
    dims, N = (8, 96, 64, 4), 40
    Ws, bs = _net(dims, 9, np.float32)
    x = synth.make_points(N, 8, 9, np.float32)
    mlp = ctm.ctm_create_mlp([_t(W) for W in Ws], [_t(b) for b in bs], mfma=ctm.CTM_F32_BF16X3 if mode == "bf16x3" else ctm.CTM_F32_BF16)
    u, op = ctm.ctm_laplacian(mlp, _t(x))
    ru, rop = orc.per_output(orc.laplacian, Ws, bs, x, None, 1.0, mode="directional")
    eu, eo = _err(u.double().cpu().numpy(), ru), _err(op.double().cpu().numpy(), rop)
    print(f"case vector {mode}: u {eu:.2e} op {eo:.2e}", flush=True)
    assert eu <= 2e-2 and eo <= 2e-2
    mlp.close()


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("dims,N,R,per_point", [((5, 16, 16, 3), 8, None, False), ((6, 40, 24, 7), 37, 9, True),
                                                ((50, 160, 144, 2), 120, None, False)])
def test_weight_gradients_with_several_outputs(dtype, dims, N, R, per_point):
    import torch
    import paper_2505_13644_amd as ctm
    C = dims[-1]
    Ws, bs = _net(dims, N + 1, dtype)
    x = synth.make_points(N, dims[0], N, dtype)
    V = None if R is None else synth.make_directions("gaussian", (N, R, dims[0]) if per_point else (R, dims[0]), N, dtype)
    rng = np.random.default_rng(N)
    gu, gop = rng.standard_normal((N, C)).astype(dtype), rng.standard_normal((N, C)).astype(dtype)
    print(f"case vector backward dims={dims} N={N} R={R} {dtype.__name__}", flush=True)
    mlp = ctm.ctm_create_mlp([_t(W) for W in Ws], [_t(b) for b in bs])
    Rn = dims[0] if V is None else V.shape[-2]
    u, op, tape = ctm.ctm_laplacian_fwd(mlp, _t(x), _t(V), 0.37)
    gW, gb = ctm.ctm_laplacian_bwd(mlp, N, Rn, 0.37, tape, _t(gu), _t(gop))
    # gradients the caller does not ask for land in the workspace, not in caller memory
    gW2, gb2 = ctm.ctm_laplacian_bwd(mlp, N, Rn, 0.37, tape, _t(gu), _t(gop),
                                     gW=[None] * (len(dims) - 2) + [torch.empty_like(gW[-1])], gb=[None] * (len(dims) - 1))
    torch.cuda.synchronize()
    assert (gW2[-1] == gW[-1]).all()
    _, rW, rb = og.laplacian_loss_grads(Ws, bs, x, V, 0.37, gu.astype(np.float64), gop.astype(np.float64))
    tol = 1e-9 if dtype == np.float64 else 2e-4
    for l in range(len(dims) - 1):
        eW, eb = _err(gW[l].double().cpu().numpy(), rW[l]), _err(gb[l].double().cpu().numpy(), rb[l])
        print(f"  layer {l}: dW err {eW:.2e}  db err {eb:.2e}", flush=True)
        assert eW <= tol and eb <= tol, (l, eW, eb)
    mlp.close()


@pytest.mark.gpu
def test_autograd_glue_with_several_outputs():
    import torch
    import paper_2505_13644_amd as ctm
    from paper_2505_13644_amd import autograd as ag
    dims, N = (4, 32, 24, 3), 17
    Ws, bs = _net(dims, 3, np.float64)
    x = synth.make_points(N, 4, 3, np.float64)
    Wt = [_t(W).requires_grad_(True) for W in Ws]
    bt = [_t(b).requires_grad_(True) for b in bs]
    mlp = ctm.ctm_create_mlp([W.detach() for W in Wt], [b.detach() for b in bt])
    u, op = ag.laplacian(mlp, Wt, bt, _t(x))
    tgt = torch.linspace(-1, 1, N * 3, dtype=torch.float64, device="cuda:0").reshape(N, 3)
    loss = ((op + u - tgt) ** 2).sum()
    loss.backward()
    ru, rop = orc.per_output(orc.laplacian, Ws, bs, x)
    g = 2 * (rop + ru - tgt.cpu().numpy())
    _, rW, rb = og.laplacian_loss_grads(Ws, bs, x, None, 1.0, g, g)
    for l in range(3):
        assert _err(Wt[l].grad.cpu().numpy(), rW[l]) <= 1e-9
        assert _err(bt[l].grad.cpu().numpy(), rb[l]) <= 1e-9
    mlp.close()
