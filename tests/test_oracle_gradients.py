"""Pins for the gradient oracle (nested first-order autograd, PyTorch CPU fp64): central finite differences of
the numpy nested-dual oracle with respect to every parameter, and a closed form for one hidden layer."""
import numpy as np
import pytest

from oracle import gradients as og
from oracle import operators as orc


def tiny(dims, seed):
    rng = np.random.default_rng(seed)
    Ws = [rng.standard_normal((dims[l + 1], dims[l])) * np.sqrt(2.0 / (dims[l] + dims[l + 1])) for l in range(len(dims) - 1)]
    bs = [rng.standard_normal(dims[l + 1]) * 0.2 for l in range(len(dims) - 1)]
    return Ws, bs


def numpy_loss(Ws, bs, x, V, scale, gu, gop):
    u, op = orc.laplacian(Ws, bs, x, V, scale, mode="hessian")
    return float((gu * u + gop * op).sum())


@pytest.mark.parametrize("dims,per_point", [((3, 5, 4, 1), True), ((4, 6, 1), False), ((3, 4, 4, 3, 1), None)])
def test_gradients_against_finite_differences_of_the_numpy_oracle(dims, per_point):
    Ws, bs = tiny(dims, 31)
    rng = np.random.default_rng(32)
    N, R, D = 4, 3, dims[0]
    x = rng.random((N, D))
    V = None if per_point is None else rng.standard_normal((N, R, D) if per_point else (R, D))
    gu, gop = rng.standard_normal(N), rng.standard_normal(N)
    L, gW, gb = og.laplacian_loss_grads(Ws, bs, x, V, 0.7, gu, gop)
    assert L == pytest.approx(numpy_loss(Ws, bs, x, V, 0.7, gu, gop), rel=1e-12)
    h = 1e-5
    for group, grads in ((Ws, gW), (bs, gb)):
        for arr, g in zip(group, grads):
            it = np.nditer(arr, flags=["multi_index"])
            for _ in it:
                i = it.multi_index
                old = arr[i]
                arr[i] = old + h
                lp = numpy_loss(Ws, bs, x, V, 0.7, gu, gop)
                arr[i] = old - h
                lm = numpy_loss(Ws, bs, x, V, 0.7, gu, gop)
                arr[i] = old
                fd = (lp - lm) / (2 * h)
                assert g[i] == pytest.approx(fd, rel=2e-6, abs=2e-8), (i, g[i], fd)


def test_one_hidden_layer_closed_form_gradient():
    # u = a.tanh(W x + b) + c, Lap u = sum_j a_j |w_j|^2 tanh''(z_j):  d Lap / d a_j = |w_j|^2 tanh''(z_j),
    # d Lap / d c = 0, d u / d c = 1
    rng = np.random.default_rng(5)
    W1, b1 = rng.standard_normal((7, 4)) * 0.5, rng.standard_normal(7) * 0.2
    a, c = rng.standard_normal((1, 7)), rng.standard_normal(1)
    x = rng.random((3, 4))
    gu, gop = rng.standard_normal(3), rng.standard_normal(3)
    _, gW, gb = og.laplacian_loss_grads([W1, a], [b1, c], x, None, 1.0, gu, gop)
    z = x @ W1.T + b1
    t = np.tanh(z)
    d2 = -2 * t * (1 - t * t)
    want_a = gu @ t + gop @ (d2 * (W1 ** 2).sum(1))
    np.testing.assert_allclose(gW[1][0], want_a, rtol=1e-11)
    np.testing.assert_allclose(gb[1][0], gu.sum(), rtol=1e-12)


def numpy_biharmonic_loss(Ws, bs, x, V, gu, gop):
    u, op = orc.biharmonic_rand(Ws, bs, x, V)
    return float((gu * u + gop * op).sum())


@pytest.mark.parametrize("dims,per_point", [((3, 5, 4, 1), True), ((2, 6, 1), False)])
def test_biharmonic_gradients_against_finite_differences_of_the_numpy_oracle(dims, per_point):
    Ws, bs = tiny(dims, 41)
    rng = np.random.default_rng(42)
    N, S, D = 3, 2, dims[0]
    x = rng.random((N, D))
    V = rng.standard_normal((N, S, D) if per_point else (S, D))
    gu, gop = rng.standard_normal(N), rng.standard_normal(N)
    L, gW, gb = og.biharmonic_loss_grads(Ws, bs, x, V, gu, gop)
    assert L == pytest.approx(numpy_biharmonic_loss(Ws, bs, x, V, gu, gop), rel=1e-11)
    h = 1e-5
    for group, grads in ((Ws, gW), (bs, gb)):
        for arr, g in zip(group, grads):
            it = np.nditer(arr, flags=["multi_index"])
            for _ in it:
                i = it.multi_index
                old = arr[i]
                arr[i] = old + h
                lp = numpy_biharmonic_loss(Ws, bs, x, V, gu, gop)
                arr[i] = old - h
                lm = numpy_biharmonic_loss(Ws, bs, x, V, gu, gop)
                arr[i] = old
                assert g[i] == pytest.approx((lp - lm) / (2 * h), rel=5e-6, abs=5e-8), (i, g[i])


def test_biharmonic_closed_form_gradient_one_hidden_layer():
    # <d^4 u, v^4> = sum_j a_j (w_j.v)^4 tanh''''(z_j):  d/da_j = (w_j.v)^4 tanh''''(z_j), d/dc = 0
    rng = np.random.default_rng(6)
    W1, b1 = rng.standard_normal((6, 3)) * 0.5, rng.standard_normal(6) * 0.2
    a, c = rng.standard_normal((1, 6)), rng.standard_normal(1)
    x, V = rng.random((4, 3)), rng.standard_normal((2, 3))
    gu, gop = rng.standard_normal(4), rng.standard_normal(4)
    _, gW, gb = og.biharmonic_loss_grads([W1, a], [b1, c], x, V, gu, gop)
    t = np.tanh(x @ W1.T + b1)
    d4 = 8 * t * (1 - t * t) * (2 - 3 * t * t)
    proj4 = ((V @ W1.T) ** 4).sum(0) / (3.0 * 2)
    np.testing.assert_allclose(gW[1][0], gu @ t + gop @ (d4 * proj4), rtol=1e-11)
    np.testing.assert_allclose(gb[1][0], gu.sum(), rtol=1e-12)


def test_exact_biharmonic_gradients_against_finite_differences_and_a_closed_form():
    Ws, bs = tiny((3, 5, 4, 1), 51)
    rng = np.random.default_rng(52)
    N = 3
    x = rng.random((N, 3))
    gu, gop = rng.standard_normal(N), rng.standard_normal(N)

    def loss():
        return float((gu * orc.value(Ws, bs, x) + gop * orc.biharmonic_exact(Ws, bs, x)).sum())

    L, gW, gb = og.biharmonic_exact_loss_grads(Ws, bs, x, gu, gop)
    assert L == pytest.approx(loss(), rel=1e-11)
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
                assert g[i] == pytest.approx((lp - lm) / (2 * h), rel=5e-6, abs=5e-8), (i, g[i])
    # one hidden layer: Delta^2 u = sum_j a_j |w_j|^4 tanh''''(z_j)  =>  d/da_j = |w_j|^4 tanh''''(z_j)
    rng = np.random.default_rng(7)
    W1, b1 = rng.standard_normal((6, 3)) * 0.5, rng.standard_normal(6) * 0.2
    a, c = rng.standard_normal((1, 6)), rng.standard_normal(1)
    x = rng.random((4, 3))
    gu, gop = rng.standard_normal(4), rng.standard_normal(4)
    _, gW, gb = og.biharmonic_exact_loss_grads([W1, a], [b1, c], x, gu, gop)
    t = np.tanh(x @ W1.T + b1)
    d4 = 8 * t * (1 - t * t) * (2 - 3 * t * t)
    np.testing.assert_allclose(gW[1][0], gu @ t + gop @ (d4 * (W1 ** 2).sum(1) ** 2), rtol=1e-10)
