"""Pins for the fp64 CPU oracle: each test checks it against something other than
itself -- finite differences, closed forms, textbook derivatives, values and
formulas the paper prints, or brute force on tiny inputs.  No GPU needed.
"""
import math
import os

import numpy as np
import pytest

from oracle import nested_dual as nd
from oracle import operators as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def tiny_mlp(dims, seed, bias=True):
    rng = np.random.default_rng(seed)
    Ws = [rng.standard_normal((dims[l + 1], dims[l])) * math.sqrt(2.0 / (dims[l] + dims[l + 1])) for l in range(len(dims) - 1)]
    bs = [rng.standard_normal(dims[l + 1]) * (0.3 if bias else 0.0) for l in range(len(dims) - 1)]
    return Ws, bs


def u_plain(Ws, bs, x):
    """Independent plain evaluation of the MLP (no dual machinery)."""
    h = np.asarray(x, dtype=np.float64)
    for l, (W, b) in enumerate(zip(Ws, bs)):
        h = h @ W.T + b
        if l < len(Ws) - 1:
            h = np.tanh(h)
    return h[..., 0]


# ---------------------------------------------------------------------------
# dual arithmetic against textbook calculus and the paper's printed rules
# ---------------------------------------------------------------------------
def test_sin_two_jet_rule_printed_in_paper():
    # App. C (graph-rewrite example): the 2-jet of sin is
    #   f2 = -sin(x0) * x1 * x1 + cos(x0) * x2
    rng = np.random.default_rng(1)
    x0, x1, x2 = rng.standard_normal((3, 7))
    f = nd.sin(nd.from_jet([x0, x1, x2]))
    np.testing.assert_allclose(nd.value(f), np.sin(x0), rtol=0, atol=1e-15)
    np.testing.assert_allclose(nd.part(f, [1, 0]), np.cos(x0) * x1, rtol=1e-14)
    np.testing.assert_allclose(nd.top(f), -np.sin(x0) * x1 * x1 + np.cos(x0) * x2, rtol=1e-13, atol=1e-15)


def test_scalar_three_jet_rule_eq1():
    # Eq. 1 (scalar case, K = 3) with f = sin, whose derivatives are cos, -sin, -cos.
    rng = np.random.default_rng(2)
    x0, x1, x2, x3 = rng.standard_normal((4, 9))
    f = nd.sin(nd.from_jet([x0, x1, x2, x3]))
    f3 = -np.cos(x0) * x1 ** 3 + 3 * (-np.sin(x0)) * x1 * x2 + np.cos(x0) * x3
    np.testing.assert_allclose(nd.top(f), f3, rtol=1e-12, atol=1e-14)


def _read_multiplicities():
    rows = []
    with open(os.path.join(GOLDEN, "faa_di_bruno_multiplicities.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            k, parts, nu = line.split("|")
            rows.append((int(k), tuple(int(p) for p in parts.split()), int(nu)))
    return rows


def test_multiplicity_fixture_is_consistent():
    # nu(sigma) = k! / (prod n_s! * prod s!)  (Eq. 3) and sum over partitions = Bell number.
    rows = _read_multiplicities()
    bell = {2: 2, 3: 5, 4: 15}
    tot = {}
    for k, parts, nu in rows:
        assert sum(parts) == k
        den = 1
        for s in set(parts):
            den *= math.factorial(parts.count(s))
        for s in parts:
            den *= math.factorial(s)
        assert nu == math.factorial(k) // den
        tot[k] = tot.get(k, 0) + nu
    assert tot == bell


@pytest.mark.parametrize("k", [2, 3, 4])
def test_full_jet_through_sin_matches_cheat_sheet(k):
    # App. A cheat sheet: h_k = sum_sigma nu(sigma) <d^{|sigma|} h, (x)_{s in sigma} x_s>.
    # Elementwise h = sin: d^m sin = sin(x + m pi/2) (textbook).
    rng = np.random.default_rng(10 + k)
    coeffs = list(rng.standard_normal((k + 1, 6)))
    x0 = coeffs[0]
    want = np.zeros(6)
    for kk, parts, nu in _read_multiplicities():
        if kk != k:
            continue
        term = np.sin(x0 + len(parts) * np.pi / 2) * nu
        for s in parts:
            term = term * coeffs[s]
        want += term
    got = nd.top(nd.sin(nd.from_jet(coeffs)))
    np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-13)


def test_tanh_derivatives_printed_in_appendix_h():
    # App. H: tanh' = 1 - phi0^2 ; tanh'' = -2 phi0 (1 - phi0^2)
    z = np.linspace(-2.5, 2.5, 41)
    one = np.ones_like(z)
    f = nd.tanh(nd.seed(z, [one, one]))
    t = np.tanh(z)
    np.testing.assert_allclose(nd.part(f, [1, 0]), 1 - t * t, rtol=1e-14)
    np.testing.assert_allclose(nd.part(f, [0, 1]), 1 - t * t, rtol=1e-14)
    np.testing.assert_allclose(nd.top(f), -2 * t * (1 - t * t), rtol=1e-13, atol=1e-16)


def test_tanh_third_and_fourth_derivative_by_finite_differences():
    # The paper does not print tanh''' and tanh''''; pin the oracle's 4-level dual by central
    # differences of the (paper-printed) second derivative, in extended precision.
    z = np.linspace(-2.0, 2.0, 17)
    one = np.ones_like(z)
    f4 = nd.tanh(nd.seed(z, [one] * 4))
    d3 = nd.part(f4, [1, 1, 1, 0])
    d4 = nd.top(f4)

    def d2(zz):
        t = np.tanh(zz.astype(np.longdouble))
        return -2 * t * (1 - t * t)

    h = np.longdouble(1e-3)
    zl = z.astype(np.longdouble)
    fd3 = (-d2(zl + 2 * h) + 8 * d2(zl + h) - 8 * d2(zl - h) + d2(zl - 2 * h)) / (12 * h)
    fd4 = (-d2(zl + 2 * h) + 16 * d2(zl + h) - 30 * d2(zl) + 16 * d2(zl - h) - d2(zl - 2 * h)) / (12 * h * h)
    np.testing.assert_allclose(d3, fd3.astype(np.float64), rtol=1e-8, atol=1e-9)
    np.testing.assert_allclose(d4, fd4.astype(np.float64), rtol=1e-7, atol=1e-8)


def test_dual_product_rule_on_polynomial():
    # f(x) = (sum x_i^2)^2 : Laplacian 4(D+2) r^2, biharmonic 8 D (D+2)   (textbook, radial functions)
    D = 4
    rng = np.random.default_rng(3)
    x = rng.standard_normal((3, D))

    def fn(v):
        r2 = nd.sum_last(v * v)
        return r2 * r2

    H = orc.hessian(None, None, x, fn=fn)
    r2 = (x * x).sum(1)
    np.testing.assert_allclose(np.trace(H, axis1=1, axis2=2), 4 * (D + 2) * r2, rtol=1e-12)
    bi = orc.biharmonic_exact(None, None, x, fn=fn)
    np.testing.assert_allclose(bi, 8 * D * (D + 2) * np.ones(3), rtol=1e-12)


# ---------------------------------------------------------------------------
# closed forms that do not involve an MLP
# ---------------------------------------------------------------------------
def test_sum_of_sines_closed_forms():
    D = 5
    rng = np.random.default_rng(4)
    x = rng.uniform(-2, 2, (6, D))
    V = rng.standard_normal((6, 3, D))
    fn = lambda v: nd.sum_last(nd.sin(v))
    f = np.sin(x).sum(1)
    H = orc.hessian(None, None, x, fn=fn)
    np.testing.assert_allclose(np.trace(H, axis1=1, axis2=2), -f, rtol=1e-13)
    # off-diagonal entries vanish, diagonal is -sin x_i
    np.testing.assert_allclose(H, -np.sin(x)[:, :, None] * np.eye(D)[None], atol=1e-15)
    np.testing.assert_allclose(orc.biharmonic_exact(None, None, x, fn=fn), f, rtol=1e-12)
    d4 = orc.directional_derivative(None, None, x, V, 4, fn=fn)
    np.testing.assert_allclose(d4, np.einsum("nsd,nd->ns", V ** 4, np.sin(x)), rtol=1e-12, atol=1e-13)
    d2 = orc.directional_derivative(None, None, x, V, 2, fn=fn)
    np.testing.assert_allclose(d2, -np.einsum("nsd,nd->ns", V ** 2, np.sin(x)), rtol=1e-12, atol=1e-13)


# ---------------------------------------------------------------------------
# MLP: finite differences, closed forms for one hidden layer, special cases
# ---------------------------------------------------------------------------
def test_value_matches_plain_evaluation():
    Ws, bs = tiny_mlp((5, 16, 16, 1), 5)
    x = np.random.default_rng(5).random((8, 5))
    np.testing.assert_allclose(orc.value(Ws, bs, x), u_plain(Ws, bs, x), rtol=1e-14)


def test_hessian_against_central_finite_differences():
    Ws, bs = tiny_mlp((5, 16, 16, 1), 6)
    x = np.random.default_rng(6).random((4, 5))
    H = orc.hessian(Ws, bs, x)
    np.testing.assert_allclose(H, H.transpose(0, 2, 1), atol=1e-15)
    h = 1e-4
    D = 5
    E = np.eye(D)
    for i in range(D):
        for j in range(D):
            if i == j:
                fd = (u_plain(Ws, bs, x + h * E[i]) - 2 * u_plain(Ws, bs, x) + u_plain(Ws, bs, x - h * E[i])) / h ** 2
            else:
                fd = (u_plain(Ws, bs, x + h * E[i] + h * E[j]) - u_plain(Ws, bs, x + h * E[i] - h * E[j])
                      - u_plain(Ws, bs, x - h * E[i] + h * E[j]) + u_plain(Ws, bs, x - h * E[i] - h * E[j])) / (4 * h ** 2)
            np.testing.assert_allclose(H[:, i, j], fd, rtol=2e-5, atol=2e-7)


def test_fourth_directional_derivative_against_finite_differences():
    Ws, bs = tiny_mlp((5, 16, 16, 1), 7)
    rng = np.random.default_rng(7)
    x = rng.random((3, 5))
    V = rng.standard_normal((3, 2, 5))
    d4 = orc.directional_derivative(Ws, bs, x, V, 4)

    def stencil(h, n, s):
        g = lambda a: u_plain(Ws, bs, (x[n] + a * V[n, s]).astype(np.longdouble).astype(np.float64))
        return (g(-2 * h) - 4 * g(-h) + 6 * g(0.0) - 4 * g(h) + g(2 * h)) / h ** 4

    for n in range(3):
        for s in range(2):
            a, b = stencil(2e-2, n, s), stencil(1e-2, n, s)
            rich = (4 * b - a) / 3  # Richardson: the 5-point stencil has an h^2 error term
            assert abs(d4[n, s] - rich) <= 2e-4 * max(1.0, abs(rich))


def one_hidden(seed, D=6, I=11):
    rng = np.random.default_rng(seed)
    W1 = rng.standard_normal((I, D)) * 0.6
    b1 = rng.standard_normal(I) * 0.3
    a = rng.standard_normal((1, I))
    c = rng.standard_normal(1)
    return [W1, a], [b1, c]


def tanh_derivs_longdouble(z):
    """tanh'' and tanh'''' from scratch by differentiating 1 - t^2 symbolically in t:
    t' = 1 - t^2 =: s, t'' = -2 t s, t''' = -2 s^2 + 4 t^2 s, t'''' = 16 t s^2 - 8 t^3 s."""
    t = np.tanh(z)
    s = 1 - t * t
    return -2 * t * s, 16 * t * s * s - 8 * t ** 3 * s


def test_one_hidden_layer_closed_forms():
    # Special case of the App. H two-layer scheme: u = sum_j a_j tanh(w_j.x + b_j) + c
    #   Lap u = sum_j a_j |w_j|^2 tanh''(z_j);  Tr(s s^T H) = sum_j a_j |s^T w_j|^2 tanh''(z_j)
    #   <d^4 u, v^4> = sum_j a_j (w_j.v)^4 tanh''''(z_j);  Lap^2 u = sum_j a_j |w_j|^4 tanh''''(z_j)
    (W1, a), (b1, c) = one_hidden(8)
    Ws, bs = [W1, a], [b1, c]
    rng = np.random.default_rng(8)
    x = rng.random((5, 6))
    z = x @ W1.T + b1
    d2, d4 = tanh_derivs_longdouble(z)
    u, lap = orc.laplacian(Ws, bs, x)
    np.testing.assert_allclose(u, np.tanh(z) @ a[0] + c[0], rtol=1e-14)
    np.testing.assert_allclose(lap, (d2 * (W1 ** 2).sum(1)) @ a[0], rtol=1e-12)
    sigma = rng.standard_normal((6, 3))
    _, wl = orc.weighted_laplacian(Ws, bs, x, sigma)
    np.testing.assert_allclose(wl, (d2 * ((W1 @ sigma) ** 2).sum(1)) @ a[0], rtol=1e-12)
    V = rng.standard_normal((5, 4, 6))
    _, bh = orc.biharmonic_rand(Ws, bs, x, V)
    wv = np.einsum("id,nsd->nsi", W1, V)
    want = np.einsum("nsi,ni,i->n", wv ** 4, d4, a[0]) / (3 * 4)
    np.testing.assert_allclose(bh, want, rtol=1e-11)
    np.testing.assert_allclose(orc.biharmonic_exact(Ws, bs, x), (d4 * (W1 ** 2).sum(1) ** 2) @ a[0], rtol=1e-11)


def test_identity_activation_gives_zero_operator_and_affine_value():
    Ws, bs = tiny_mlp((5, 16, 16, 1), 9)
    rng = np.random.default_rng(9)
    x = rng.random((4, 5))
    u, lap = orc.laplacian(Ws, bs, x, act="identity")
    A = Ws[2] @ Ws[1] @ Ws[0]
    c = Ws[2] @ (Ws[1] @ bs[0] + bs[1]) + bs[2]
    np.testing.assert_allclose(u, (x @ A.T + c)[:, 0], rtol=1e-13)
    assert np.max(np.abs(lap)) == 0.0
    _, bh = orc.biharmonic_rand(Ws, bs, x, rng.standard_normal((4, 3, 5)), act="identity")
    assert np.max(np.abs(bh)) == 0.0


def test_hessian_mode_equals_directional_mode():
    # The collapsed sum equals the sum of R separate single-direction passes (Sec. 3.1).
    Ws, bs = tiny_mlp((5, 16, 16, 1), 11)
    rng = np.random.default_rng(11)
    x = rng.random((6, 5))
    for V in (None, rng.standard_normal((3, 5)), rng.standard_normal((6, 4, 5))):
        u1, a = orc.laplacian(Ws, bs, x, V, 0.5, mode="hessian")
        u2, b = orc.laplacian(Ws, bs, x, V, 0.5, mode="directional")
        np.testing.assert_allclose(a, b, rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(u1, u2, rtol=0, atol=0)
        if V is not None and V.ndim == 2:
            single = sum(orc.laplacian(Ws, bs, x, V[r:r + 1], 0.5, mode="directional")[1] for r in range(V.shape[0]))
            np.testing.assert_allclose(a, single, rtol=1e-11, atol=1e-13)
    sigma = rng.standard_normal((5, 2))
    np.testing.assert_allclose(orc.weighted_laplacian(Ws, bs, x, sigma, mode="hessian")[1],
                               orc.weighted_laplacian(Ws, bs, x, sigma, mode="directional")[1], rtol=1e-11, atol=1e-13)


def test_basis_invariance_and_homogeneity():
    Ws, bs = tiny_mlp((5, 16, 16, 1), 12)
    rng = np.random.default_rng(12)
    x = rng.random((4, 5))
    Q, _ = np.linalg.qr(rng.standard_normal((5, 5)))
    _, exact = orc.laplacian(Ws, bs, x)
    _, rot = orc.laplacian(Ws, bs, x, Q, mode="directional")
    np.testing.assert_allclose(rot, exact, rtol=1e-11, atol=1e-13)
    _, wl = orc.weighted_laplacian(Ws, bs, x, np.eye(5))
    np.testing.assert_allclose(wl, exact, rtol=1e-12, atol=1e-14)
    V = rng.standard_normal((4, 3, 5))
    _, a = orc.laplacian(Ws, bs, x, V, mode="directional")
    _, b = orc.laplacian(Ws, bs, x, 1.7 * V, mode="directional")
    np.testing.assert_allclose(b, 1.7 ** 2 * a, rtol=1e-11)
    _, a4 = orc.biharmonic_rand(Ws, bs, x, V)
    _, b4 = orc.biharmonic_rand(Ws, bs, x, 1.7 * V)
    np.testing.assert_allclose(b4, 1.7 ** 4 * a4, rtol=1e-10)
    # each point is independent of the rest of the batch
    _, solo = orc.biharmonic_rand(Ws, bs, x[2:3], V[2:3])
    np.testing.assert_allclose(solo, a4[2:3], rtol=1e-12)


def test_estimators_are_unbiased_statistically():
    # E[v^T H v] = Tr H for unit-covariance v (App. I.1); E<d^4 u, v^4> = 3 Lap^2 u for Gaussian v (Eq. 9).
    Ws, bs = tiny_mlp((3, 8, 8, 1), 13)
    rng = np.random.default_rng(13)
    x = rng.random((2, 3))
    _, exact = orc.laplacian(Ws, bs, x)
    S = 20000
    Vr = 2.0 * rng.integers(0, 2, (2, S, 3)) - 1.0
    d2 = orc.directional_derivative(Ws, bs, x, Vr, 2)
    se = d2.std(axis=1) / math.sqrt(S)
    assert np.all(np.abs(d2.mean(axis=1) - exact) <= 5 * se + 1e-12)
    bi = orc.biharmonic_exact(Ws, bs, x)
    Vg = rng.standard_normal((2, S, 3))
    d4 = orc.directional_derivative(Ws, bs, x, Vg, 4) / 3.0
    se4 = d4.std(axis=1) / math.sqrt(S)
    assert np.all(np.abs(d4.mean(axis=1) - bi) <= 5 * se4)
    # the estimator must actually have resolved the signal, or the check above is vacuous
    assert np.all(se4 < 0.25 * np.abs(bi) + 0.05)


def test_stochastic_weighted_laplacian_special_cases_and_mean():
    # Eq. 8: directions sigma v_s.  V = I_K gives K * (1/K) ... i.e. the exact operator; a point-dependent sigma
    # must equal a loop over points; the sample mean converges to Tr(sigma sigma^T H).
    Ws, bs = tiny_mlp((4, 10, 10, 1), 21)
    rng = np.random.default_rng(21)
    x = rng.random((3, 4))
    sig = rng.standard_normal((3, 4, 2))
    _, exact = orc.weighted_laplacian_rand(Ws, bs, x, sig)
    for n in range(3):
        np.testing.assert_allclose(exact[n], orc.weighted_laplacian(Ws, bs, x[n:n + 1], sig[n])[1][0], rtol=1e-12)
    _, viaI = orc.weighted_laplacian_rand(Ws, bs, x, sig, np.eye(2))
    np.testing.assert_allclose(viaI * 2, exact, rtol=1e-12)
    S = 20000
    V = rng.standard_normal((3, S, 2))
    H = orc.hessian(Ws, bs, x)
    dirs = np.einsum("ndk,nsk->nsd", sig, V)
    samples = np.einsum("nsd,nde,nse->ns", dirs, H, dirs)
    _, est = orc.weighted_laplacian_rand(Ws, bs, x, sig, V)
    np.testing.assert_allclose(est, samples.mean(axis=1), rtol=1e-12)
    assert np.all(np.abs(est - exact) <= 5 * samples.std(axis=1) / math.sqrt(S))
    _, shared = orc.weighted_laplacian_rand(Ws, bs, x, sig[0], V[0])
    np.testing.assert_allclose(shared[0], est[0], rtol=1e-12)


def test_biharmonic_exact_equals_laplacian_of_laplacian_by_finite_differences():
    Ws, bs = tiny_mlp((3, 8, 1), 14)
    x = np.random.default_rng(14).random((2, 3))
    bi = orc.biharmonic_exact(Ws, bs, x)
    h = 2e-3
    E = np.eye(3)
    lap = lambda p: orc.laplacian(Ws, bs, p)[1]
    fd = sum((lap(x + h * E[i]) - 2 * lap(x) + lap(x - h * E[i])) / h ** 2 for i in range(3))
    np.testing.assert_allclose(bi, fd, rtol=5e-5, atol=1e-6)


def test_scaled_max_err_metric():
    assert orc.scaled_max_err([1.0, 2.0, 4.0], [1.0, 2.0, 4.0]) == 0.0
    assert orc.scaled_max_err([1.0, 2.5, 4.0], [1.0, 2.0, 4.0]) == pytest.approx(0.125)
