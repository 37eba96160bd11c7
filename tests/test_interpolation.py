"""CPU pins for the interpolation coefficients used by the exact biharmonic (host arithmetic of the
library) against the values the paper prints and against mixed partials from the oracle."""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import paper_2505_13644_amd as ctm
from oracle import nested_dual as nd

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_gamma_matches_values_printed_in_the_paper():
    with open(os.path.join(GOLDEN, "biharmonic_gamma.txt")) as fh:
        rows = [tuple(map(int, l.split())) for l in fh if l.strip() and not l.startswith("#")]
    assert len(rows) == 5
    for j1, j2, num, den in rows:
        assert ctm.ctm_interpolation_gamma((2, 2), (j1, j2)) == Fraction(num, den)


def test_biharmonic_weights_reduce_to_fourth_derivative_in_one_dimension():
    # D = 1: the off-diagonal families are empty and 1/24 (2 g40 + 2 g31 + g22) 4^4 must be 1
    g40, g31, g22 = (ctm.ctm_interpolation_gamma((2, 2), j) for j in ((4, 0), (3, 1), (2, 2)))
    assert Fraction(1, 24) * (2 * g40 + 2 * g31 + g22) * 4 ** 4 == 1


def mixed_partial(fn, x, dirs):
    """<d^m f(x), dirs[0] (x) ... (x) dirs[m-1]> from the oracle's nested duals."""
    return float(nd.top(fn(nd.seed(x, [np.asarray(d, dtype=float) for d in dirs]))))


@pytest.mark.parametrize("i", [(2, 2), (2, 1), (1, 1), (3, 1), (1, 1, 1), (2, 1, 1)])
def test_interpolation_identity_against_oracle_mixed_partials(i):
    # <d^K f, v_1^{i_1} (x) ... (x) v_I^{i_I}> = sum_{|j| = K} gamma_{i,j} / K! <d^K f, (sum_t j_t v_t)^{(x) K}>   (Sec. 3.3)
    rng = np.random.default_rng(sum(i) * 10 + len(i))
    D, I, K = 4, len(i), sum(i)
    A = rng.standard_normal((3, D)) * 0.7
    fn = lambda v: nd.sum_last(nd.sin(nd.affine(v, A, None)) * nd.tanh(nd.affine(v, A[::-1].copy(), None)))
    x = rng.standard_normal(D)
    vs = rng.standard_normal((I, D))
    want = mixed_partial(fn, x, [vs[t] for t in range(I) for _ in range(i[t])])
    got = 0.0
    for j in itertools.product(range(K + 1), repeat=I):
        if sum(j) != K:
            continue
        g = ctm.ctm_interpolation_gamma(i, j)
        d = sum(j[t] * vs[t] for t in range(I))
        got += float(g) / math.factorial(K) * mixed_partial(fn, x, [d] * K)
    assert got == pytest.approx(want, rel=1e-9, abs=1e-10)


def test_gamma_rejects_bad_arguments():
    with pytest.raises(ctm.CtmError):
        ctm.ctm_interpolation_gamma((2, 2), (3, 2))
    with pytest.raises(ctm.CtmError):
        ctm.ctm_interpolation_gamma((9, 0), (9, 0))


def gamma_bigint(i, j):
    """The coefficient formula of App. E in Python's unbounded fractions (no 64-bit limit anywhere):
    gamma_{i,j} = sum_{0 < m <= i} (-1)^{|i-m|} (i over m) (|i| m / |m| over j) (|m| / |i|)^{|i|}."""
    def gbinom(a, b):
        r = Fraction(1)
        for l in range(b):
            r *= (a - l) / Fraction(b - l)
        return r
    K = sum(i)
    total = Fraction(0)
    for m in itertools.product(*[range(t + 1) for t in i]):
        if sum(m) == 0:
            continue
        term = Fraction((-1) ** (K - sum(m)))
        for t in range(len(i)):
            term *= gbinom(Fraction(i[t]), m[t]) * gbinom(Fraction(K * m[t], sum(m)), j[t])
        total += term * Fraction(sum(m), K) ** K
    return total


@pytest.mark.parametrize("i", [(2, 2, 2, 2), (5, 1, 1, 1), (3, 3, 1, 1), (4, 4), (7, 1), (2, 2, 2, 1), (4, 2, 1), (8,), (3, 2, 2, 1)])
def test_gamma_at_the_largest_orders_matches_unbounded_fractions(i):
    # the library's 64-bit fractions (128-bit intermediates) at |i| = 7 and 8 with up to four directions, every j
    K, I = sum(i), len(i)
    worst = 0
    for j in itertools.product(range(K + 1), repeat=I):
        if sum(j) != K:
            continue
        want = gamma_bigint(i, j)
        assert ctm.ctm_interpolation_gamma(i, j) == want, (i, j)
        worst = max(worst, abs(want.numerator), want.denominator)
    assert worst < 2 ** 63
