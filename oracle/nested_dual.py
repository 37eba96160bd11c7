"""Nested dual numbers over numpy fp64 arrays.

TEST INFRASTRUCTURE ONLY.  This module belongs to the slow CPU oracle that the
GPU library is checked against.  Nothing in the product package may import it;
only tests, the smoke check and the benchmark's cpu_baseline leg do.

A dual number is  a + b*eps  with eps*eps = 0.  Nesting m levels (each level
with its own eps_k) and seeding level k with direction d_k makes the coefficient
of eps_1*eps_2*...*eps_m in f(x + sum_k eps_k d_k) equal to the m-th derivative
tensor of f at x contracted with d_1 (x) ... (x) d_m, i.e. the quantity the
paper writes <d^m f(x0), d_1 (x) ... (x) d_m> (Section 2, the inner product
defined right after the tensor-product notation).  The only calculus used is
the first-order rule  g(a + b eps) = g(a) + g'(a) b eps  applied recursively,
so no higher-derivative formula of any activation and no Faa di Bruno
multiplicity appears anywhere in the oracle.
"""
from __future__ import annotations

import numpy as np


class Dual:
    """re + du * eps; `re` and `du` are ndarrays or Duals of one level less."""

    __slots__ = ("re", "du")

    def __init__(self, re, du):
        self.re = re
        self.du = du

    # -- ring operations ---------------------------------------------------
    def __add__(self, other):
        if isinstance(other, Dual):
            return Dual(self.re + other.re, self.du + other.du)
        return Dual(self.re + other, self.du)

    __radd__ = __add__

    def __neg__(self):
        return Dual(-self.re, -self.du)

    def __sub__(self, other):
        return self + (-other)

    def __rsub__(self, other):
        return (-self) + other

    def __mul__(self, other):
        if isinstance(other, Dual):
            # (a + b eps)(c + d eps) = ac + (ad + bc) eps
            return Dual(self.re * other.re, self.re * other.du + self.du * other.re)
        return Dual(self.re * other, self.du * other)

    __rmul__ = __mul__


def depth(v) -> int:
    d = 0
    while isinstance(v, Dual):
        v = v.re
        d += 1
    return d


def lift(a, levels: int):
    """Embed `a` as a nested dual with `levels` levels and all eps parts zero."""
    for _ in range(levels):
        a = Dual(a, _zeros_like(a))
    return a


def _zeros_like(v):
    if isinstance(v, Dual):
        return Dual(_zeros_like(v.re), _zeros_like(v.du))
    return np.zeros_like(v)


def seed(x, directions):
    """x + sum_k eps_k directions[k] as an m-level nested dual (m = len(directions)).

    x and every direction are fp64 arrays that broadcast against each other.
    """
    v = np.asarray(x, dtype=np.float64)
    for k, d in enumerate(directions):
        d = np.asarray(d, dtype=np.float64)
        shape = np.broadcast_shapes(_shape(v), d.shape)
        v = Dual(_broadcast(v, shape), lift(np.broadcast_to(d, shape).copy(), k))
    return v


def _shape(v):
    while isinstance(v, Dual):
        v = v.re
    return v.shape


def _broadcast(v, shape):
    if isinstance(v, Dual):
        return Dual(_broadcast(v.re, shape), _broadcast(v.du, shape))
    return np.broadcast_to(v, shape).copy()


def top(v):
    """Coefficient of eps_1*...*eps_m (the pure mixed part) of an m-level dual."""
    while isinstance(v, Dual):
        v = v.du
    return v


def value(v):
    """The eps-free part."""
    while isinstance(v, Dual):
        v = v.re
    return v


def part(v, mask):
    """Coefficient of prod_{k: mask[k]} eps_k; mask[k] refers to level k (0 = innermost)."""
    m = depth(v)
    assert len(mask) == m
    for k in reversed(range(m)):
        v = v.du if mask[k] else v.re
    return v


# -- elementary functions ---------------------------------------------------
def tanh(v):
    if isinstance(v, Dual):
        t = tanh(v.re)
        return Dual(t, (1.0 - t * t) * v.du)  # d tanh = 1 - tanh^2
    return np.tanh(v)


def sin(v):
    if isinstance(v, Dual):
        return Dual(sin(v.re), cos(v.re) * v.du)
    return np.sin(v)


def cos(v):
    if isinstance(v, Dual):
        return Dual(cos(v.re), -(sin(v.re) * v.du))
    return np.cos(v)


def identity(v):
    return v


def affine(v, W, b):
    """W v + b on the trailing axis; the bias only touches the eps-free part."""
    if isinstance(v, Dual):
        return Dual(affine(v.re, W, b), affine(v.du, W, None))
    out = v @ W.T
    if b is not None:
        out = out + b
    return out


def sum_last(v):
    if isinstance(v, Dual):
        return Dual(sum_last(v.re), sum_last(v.du))
    return v.sum(axis=-1)


def from_jet(coeffs):
    """Nested dual carrying a whole jet (x_0, ..., x_m) of the path x(t) = sum_k t^k/k! x_k.

    Substituting t -> eps_1 + ... + eps_m gives t^k/k! = sum over k-subsets of
    the product of their eps, so the coefficient of any product of k distinct
    eps is x_k.  The top coefficient of f(from_jet(...)) is then
    d^m/dt^m f(x(t)) at t = 0, the derivative-normalised m-th output
    coefficient of Section 2.
    """
    m = len(coeffs) - 1
    coeffs = [np.asarray(c, dtype=np.float64) for c in coeffs]

    def build(level, ones):
        if level == 0:
            return coeffs[ones].copy()
        return Dual(build(level - 1, ones), build(level - 1, ones + 1))

    return build(m, 0)
