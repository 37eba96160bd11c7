"""fp64 CPU oracle for u(x) and linear PDE operators of a tanh MLP.

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the
benchmark's cpu_baseline leg, never by the product package, and it shares no
code with the HIP path.

Every operator below is the plain definition written out (the collapsed
scheme is mathematically the same number, Section 3.1, so the oracle is the
definition, not the scheme):

  * Laplacian            = trace of the Hessian                  (Sec. 3.2, Eq. 7, exact case)
  * randomized Laplacian = (1/S) sum_s v_s^T H v_s               (Eq. 7, stochastic case)
  * weighted Laplacian   = Tr(sigma sigma^T H)                   (Eq. 8, exact case)
  * randomized biharmonic= (1/(3S)) sum_s <d^4 u, v_s^{(x)4}>     (Eq. 9, stochastic case)
  * exact biharmonic     = sum_{i,j} d^4 u / dx_i^2 dx_j^2       (Eq. 9, exact case; tiny D only)

Derivative tensors come from nested dual numbers (see nested_dual.py); the
MLP is  u(x) = W_L act(... act(W_1 x + b_1) ...) + b_L  with the activation
after every layer except the last and a scalar output (Sec. 4 setup and
App. H model g o phi o h with a linear g).

Conventions: `Ws[l]` has shape [d_out, d_in]; `bs[l]` is [d_out] or None;
`x` is [N, D]; directions `V` are [R, D] (shared by all points) or [N, R, D]
(per point); `sigma` is [D, K].  Everything is widened to fp64 on entry.
"""
from __future__ import annotations

import numpy as np

from . import nested_dual as nd

_ACT = {"tanh": nd.tanh, "identity": nd.identity, "sin": nd.sin}


def _as64(a):
    return None if a is None else np.asarray(a, dtype=np.float64)


def mlp(Ws, bs, v, act="tanh"):
    """Evaluate the MLP on an ndarray or nested dual `v` (trailing axis = D). Returns [...]."""
    f = _ACT[act]
    L = len(Ws)
    for l in range(L):
        v = nd.affine(v, _as64(Ws[l]), _as64(bs[l]) if bs is not None else None)
        if l < L - 1:
            v = f(v)
    # scalar output: drop the trailing axis of length 1
    return _squeeze_last(v)


def _squeeze_last(v):
    if isinstance(v, nd.Dual):
        return nd.Dual(_squeeze_last(v.re), _squeeze_last(v.du))
    assert v.shape[-1] == 1, "the oracle covers scalar-output MLPs"
    return v[..., 0]


def value(Ws, bs, x, act="tanh"):
    return mlp(Ws, bs, _as64(x), act)


def _point_chunks(N, per_point_bytes, budget=1 << 28):
    step = max(1, int(budget // max(1, per_point_bytes)))
    for s in range(0, N, step):
        yield s, min(N, s + step)


def _widest(Ws):
    return max(max(W.shape) for W in Ws)


def hessian(Ws, bs, x, act="tanh", fn=None):
    """Full Hessian [N, D, D] of the scalar function at each point.

    H_ij is the eps_1 eps_2 coefficient of f(x + eps_1 e_i + eps_2 e_j), one
    2-level dual evaluation per pair i <= j (mirrored for i > j).
    `fn` overrides the MLP with any scalar function built from nested_dual
    primitives (used to pin the machinery on closed forms).
    """
    x = _as64(x)
    N, D = x.shape
    f = fn if fn is not None else (lambda v: mlp(Ws, bs, v, act))
    ii, jj = np.triu_indices(D)
    E = np.eye(D)
    Ei, Ej = E[ii], E[jj]  # [P, D]
    P = len(ii)
    H = np.empty((N, D, D))
    width = D if fn is not None else _widest(Ws)
    for s, e in _point_chunks(N, P * width * 8 * 8):
        out = f(nd.seed(x[s:e, None, :], [Ei[None], Ej[None]]))  # [n, P]
        h = nd.top(out)
        H[s:e, ii, jj] = h
        H[s:e, jj, ii] = h
    return H


def directional_derivative(Ws, bs, x, V, order, act="tanh", fn=None):
    """<d^order f(x_n), v^{(x) order}> for every direction: returns [N, R].

    An `order`-level nested dual with every level seeded by the same v.
    V is [R, D] (shared) or [N, R, D] (per point).
    """
    x = _as64(x)
    V = _as64(V)
    N, D = x.shape
    if V.ndim == 2:
        V = np.broadcast_to(V[None], (N,) + V.shape)
    R = V.shape[1]
    f = fn if fn is not None else (lambda v: mlp(Ws, bs, v, act))
    out = np.empty((N, R))
    width = D if fn is not None else _widest(Ws)
    for s, e in _point_chunks(N, R * width * 8 * (2 ** order) * 3):
        seeds = [V[s:e]] * order
        out[s:e] = nd.top(f(nd.seed(x[s:e, None, :], seeds)))
    return out


def laplacian(Ws, bs, x, V=None, scale=1.0, act="tanh", mode="hessian"):
    """(u, op) with op_n = scale * sum_r v_r^T H(x_n) v_r.

    V=None means the standard basis, i.e. the exact Laplacian Tr H (Eq. 7).
    mode="hessian" builds the full Hessian and contracts it; mode="directional"
    takes R second directional derivatives instead (same number; the two modes
    are checked against each other in the tests).
    """
    x = _as64(x)
    N, D = x.shape
    u = value(Ws, bs, x, act)
    if mode == "hessian":
        H = hessian(Ws, bs, x, act)
        if V is None:
            op = np.trace(H, axis1=1, axis2=2)
        else:
            V = _as64(V)
            if V.ndim == 2:
                op = np.einsum("rd,nde,re->n", V, H, V)
            else:
                op = np.einsum("nrd,nde,nre->n", V, H, V)
    elif mode == "directional":
        Vd = np.eye(D) if V is None else V
        op = directional_derivative(Ws, bs, x, Vd, 2, act).sum(axis=1)
    else:
        raise ValueError(mode)
    return u, scale * op


def weighted_laplacian(Ws, bs, x, sigma, act="tanh", mode="hessian"):
    """(u, Tr(sigma sigma^T H)) with sigma [D, K] shared by all points (Eq. 8)."""
    sigma = _as64(sigma)
    if mode == "hessian":
        u = value(Ws, bs, x, act)
        H = hessian(Ws, bs, x, act)
        Dm = sigma @ sigma.T
        return u, np.einsum("nde,de->n", H, Dm)
    return laplacian(Ws, bs, x, V=sigma.T, scale=1.0, act=act, mode="directional")


def weighted_laplacian_rand(Ws, bs, x, sigma, V=None, act="tanh"):
    """(u, (1/S) sum_s (sigma_n v_{n,s})^T H(x_n) (sigma_n v_{n,s}))  (Eq. 8, stochastic case).

    sigma is [D, K] (shared) or [N, D, K] (depends on the point); V is [S, K] or [N, S, K].
    V=None gives the exact operator Tr(sigma_n sigma_n^T H(x_n)) for a point-dependent sigma.
    """
    x = _as64(x)
    N, D = x.shape
    sigma = _as64(sigma)
    if sigma.ndim == 2:
        sigma = np.broadcast_to(sigma[None], (N,) + sigma.shape)
    u = value(Ws, bs, x, act)
    H = hessian(Ws, bs, x, act)
    if V is None:
        return u, np.einsum("nde,ndk,nek->n", H, sigma, sigma)
    V = _as64(V)
    if V.ndim == 2:
        V = np.broadcast_to(V[None], (N,) + V.shape)
    S = V.shape[1]
    dirs = np.einsum("ndk,nsk->nsd", sigma, V)
    return u, np.einsum("nsd,nde,nse->n", dirs, H, dirs) / S


def biharmonic_rand(Ws, bs, x, V, act="tanh"):
    """(u, (1/(3S)) sum_s <d^4 u, v_s^{(x)4}>) (Eq. 9, stochastic case)."""
    V = _as64(V)
    S = V.shape[-2]
    u = value(Ws, bs, x, act)
    d4 = directional_derivative(Ws, bs, x, V, 4, act)
    return u, d4.sum(axis=1) / (3.0 * S)


def biharmonic_exact(Ws, bs, x, act="tanh", fn=None):
    """sum_{i,j} d^4 f / dx_i^2 dx_j^2 per point (Eq. 9, exact case).

    One 4-level dual per (i, j) with seeds (e_i, e_i, e_j, e_j); D^2 evaluations
    per point, meant for tiny D only.
    """
    x = _as64(x)
    N, D = x.shape
    f = fn if fn is not None else (lambda v: mlp(Ws, bs, v, act))
    E = np.eye(D)
    ii, jj = np.meshgrid(np.arange(D), np.arange(D), indexing="ij")
    Ei, Ej = E[ii.ravel()], E[jj.ravel()]
    out = np.empty(N)
    for n in range(N):
        v = nd.seed(x[n][None, :], [Ei, Ei, Ej, Ej])
        out[n] = nd.top(f(v)).sum()
    return out


def per_output(fn, Ws, bs, *args, **kwargs):
    """Apply a scalar-output operator `fn(Ws, bs, ...)` to every output of a C-output network.

    The operators act on each output component on its own (Sec. 3.2, Eq. 7: the Laplacian of a
    vector-valued function stacks the Hessian traces of its elements), so output c is the operator
    of the scalar network whose last layer is row c of W_L and entry c of b_L.
    Arrays come back with a trailing axis of length C.
    """
    C = np.asarray(Ws[-1]).shape[0]
    cols = []
    for c in range(C):
        Wc = list(Ws[:-1]) + [np.asarray(Ws[-1])[c:c + 1]]
        last_b = None if bs is None or bs[-1] is None else np.asarray(bs[-1])[c:c + 1]
        bc = None if bs is None else list(bs[:-1]) + [last_b]
        cols.append(fn(Wc, bc, *args, **kwargs))
    if isinstance(cols[0], tuple):
        return tuple(np.stack([col[i] for col in cols], axis=-1) for i in range(len(cols[0])))
    return np.stack(cols, axis=-1)


def scaled_max_err(got, ref):
    """max_n |got_n - ref_n| / max_n |ref_n| : the pass/fail error metric."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.max(np.abs(ref))
    num = np.max(np.abs(got - ref)) if got.size else 0.0
    return num / den if den > 0 else num
