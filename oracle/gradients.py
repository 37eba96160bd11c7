"""fp64 CPU oracle for parameter gradients of Laplacian-type losses.  TEST INFRASTRUCTURE ONLY.

For  L = sum_{n,c} [ gu_{n,c} * u_c(x_n) + gop_{n,c} * op_c(x_n) ],  op_c(x_n) = scale * sum_r v_r^T H_c(x_n) v_r
(Sec. 3.2, Eq. 7-8; H_c the Hessian of output c), it returns dL/dW_l and dL/db_l.  The operator is written from its definition with nested first-order
automatic differentiation (PyTorch CPU, fp64): the Hessian of the scalar network by forward-over-reverse,
contracted with the directions, then one reverse sweep to the parameters.  No Taylor-mode rule and no code of
the HIP path is involved.  The paper calls evaluating the operator so that it can be differentiated again the
"differentiable" setting of its benchmark (Sec. 4).
"""
from __future__ import annotations

import numpy as np
import torch


def _mlp(params, x, act):
    Ws, bs = params
    h = x
    for l, (W, b) in enumerate(zip(Ws, bs)):
        h = h @ W.T + b
        if l < len(Ws) - 1:
            h = torch.tanh(h) if act == "tanh" else (torch.sin(h) if act == "sin" else h)
    return h  # [..., C]


def laplacian_loss_grads(Ws, bs, x, V, scale, gu, gop, act="tanh"):
    """Returns (L, [dL/dW_l], [dL/db_l]) as fp64 numpy.  V: None (standard basis), [R, D] or [N, R, D];
    gu, gop: [N] for a scalar-output network, [N, C] otherwise."""
    t = lambda a: torch.as_tensor(np.asarray(a, dtype=np.float64))
    Ws_t = [t(W).requires_grad_(True) for W in Ws]
    bs_t = [t(b).requires_grad_(True) for b in bs]
    xt, gut, gopt = t(x), t(gu), t(gop)
    N, D = xt.shape
    C = Ws_t[-1].shape[0]
    gut, gopt = gut.reshape(N, C), gopt.reshape(N, C)
    if V is None:
        Vt = torch.eye(D, dtype=torch.float64).expand(N, D, D)
    else:
        Vt = t(V)
        if Vt.dim() == 2:
            Vt = Vt.expand(N, *Vt.shape)

    def loss(params):
        f = lambda p: _mlp(params, p, act)                       # the C outputs at one point
        H = torch.func.vmap(torch.func.hessian(f))(xt)            # [N, C, D, D]
        u = _mlp(params, xt, act)
        op = scale * torch.einsum("nrd,ncde,nre->nc", Vt, H, Vt)
        return (gut * u + gopt * op).sum()

    L = loss((Ws_t, bs_t))
    grads = torch.autograd.grad(L, Ws_t + bs_t, allow_unused=True)
    gW = [(g if g is not None else torch.zeros_like(p)).numpy() for g, p in zip(grads[:len(Ws_t)], Ws_t)]
    gb = [(g if g is not None else torch.zeros_like(p)).numpy() for g, p in zip(grads[len(Ws_t):], bs_t)]
    return float(L.detach()), gW, gb


def biharmonic_loss_grads(Ws, bs, x, V, gu, gop, act="tanh"):
    """Gradients of  L = sum_{n,c} gu_{n,c} u_c(x_n) + gop_{n,c} op_c(x_n)  for the randomized biharmonic
    op_c(x_n) = 1/(3S) sum_s d^4/dt^4 f_c(x_n + t v_s) at t = 0  (Sec. 3.3, Eq. 9, stochastic case).

    The fourth directional derivative is four nested first-order forward derivatives of the scalar path
    t -> f(x + t v); one reverse sweep then goes to the parameters.  V: [S, D] or [N, S, D].
    Returns (L, [dL/dW_l], [dL/db_l]) as fp64 numpy.
    """
    t = lambda a: torch.as_tensor(np.asarray(a, dtype=np.float64))
    Ws_t = [t(W).requires_grad_(True) for W in Ws]
    bs_t = [t(b).requires_grad_(True) for b in bs]
    xt, Vt = t(x), t(V)
    N, D = xt.shape
    C = Ws_t[-1].shape[0]
    if Vt.dim() == 2:
        Vt = Vt.expand(N, *Vt.shape)
    S = Vt.shape[1]
    gut, gopt = t(gu).reshape(N, C), t(gop).reshape(N, C)
    zero = torch.zeros((), dtype=torch.float64)

    def loss(params):
        def d4(p, v):  # [C]: fourth derivative along v at the point p
            g = lambda s: _mlp(params, p + s * v, act)
            for _ in range(4):
                g = torch.func.jacfwd(g)
            return g(zero)

        per_dir = torch.func.vmap(torch.func.vmap(d4, in_dims=(None, 0)))(xt, Vt)  # [N, S, C]
        u = _mlp(params, xt, act)
        op = per_dir.sum(dim=1) / (3.0 * S)
        return (gut * u + gopt * op).sum()

    L = loss((Ws_t, bs_t))
    grads = torch.autograd.grad(L, Ws_t + bs_t, allow_unused=True)
    gW = [(g if g is not None else torch.zeros_like(p)).numpy() for g, p in zip(grads[:len(Ws_t)], Ws_t)]
    gb = [(g if g is not None else torch.zeros_like(p)).numpy() for g, p in zip(grads[len(Ws_t):], bs_t)]
    return float(L.detach()), gW, gb


def biharmonic_exact_loss_grads(Ws, bs, x, gu, gop, act="tanh"):
    """Gradients of  L = sum_{n,c} gu_{n,c} u_c(x_n) + gop_{n,c} (Delta^2 u_c)(x_n)  with the exact biharmonic
    Delta^2 u = Delta(Delta u) = sum_{i,j} d^4 u / dx_i^2 dx_j^2  (Sec. 3.3, Eq. 9, exact case).

    Written as the Laplacian of the Laplacian with nested first-order automatic differentiation (trace of the
    Hessian, twice), then one reverse sweep to the parameters.  Meant for tiny D and narrow networks.
    Returns (L, [dL/dW_l], [dL/db_l]) as fp64 numpy.
    """
    t = lambda a: torch.as_tensor(np.asarray(a, dtype=np.float64))
    Ws_t = [t(W).requires_grad_(True) for W in Ws]
    bs_t = [t(b).requires_grad_(True) for b in bs]
    xt = t(x)
    N, D = xt.shape
    C = Ws_t[-1].shape[0]
    gut, gopt = t(gu).reshape(N, C), t(gop).reshape(N, C)

    def loss(params):
        def bih(p):  # [C]
            f = lambda q: _mlp(params, q, act)                                             # [C]
            lap = lambda q: torch.diagonal(torch.func.hessian(f)(q), dim1=-2, dim2=-1).sum(-1)   # [C]
            return torch.diagonal(torch.func.hessian(lap)(p), dim1=-2, dim2=-1).sum(-1)
        op = torch.func.vmap(bih)(xt)
        u = _mlp(params, xt, act)
        return (gut * u + gopt * op).sum()

    L = loss((Ws_t, bs_t))
    grads = torch.autograd.grad(L, Ws_t + bs_t, allow_unused=True)
    gW = [(g if g is not None else torch.zeros_like(p)).numpy() for g, p in zip(grads[:len(Ws_t)], Ws_t)]
    gb = [(g if g is not None else torch.zeros_like(p)).numpy() for g, p in zip(grads[len(Ws_t):], bs_t)]
    return float(L.detach()), gW, gb
