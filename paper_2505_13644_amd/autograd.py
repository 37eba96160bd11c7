"""torch.autograd glue around the recording forward and the reverse pass of libctm.so.

    u, op = laplacian(mlp, Ws, bs, x, V=None, scale=1.0)
    u, op = biharmonic_rand(mlp, Ws, bs, x, V)
    u, op = biharmonic_exact(mlp, Ws, bs, x)

return tensors that are differentiable with respect to the weight tensors Ws / bs (not x or V).  Every number is
produced by the library's kernels; this module only re-packs the current weights into the handle
(ctm_update_mlp), keeps the tape alive between forward and backward, and hands the gradients to autograd.
"""
from __future__ import annotations

import torch

from . import binding as B


def _sync_weights(mlp, Ws, bs):
    """Re-pack the weights into the handle unless it already holds exactly these tensors at these versions.

    The reverse pass reads the weights from the handle, so the handle must still hold a forward's weights when its
    backward runs: several forwards with unchanged parameters (interior and boundary points of one loss) share one
    packing, and a parameter update between a forward and its backward makes the library refuse that backward
    (CTM_ERR_UNSUPPORTED) instead of returning gradients of the wrong network."""
    key = tuple((t.data_ptr(), t._version, tuple(t.shape)) for t in (*Ws, *bs))
    if getattr(mlp, "_packed_key", None) != key:
        B.ctm_update_mlp(mlp, [W.detach().contiguous() for W in Ws], [b.detach().contiguous() for b in bs])
        mlp._packed_key = key


class _Laplacian(torch.autograd.Function):
    @staticmethod
    def forward(ctx, mlp, x, V, scale, n_layers, *params):
        Ws, bs = list(params[:n_layers]), list(params[n_layers:])
        _sync_weights(mlp, Ws, bs)
        u, op, tape = B.ctm_laplacian_fwd(mlp, x, V, scale)
        ctx.mlp, ctx.tape, ctx.scale, ctx.n_layers = mlp, tape, scale, n_layers
        ctx.N = x.shape[0]
        ctx.R = x.shape[1] if V is None else V.shape[-2]
        return u, op

    @staticmethod
    def backward(ctx, gu, gop):
        gu = None if gu is None else gu.contiguous()
        gop = None if gop is None else gop.contiguous()
        gW, gb = B.ctm_laplacian_bwd(ctx.mlp, ctx.N, ctx.R, ctx.scale, ctx.tape, gu, gop)
        return (None, None, None, None, None, *gW, *gb)


class _BiharmonicRand(torch.autograd.Function):
    @staticmethod
    def forward(ctx, mlp, x, V, n_layers, *params):
        Ws, bs = list(params[:n_layers]), list(params[n_layers:])
        _sync_weights(mlp, Ws, bs)
        u, op, tape = B.ctm_biharmonic_rand_fwd(mlp, x, V)
        ctx.mlp, ctx.tape, ctx.N, ctx.S = mlp, tape, x.shape[0], V.shape[-2]
        return u, op

    @staticmethod
    def backward(ctx, gu, gop):
        gu = None if gu is None else gu.contiguous()
        gop = None if gop is None else gop.contiguous()
        gW, gb = B.ctm_biharmonic_rand_bwd(ctx.mlp, ctx.N, ctx.S, ctx.tape, gu, gop)
        return (None, None, None, None, *gW, *gb)


class _BiharmonicExact(torch.autograd.Function):
    @staticmethod
    def forward(ctx, mlp, x, n_layers, *params):
        Ws, bs = list(params[:n_layers]), list(params[n_layers:])
        _sync_weights(mlp, Ws, bs)
        u, op, tape = B.ctm_biharmonic_exact_fwd(mlp, x)
        ctx.mlp, ctx.tape, ctx.N = mlp, tape, x.shape[0]
        return u, op

    @staticmethod
    def backward(ctx, gu, gop):
        gu = None if gu is None else gu.contiguous()
        gop = None if gop is None else gop.contiguous()
        gW, gb = B.ctm_biharmonic_exact_bwd(ctx.mlp, ctx.N, ctx.tape, gu, gop)
        return (None, None, None, *gW, *gb)


def biharmonic_exact(mlp, Ws, bs, x):
    """(u, op) of ctm_biharmonic_exact, differentiable with respect to the tensors in Ws and bs."""
    return _BiharmonicExact.apply(mlp, x, len(Ws), *Ws, *bs)


def biharmonic_rand(mlp, Ws, bs, x, V):
    """(u, op) of ctm_biharmonic_rand, differentiable with respect to the tensors in Ws and bs."""
    return _BiharmonicRand.apply(mlp, x, V, len(Ws), *Ws, *bs)


def laplacian(mlp, Ws, bs, x, V=None, scale=1.0):
    """(u, op) of ctm_laplacian, differentiable with respect to the tensors in Ws and bs."""
    return _Laplacian.apply(mlp, x, V, float(scale), len(Ws), *Ws, *bs)
