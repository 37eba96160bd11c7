"""ctypes binding of libctm.so.  Argument marshalling only: every step of the path
runs in the library's HIP kernels.  PyTorch supplies device memory and the stream.

The functions carry the names of the C entry points declared in include/ctm.h (and include/ctm_bench.h).
There is no fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, c_char_p, c_double, c_int, c_long, c_size_t, c_void_p

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libctm.so")

CTM_F64, CTM_F32, CTM_F32_BF16X3, CTM_F32_BF16 = 0, 1, 2, 3
CTM_ACT_TANH, CTM_ACT_IDENTITY, CTM_ACT_SIN = 0, 1, 2
CTM_OK = 0
CTM_STATIC_SCRATCH_BYTES = 64 << 20   # size of the device array behind ctm_laplacian_static
STATUS_NAMES = {
    0: "CTM_OK", -1: "CTM_ERR_NULL", -2: "CTM_ERR_SHAPE", -3: "CTM_ERR_DTYPE", -4: "CTM_ERR_UNSUPPORTED",
    -5: "CTM_ERR_WORKSPACE", -6: "CTM_ERR_ALIGN", -7: "CTM_ERR_ALLOC", -8: "CTM_ERR_HIP",
}

# name -> (restype, argtypes); mirrors include/ctm.h and include/ctm_bench.h
SIGNATURES = {
    "ctm_create_mlp": (c_int, [c_int, POINTER(c_int), POINTER(c_void_p), POINTER(c_void_p), c_int, c_int, c_void_p,
                               POINTER(c_void_p)]),
    "ctm_destroy_mlp": (c_int, [c_void_p]),
    "ctm_rows_per_point": (c_long, [c_int, c_int]),
    "ctm_workspace_bytes": (c_size_t, [c_void_p, c_int, c_long, c_int]),
    "ctm_laplacian": (c_int, [c_void_p, c_void_p, c_long, c_void_p, c_int, c_long, c_double, c_void_p, c_void_p,
                              c_void_p, c_size_t, c_void_p]),
    "ctm_laplacian_static": (c_int, [c_void_p, c_void_p, c_long, c_void_p, c_int, c_long, c_double, c_void_p, c_void_p,
                                     c_void_p]),
    "ctm_weighted_laplacian": (c_int, [c_void_p, c_void_p, c_long, c_void_p, c_int, c_void_p, c_void_p, c_void_p,
                                       c_size_t, c_void_p]),
    "ctm_biharmonic_rand": (c_int, [c_void_p, c_void_p, c_long, c_void_p, c_int, c_long, c_void_p, c_void_p,
                                    c_void_p, c_size_t, c_void_p]),
    "ctm_weighted_laplacian_rand_workspace_bytes": (c_size_t, [c_void_p, c_long, c_int, c_int, c_long, c_long]),
    "ctm_weighted_laplacian_rand": (c_int, [c_void_p, c_void_p, c_long, c_void_p, c_int, c_long, c_void_p, c_int, c_long,
                                            c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]),
    "ctm_tape_bytes": (c_size_t, [c_void_p, c_long, c_int]),
    "ctm_backward_workspace_bytes": (c_size_t, [c_void_p, c_long, c_int]),
    "ctm_laplacian_fwd": (c_int, [c_void_p, c_void_p, c_long, c_void_p, c_int, c_long, c_double, c_void_p, c_void_p, c_void_p,
                                  c_size_t, c_void_p]),
    "ctm_laplacian_bwd": (c_int, [c_void_p, c_long, c_int, c_double, c_void_p, c_size_t, c_void_p, c_void_p, POINTER(c_void_p),
                                  POINTER(c_void_p), c_void_p, c_size_t, c_void_p]),
    "ctm_update_mlp": (c_int, [c_void_p, POINTER(c_void_p), POINTER(c_void_p), c_void_p]),
    "ctm_biharmonic_tape_bytes": (c_size_t, [c_void_p, c_long, c_int]),
    "ctm_biharmonic_backward_workspace_bytes": (c_size_t, [c_void_p, c_long, c_int]),
    "ctm_biharmonic_rand_fwd": (c_int, [c_void_p, c_void_p, c_long, c_void_p, c_int, c_long, c_void_p, c_void_p, c_void_p,
                                        c_size_t, c_void_p]),
    "ctm_biharmonic_rand_bwd": (c_int, [c_void_p, c_long, c_int, c_void_p, c_size_t, c_void_p, c_void_p, POINTER(c_void_p),
                                        POINTER(c_void_p), c_void_p, c_size_t, c_void_p]),
    "ctm_biharmonic_exact_tape_bytes": (c_size_t, [c_void_p, c_long]),
    "ctm_biharmonic_exact_backward_workspace_bytes": (c_size_t, [c_void_p, c_long]),
    "ctm_biharmonic_exact_fwd": (c_int, [c_void_p, c_void_p, c_long, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]),
    "ctm_biharmonic_exact_bwd": (c_int, [c_void_p, c_long, c_void_p, c_size_t, c_void_p, c_void_p, POINTER(c_void_p),
                                         POINTER(c_void_p), c_void_p, c_size_t, c_void_p]),
    "ctm_workspace_bytes_standard": (c_size_t, [c_void_p, c_int, c_long, c_int]),
    "ctm_taylor_standard": (c_int, [c_void_p, c_int, c_void_p, c_long, c_void_p, c_int, c_long, c_double, c_void_p, c_void_p,
                                    c_void_p, c_size_t, c_void_p]),
    "ctm_biharmonic_exact_workspace_bytes": (c_size_t, [c_void_p, c_long]),
    "ctm_biharmonic_exact": (c_int, [c_void_p, c_void_p, c_long, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]),
    "ctm_interpolation_gamma": (c_int, [c_int, POINTER(c_int), POINTER(c_int), POINTER(ctypes.c_longlong),
                                        POINTER(ctypes.c_longlong)]),
    "ctm_tile_plan": (c_int, [c_int, c_int, c_int, POINTER(c_int), POINTER(c_int), POINTER(c_int), POINTER(c_int)]),
    "ctm_profile_begin": (c_int, []),
    "ctm_profile_end": (c_int, [POINTER(c_double), POINTER(c_long)]),
    "ctm_last_error": (c_char_p, []),
}


class CtmError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


_lib = None


def lib():
    """Load libctm.so once; raise if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2505_13644_amd.build`")
        # PyTorch ships its own copy of the HIP runtime.  Import it first so that libctm.so binds to
        # that copy (same soname) and both see the same device context; two runtimes in one
        # process do not share devices or allocations.
        _torch()
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype, fn.argtypes = res, args
        _lib = handle
    return _lib


def ctm_last_error() -> str:
    return lib().ctm_last_error().decode()


def _check(status):
    if status != CTM_OK:
        raise CtmError(status, ctm_last_error())


def ctm_rows_per_point(K: int, R: int) -> int:
    return lib().ctm_rows_per_point(K, R)


def ctm_tile_plan(dtype: int, K: int, R: int):
    """(points_per_tile, row_blocks, dirs_per_pass, n_passes)"""
    out = [c_int(0) for _ in range(4)]
    _check(lib().ctm_tile_plan(dtype, K, R, *[ctypes.byref(o) for o in out]))
    return tuple(o.value for o in out)


def ctm_interpolation_gamma(i, j):
    """gamma_{i,j} as a fractions.Fraction."""
    from fractions import Fraction
    I = len(i)
    num, den = ctypes.c_longlong(0), ctypes.c_longlong(1)
    _check(lib().ctm_interpolation_gamma(I, (c_int * I)(*i), (c_int * I)(*j), ctypes.byref(num), ctypes.byref(den)))
    return Fraction(num.value, den.value)


def ctm_profile_begin():
    _check(lib().ctm_profile_begin())


def ctm_profile_end():
    """({'seed': ms, 'layer': ms, 'final': ms}, {'seed': launches, ...})"""
    ms = (c_double * 3)()
    n = (c_long * 3)()
    _check(lib().ctm_profile_end(ms, n))
    names = ("seed", "layer", "final")
    return dict(zip(names, ms)), dict(zip(names, n))


def _torch():
    import torch
    return torch


def _stream_ptr():
    return c_void_p(_torch().cuda.current_stream().cuda_stream)


def _dtype_code(t):
    torch = _torch()
    if t == torch.float32:
        return CTM_F32
    if t == torch.float64:
        return CTM_F64
    raise CtmError(-3, f"unsupported tensor dtype {t}")


def _dev_ptr(t, dtype, name):
    if t is None:
        return c_void_p(None)
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if t.dtype != dtype:
        raise ValueError(f"{name} has dtype {t.dtype}, the handle uses {dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return c_void_p(t.data_ptr())


class Mlp:
    """Owner of a ctm_mlp handle (freed on close() / garbage collection)."""

    def __init__(self, handle, dims, dtype, act):
        self.handle, self.dims, self.dtype, self.act = handle, tuple(dims), dtype, act

    def close(self):
        if self.handle:
            h, self.handle = self.handle, None
            _check(lib().ctm_destroy_mlp(h))

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def ctm_create_mlp(Ws, bs=None, act=CTM_ACT_TANH, mfma=None) -> Mlp:
    """Ws[l]: device tensor [d_out, d_in]; bs[l]: device tensor [d_out] or None.
    mfma: None (matrix cores of the storage type) or CTM_F32_BF16X3 / CTM_F32_BF16 for fp32 tensors."""
    L = len(Ws)
    dtype = Ws[0].dtype
    dims = [Ws[0].shape[1]] + [W.shape[0] for W in Ws]
    for l, W in enumerate(Ws):
        if W.dim() != 2 or W.shape[1] != dims[l]:
            raise ValueError(f"W[{l}] has shape {tuple(W.shape)}, expected [*, {dims[l]}]")
    c_dims = (c_int * (L + 1))(*dims)
    c_W = (c_void_p * L)(*[_dev_ptr(W, dtype, f"W[{l}]") for l, W in enumerate(Ws)])
    if bs is None:
        c_b = None
    else:
        for l, b in enumerate(bs):
            if b is not None and tuple(b.shape) != (dims[l + 1],):
                raise ValueError(f"b[{l}] has shape {tuple(b.shape)}, expected [{dims[l + 1]}]")
        c_b = (c_void_p * L)(*[_dev_ptr(b, dtype, f"b[{l}]") for l, b in enumerate(bs)])
    out = c_void_p(None)
    code = _dtype_code(dtype)
    if mfma is not None:
        if code != CTM_F32 or mfma not in (CTM_F32, CTM_F32_BF16X3, CTM_F32_BF16):
            raise CtmError(-3, "the bf16 matrix-core variants need fp32 tensors")
        code = mfma
    _check(lib().ctm_create_mlp(L, c_dims, c_W, c_b, code, act, _stream_ptr(), ctypes.byref(out)))
    return Mlp(out, dims, dtype, act)


def ctm_destroy_mlp(mlp: Mlp):
    mlp.close()


def ctm_workspace_bytes(mlp: Mlp, K: int, N: int, R: int) -> int:
    n = lib().ctm_workspace_bytes(mlp.handle, K, N, R)
    if n == 0:
        raise CtmError(-2, ctm_last_error())
    return n


def _check_shapes(mlp, x, V, what="V"):
    if x.dim() != 2 or x.shape[1] != mlp.dims[0]:
        raise ValueError(f"x has shape {tuple(x.shape)}, expected [N, {mlp.dims[0]}]")
    if V is None:
        return
    if V.dim() not in (2, 3) or V.shape[-1] != x.shape[1] or (V.dim() == 3 and V.shape[0] != x.shape[0]):
        raise ValueError(f"{what} has shape {tuple(V.shape)}, expected [R, {x.shape[1]}] or [{x.shape[0]}, R, {x.shape[1]}]")


def _out_shape(mlp, N):
    """[N] for a scalar-output network, [N, C] for C > 1 outputs."""
    C = mlp.dims[-1]
    return (N,) if C == 1 else (N, C)


def _out_pair(mlp, x, u, op):
    torch = _torch()
    shape = _out_shape(mlp, x.shape[0])
    for name, t in (("u", u), ("op", op)):
        if t is not None and tuple(t.shape) != shape:
            raise ValueError(f"{name} has shape {tuple(t.shape)}, expected {list(shape)}")
    if u is None:
        u = torch.empty(shape, dtype=mlp.dtype, device=x.device)
    if op is None:
        op = torch.empty(shape, dtype=mlp.dtype, device=x.device)
    return u, op


def _outputs(mlp, x, K, R, u, op, workspace):
    torch = _torch()
    N = x.shape[0]
    u, op = _out_pair(mlp, x, u, op)
    need = ctm_workspace_bytes(mlp, K, N, R)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    return u, op, workspace


def ctm_laplacian(mlp: Mlp, x, V=None, scale=1.0, u=None, op=None, workspace=None):
    """V: None (standard basis), [R, D] shared or [N, R, D] per point.  Returns (u, op)."""
    _check_shapes(mlp, x, V)
    N, D = x.shape
    if V is None:
        R, stride = D, 0
    elif V.dim() == 2:
        R, stride = V.shape[0], 0
    else:
        R, stride = V.shape[1], V.shape[1] * V.shape[2]
    u, op, workspace = _outputs(mlp, x, 2, R, u, op, workspace)
    _check(lib().ctm_laplacian(mlp.handle, _dev_ptr(x, mlp.dtype, "x"), N, _dev_ptr(V, mlp.dtype, "V"), R, stride,
                               float(scale), _dev_ptr(u, mlp.dtype, "u"), _dev_ptr(op, mlp.dtype, "op"),
                               c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size(),
                               _stream_ptr()))
    return u, op


def ctm_laplacian_static(mlp: Mlp, x, V, scale, u, op):
    """ctm_laplacian on the library's built-in device scratch array: no workspace argument, and nothing is allocated
    here either -- u and op must be passed in.  V as in ctm_laplacian.  Returns (u, op)."""
    _check_shapes(mlp, x, V)
    N = x.shape[0]
    R, stride = _dirs_of(x, V)
    for name, t in (("u", u), ("op", op)):
        if t is None or tuple(t.shape) != _out_shape(mlp, N):
            raise ValueError(f"{name} must be a preallocated tensor of shape {list(_out_shape(mlp, N))}")
    _check(lib().ctm_laplacian_static(mlp.handle, _dev_ptr(x, mlp.dtype, "x"), N, _dev_ptr(V, mlp.dtype, "V"), R, stride,
                                      float(scale), _dev_ptr(u, mlp.dtype, "u"), _dev_ptr(op, mlp.dtype, "op"),
                                      _stream_ptr()))
    return u, op


def ctm_weighted_laplacian(mlp: Mlp, x, sigma, u=None, op=None, workspace=None):
    """sigma: [D, K] shared by all points.  Returns (u, Tr(sigma sigma^T Hessian))."""
    _check_shapes(mlp, x, None)
    N, D = x.shape
    if sigma.dim() != 2 or sigma.shape[0] != D:
        raise ValueError(f"sigma has shape {tuple(sigma.shape)}, expected [{D}, K]")
    K = sigma.shape[1]
    u, op, workspace = _outputs(mlp, x, 2, K, u, op, workspace)
    _check(lib().ctm_weighted_laplacian(mlp.handle, _dev_ptr(x, mlp.dtype, "x"), N, _dev_ptr(sigma, mlp.dtype, "sigma"),
                                        K, _dev_ptr(u, mlp.dtype, "u"), _dev_ptr(op, mlp.dtype, "op"),
                                        c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size(),
                                        _stream_ptr()))
    return u, op


def ctm_biharmonic_rand(mlp: Mlp, x, V, u=None, op=None, workspace=None):
    """V: [S, D] shared or [N, S, D] per point.  Returns (u, 1/(3S) sum_s d^4_{v_s} u)."""
    _check_shapes(mlp, x, V)
    N, D = x.shape
    if V.dim() == 2:
        S, stride = V.shape[0], 0
    else:
        S, stride = V.shape[1], V.shape[1] * V.shape[2]
    u, op, workspace = _outputs(mlp, x, 4, S, u, op, workspace)
    _check(lib().ctm_biharmonic_rand(mlp.handle, _dev_ptr(x, mlp.dtype, "x"), N, _dev_ptr(V, mlp.dtype, "V"), S, stride,
                                     _dev_ptr(u, mlp.dtype, "u"), _dev_ptr(op, mlp.dtype, "op"),
                                     c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size(),
                                     _stream_ptr()))
    return u, op


def ctm_biharmonic_exact(mlp: Mlp, x, u=None, op=None, workspace=None):
    """Exact biharmonic by interpolation with three collapsed 4-jet families.  Returns (u, op)."""
    torch = _torch()
    _check_shapes(mlp, x, None)
    N = x.shape[0]
    need = lib().ctm_biharmonic_exact_workspace_bytes(mlp.handle, N)
    if need == 0:
        raise CtmError(-2, ctm_last_error())
    u, op = _out_pair(mlp, x, u, op)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    _check(lib().ctm_biharmonic_exact(mlp.handle, _dev_ptr(x, mlp.dtype, "x"), N, _dev_ptr(u, mlp.dtype, "u"),
                                      _dev_ptr(op, mlp.dtype, "op"), c_void_p(workspace.data_ptr()),
                                      workspace.numel() * workspace.element_size(), _stream_ptr()))
    return u, op


def ctm_weighted_laplacian_rand(mlp: Mlp, x, sigma, V=None, u=None, op=None, workspace=None):
    """sigma: [D, K] or [N, D, K]; V: None (exact), [S, K] or [N, S, K].  Returns (u, op)."""
    torch = _torch()
    _check_shapes(mlp, x, None)
    N, D = x.shape
    if sigma.dim() not in (2, 3) or sigma.shape[-2] != D or (sigma.dim() == 3 and sigma.shape[0] != N):
        raise ValueError(f"sigma has shape {tuple(sigma.shape)}, expected [{D}, K] or [{N}, {D}, K]")
    K = sigma.shape[-1]
    s_stride = D * K if sigma.dim() == 3 else 0
    if V is None:
        S, v_stride = 0, 0
    else:
        if V.dim() not in (2, 3) or V.shape[-1] != K or (V.dim() == 3 and V.shape[0] != N):
            raise ValueError(f"V has shape {tuple(V.shape)}, expected [S, {K}] or [{N}, S, {K}]")
        S = V.shape[-2]
        v_stride = S * K if V.dim() == 3 else 0
    need = lib().ctm_weighted_laplacian_rand_workspace_bytes(mlp.handle, N, K, S, s_stride, v_stride)
    if need == 0:
        raise CtmError(-2, ctm_last_error())
    u, op = _out_pair(mlp, x, u, op)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    _check(lib().ctm_weighted_laplacian_rand(mlp.handle, _dev_ptr(x, mlp.dtype, "x"), N, _dev_ptr(sigma, mlp.dtype, "sigma"), K,
                                             s_stride, _dev_ptr(V, mlp.dtype, "V"), S, v_stride, _dev_ptr(u, mlp.dtype, "u"),
                                             _dev_ptr(op, mlp.dtype, "op"), c_void_p(workspace.data_ptr()),
                                             workspace.numel() * workspace.element_size(), _stream_ptr()))
    return u, op


def ctm_taylor_standard(mlp: Mlp, K, x, V=None, scale=1.0, u=None, op=None, workspace=None):
    """Un-collapsed Taylor mode of order K (comparison path).  V as in ctm_laplacian.  Returns (u, op)."""
    torch = _torch()
    _check_shapes(mlp, x, V)
    N, D = x.shape
    if V is None:
        R, stride = D, 0
    elif V.dim() == 2:
        R, stride = V.shape[0], 0
    else:
        R, stride = V.shape[1], V.shape[1] * V.shape[2]
    need = lib().ctm_workspace_bytes_standard(mlp.handle, K, N, R)
    if need == 0:
        raise CtmError(-2, ctm_last_error())
    u, op = _out_pair(mlp, x, u, op)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    _check(lib().ctm_taylor_standard(mlp.handle, K, _dev_ptr(x, mlp.dtype, "x"), N, _dev_ptr(V, mlp.dtype, "V"), R, stride,
                                     float(scale), _dev_ptr(u, mlp.dtype, "u"), _dev_ptr(op, mlp.dtype, "op"),
                                     c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size(),
                                     _stream_ptr()))
    return u, op


def _dirs_of(x, V):
    N, D = x.shape
    if V is None:
        return D, 0
    if V.dim() == 2:
        return V.shape[0], 0
    return V.shape[1], V.shape[1] * V.shape[2]


def ctm_tape_bytes(mlp: Mlp, N: int, R: int) -> int:
    n = lib().ctm_tape_bytes(mlp.handle, N, R)
    if n == 0:
        raise CtmError(-4, ctm_last_error())
    return n


def ctm_backward_workspace_bytes(mlp: Mlp, N: int, R: int) -> int:
    n = lib().ctm_backward_workspace_bytes(mlp.handle, N, R)
    if n == 0:
        raise CtmError(-4, ctm_last_error())
    return n


def ctm_laplacian_fwd(mlp: Mlp, x, V=None, scale=1.0, u=None, op=None, tape=None):
    """Forward that records a tape for ctm_laplacian_bwd.  Returns (u, op, tape)."""
    torch = _torch()
    _check_shapes(mlp, x, V)
    N = x.shape[0]
    R, stride = _dirs_of(x, V)
    u, op = _out_pair(mlp, x, u, op)
    if tape is None:
        tape = torch.empty(ctm_tape_bytes(mlp, N, R), dtype=torch.uint8, device=x.device)
    _check(lib().ctm_laplacian_fwd(mlp.handle, _dev_ptr(x, mlp.dtype, "x"), N, _dev_ptr(V, mlp.dtype, "V"), R, stride, float(scale),
                                   _dev_ptr(u, mlp.dtype, "u"), _dev_ptr(op, mlp.dtype, "op"), c_void_p(tape.data_ptr()),
                                   tape.numel(), _stream_ptr()))
    return u, op, tape


def _grad_buffers(mlp, N, tape, gu, gop, gW, gb):
    torch = _torch()
    L = len(mlp.dims) - 1
    dev = tape.device
    if gW is None:
        gW = [torch.empty(mlp.dims[l + 1], mlp.dims[l], dtype=mlp.dtype, device=dev) for l in range(L)]
    if gb is None:
        gb = [torch.empty(mlp.dims[l + 1], dtype=mlp.dtype, device=dev) for l in range(L)]
    for l in range(L):
        if gW[l] is not None and tuple(gW[l].shape) != (mlp.dims[l + 1], mlp.dims[l]):
            raise ValueError(f"gW[{l}] has shape {tuple(gW[l].shape)}")
        if gb[l] is not None and tuple(gb[l].shape) != (mlp.dims[l + 1],):
            raise ValueError(f"gb[{l}] has shape {tuple(gb[l].shape)}")
    for name, t in (("gu", gu), ("gop", gop)):
        if t is not None and tuple(t.shape) != _out_shape(mlp, N):
            raise ValueError(f"{name} has shape {tuple(t.shape)}, expected {list(_out_shape(mlp, N))}")
    c_gW = (c_void_p * L)(*[_dev_ptr(g, mlp.dtype, f"gW[{l}]") for l, g in enumerate(gW)])
    c_gb = (c_void_p * L)(*[_dev_ptr(g, mlp.dtype, f"gb[{l}]") for l, g in enumerate(gb)])
    return gW, gb, c_gW, c_gb


def ctm_laplacian_bwd(mlp: Mlp, N, R, scale, tape, gu, gop, gW=None, gb=None, workspace=None):
    """dL/dW_l, dL/db_l from dL/du (gu) and dL/dop (gop).  gW / gb: lists of preallocated tensors or None entries;
    omitted lists are allocated.  Returns (gW, gb)."""
    torch = _torch()
    gW, gb, c_gW, c_gb = _grad_buffers(mlp, N, tape, gu, gop, gW, gb)
    if workspace is None:
        workspace = torch.empty(ctm_backward_workspace_bytes(mlp, N, R), dtype=torch.uint8, device=tape.device)
    _check(lib().ctm_laplacian_bwd(mlp.handle, N, R, float(scale), c_void_p(tape.data_ptr()), tape.numel(),
                                   _dev_ptr(gu, mlp.dtype, "gu"), _dev_ptr(gop, mlp.dtype, "gop"), c_gW, c_gb,
                                   c_void_p(workspace.data_ptr()), workspace.numel(), _stream_ptr()))
    return gW, gb


def ctm_biharmonic_tape_bytes(mlp: Mlp, N: int, S: int) -> int:
    n = lib().ctm_biharmonic_tape_bytes(mlp.handle, N, S)
    if n == 0:
        raise CtmError(-4, ctm_last_error())
    return n


def ctm_biharmonic_backward_workspace_bytes(mlp: Mlp, N: int, S: int) -> int:
    n = lib().ctm_biharmonic_backward_workspace_bytes(mlp.handle, N, S)
    if n == 0:
        raise CtmError(-4, ctm_last_error())
    return n


def ctm_biharmonic_rand_fwd(mlp: Mlp, x, V, u=None, op=None, tape=None):
    """Randomized biharmonic that records a tape for ctm_biharmonic_rand_bwd.  Returns (u, op, tape)."""
    torch = _torch()
    _check_shapes(mlp, x, V)
    N = x.shape[0]
    S, stride = _dirs_of(x, V)
    u, op = _out_pair(mlp, x, u, op)
    if tape is None:
        tape = torch.empty(ctm_biharmonic_tape_bytes(mlp, N, S), dtype=torch.uint8, device=x.device)
    _check(lib().ctm_biharmonic_rand_fwd(mlp.handle, _dev_ptr(x, mlp.dtype, "x"), N, _dev_ptr(V, mlp.dtype, "V"), S, stride,
                                         _dev_ptr(u, mlp.dtype, "u"), _dev_ptr(op, mlp.dtype, "op"), c_void_p(tape.data_ptr()),
                                         tape.numel(), _stream_ptr()))
    return u, op, tape


def ctm_biharmonic_rand_bwd(mlp: Mlp, N, S, tape, gu, gop, gW=None, gb=None, workspace=None):
    """dL/dW_l, dL/db_l of the randomized biharmonic from dL/du (gu) and dL/dop (gop).  Returns (gW, gb)."""
    torch = _torch()
    gW, gb, c_gW, c_gb = _grad_buffers(mlp, N, tape, gu, gop, gW, gb)
    if workspace is None:
        workspace = torch.empty(ctm_biharmonic_backward_workspace_bytes(mlp, N, S), dtype=torch.uint8, device=tape.device)
    _check(lib().ctm_biharmonic_rand_bwd(mlp.handle, N, S, c_void_p(tape.data_ptr()), tape.numel(),
                                         _dev_ptr(gu, mlp.dtype, "gu"), _dev_ptr(gop, mlp.dtype, "gop"), c_gW, c_gb,
                                         c_void_p(workspace.data_ptr()), workspace.numel(), _stream_ptr()))
    return gW, gb


def ctm_biharmonic_exact_tape_bytes(mlp: Mlp, N: int) -> int:
    n = lib().ctm_biharmonic_exact_tape_bytes(mlp.handle, N)
    if n == 0:
        raise CtmError(-4, ctm_last_error())
    return n


def ctm_biharmonic_exact_backward_workspace_bytes(mlp: Mlp, N: int) -> int:
    n = lib().ctm_biharmonic_exact_backward_workspace_bytes(mlp.handle, N)
    if n == 0:
        raise CtmError(-4, ctm_last_error())
    return n


def ctm_biharmonic_exact_fwd(mlp: Mlp, x, u=None, op=None, tape=None):
    """Exact biharmonic that records a tape for ctm_biharmonic_exact_bwd.  Returns (u, op, tape)."""
    torch = _torch()
    _check_shapes(mlp, x, None)
    N = x.shape[0]
    u, op = _out_pair(mlp, x, u, op)
    if tape is None:
        tape = torch.empty(ctm_biharmonic_exact_tape_bytes(mlp, N), dtype=torch.uint8, device=x.device)
    _check(lib().ctm_biharmonic_exact_fwd(mlp.handle, _dev_ptr(x, mlp.dtype, "x"), N, _dev_ptr(u, mlp.dtype, "u"),
                                          _dev_ptr(op, mlp.dtype, "op"), c_void_p(tape.data_ptr()), tape.numel(), _stream_ptr()))
    return u, op, tape


def ctm_biharmonic_exact_bwd(mlp: Mlp, N, tape, gu, gop, gW=None, gb=None, workspace=None):
    """dL/dW_l, dL/db_l of the exact biharmonic from dL/du (gu) and dL/dop (gop).  Returns (gW, gb)."""
    torch = _torch()
    gW, gb, c_gW, c_gb = _grad_buffers(mlp, N, tape, gu, gop, gW, gb)
    if workspace is None:
        workspace = torch.empty(ctm_biharmonic_exact_backward_workspace_bytes(mlp, N), dtype=torch.uint8, device=tape.device)
    _check(lib().ctm_biharmonic_exact_bwd(mlp.handle, N, c_void_p(tape.data_ptr()), tape.numel(), _dev_ptr(gu, mlp.dtype, "gu"),
                                          _dev_ptr(gop, mlp.dtype, "gop"), c_gW, c_gb, c_void_p(workspace.data_ptr()),
                                          workspace.numel(), _stream_ptr()))
    return gW, gb


def ctm_update_mlp(mlp: Mlp, Ws, bs=None):
    """Re-pack new weights of the same shapes into the handle."""
    L = len(Ws)
    if L != len(mlp.dims) - 1:
        raise ValueError("wrong number of layers")
    for l, W in enumerate(Ws):
        if tuple(W.shape) != (mlp.dims[l + 1], mlp.dims[l]):
            raise ValueError(f"W[{l}] has shape {tuple(W.shape)}")
    c_W = (c_void_p * L)(*[_dev_ptr(W, mlp.dtype, f"W[{l}]") for l, W in enumerate(Ws)])
    c_b = None if bs is None else (c_void_p * L)(*[_dev_ptr(b, mlp.dtype, f"b[{l}]") for l, b in enumerate(bs)])
    _check(lib().ctm_update_mlp(mlp.handle, c_W, c_b, _stream_ptr()))
