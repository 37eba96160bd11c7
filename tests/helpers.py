"""Shared by the GPU parity tests, the smoke check and the benchmark: run one workload
through the C-ABI binding, and through the CPU oracle."""
import numpy as np


def gpu_run(arrs, op, act=None, return_mlp=False, mlp=None, mfma=None):
    """arrs: dict from synth.Workload.build() (numpy).  Returns (u, op) as fp64 numpy arrays."""
    import torch

    import paper_2505_13644_amd as ctm

    dev = torch.device("cuda:0")
    t = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    own = mlp is None
    if own:
        mlp = ctm.ctm_create_mlp([t(W) for W in arrs["Ws"]], [t(b) for b in arrs["bs"]],
                                 ctm.CTM_ACT_TANH if act is None else act, mfma)
    x = t(arrs["x"])
    if op == "laplacian":
        u, o = ctm.ctm_laplacian(mlp, x, t(arrs.get("V")), arrs.get("scale", 1.0))
    elif op == "weighted_laplacian":
        u, o = ctm.ctm_weighted_laplacian(mlp, x, t(arrs["sigma"]))
    elif op == "biharmonic_rand":
        u, o = ctm.ctm_biharmonic_rand(mlp, x, t(arrs["V"]))
    elif op == "biharmonic_exact":
        u, o = ctm.ctm_biharmonic_exact(mlp, x)
    elif op == "laplacian_standard":
        u, o = ctm.ctm_taylor_standard(mlp, 2, x, t(arrs.get("V")), arrs.get("scale", 1.0))
    elif op == "biharmonic_rand_standard":
        V = t(arrs["V"])
        u, o = ctm.ctm_taylor_standard(mlp, 4, x, V, 1.0 / (3.0 * V.shape[-2]))
    elif op == "weighted_laplacian_rand":
        u, o = ctm.ctm_weighted_laplacian_rand(mlp, x, t(arrs["sigma"]), t(arrs.get("Vk")))
    else:
        raise ValueError(op)
    torch.cuda.synchronize()
    res = (u.double().cpu().numpy(), o.double().cpu().numpy())
    if return_mlp:
        return res + (mlp,)
    if own:
        mlp.close()
    return res


def oracle_run(arrs, op, act="tanh", idx=None, mode="directional"):
    """Oracle on the same arrays (optionally only the points in idx)."""
    from oracle import operators as orc

    sel = slice(None) if idx is None else np.asarray(idx)
    x = arrs["x"][sel]
    V = arrs.get("V")
    if V is not None and V.ndim == 3:
        V = V[sel]
    if op == "laplacian":
        return orc.laplacian(arrs["Ws"], arrs["bs"], x, V, arrs.get("scale", 1.0), act=act, mode=mode)
    if op == "weighted_laplacian":
        return orc.weighted_laplacian(arrs["Ws"], arrs["bs"], x, arrs["sigma"], act=act, mode=mode)
    if op == "biharmonic_rand":
        return orc.biharmonic_rand(arrs["Ws"], arrs["bs"], x, V, act=act)
    if op == "weighted_laplacian_rand":
        sg, Vk = arrs["sigma"], arrs.get("Vk")
        if idx is not None:
            sg = sg[sel] if sg.ndim == 3 else sg
            Vk = Vk[sel] if Vk is not None and Vk.ndim == 3 else Vk
        return orc.weighted_laplacian_rand(arrs["Ws"], arrs["bs"], x, sg, Vk, act=act)
    if op == "biharmonic_exact":
        return orc.value(arrs["Ws"], arrs["bs"], x, act=act), orc.biharmonic_exact(arrs["Ws"], arrs["bs"], x, act=act)
    raise ValueError(op)
