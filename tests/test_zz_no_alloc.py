"""The entry point for callers that cannot allocate: ctm_laplacian_static runs on the library's built-in device
scratch array.  Checked through the C ABI against ctm_laplacian (same kernels, so bit for bit) on two calls in a
row, the second with a smaller input, and against the oracle at the fp32 bar."""
import numpy as np
import pytest

from paper_2505_13644_amd import synth
from helpers import oracle_run

pytestmark = pytest.mark.gpu


def test_static_scratch_entry_point_matches_the_workspace_entry_point():
    import torch
    import paper_2505_13644_amd as ctm

    dev = torch.device("cuda:0")
    t = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    w = synth.WORKLOADS["c2"]
    # first the largest-but-one tile count that fits the array (basis directions, 52 rows per point), then a smaller
    # batch with per-point directions (18 rows per point): the second call finds the first one's data in the array
    cases = [(w.build(150), None), (synth.WORKLOADS["c3"].build(41), "V")]
    mlp = ctm.ctm_create_mlp([t(W) for W in cases[0][0]["Ws"]], [t(b) for b in cases[0][0]["bs"]])
    outs = []
    for arrs, vkey in cases:
        x, V = t(arrs["x"]), t(arrs.get("V") if vkey else None)
        N = x.shape[0]
        scale = arrs.get("scale", 1.0)
        u, op = torch.full((N,), 3.0, device=dev), torch.full((N,), 3.0, device=dev)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        print(f"case static N={N} per-point V={vkey is not None}", flush=True)
        ctm.ctm_laplacian_static(mlp, x, V, scale, u, op)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        outs.append((arrs, x, V, scale, u.cpu().numpy().copy(), op.cpu().numpy().copy()))
    for arrs, x, V, scale, su, so in outs:
        ru, ro = ctm.ctm_laplacian(mlp, x, V, scale)          # own workspace, allocated by the binding
        torch.cuda.synchronize()
        assert np.array_equal(su, ru.cpu().numpy()) and np.array_equal(so, ro.cpu().numpy())
        ou, oo = oracle_run(arrs, "laplacian")
        from oracle.operators import scaled_max_err
        assert scaled_max_err(su.astype(np.float64), ou) <= 2e-4 and scaled_max_err(so.astype(np.float64), oo) <= 2e-4
    # a request beyond the array is refused before anything is launched
    big = w.build(300)
    x = t(big["x"])
    u, op = torch.full((300,), 3.0, device=dev), torch.full((300,), 3.0, device=dev)
    assert ctm.ctm_workspace_bytes(mlp, 2, 300, 50) > ctm.CTM_STATIC_SCRATCH_BYTES
    with pytest.raises(ctm.CtmError) as ei:
        ctm.ctm_laplacian_static(mlp, x, None, 1.0, u, op)
    assert ei.value.status == -5 and "built-in array" in str(ei.value)
    torch.cuda.synchronize()
    assert torch.all(u == 3.0) and torch.all(op == 3.0)
    mlp.close()


def test_static_scratch_entry_point_replays_from_a_captured_graph():
    # the callers it is for: a captured graph holds kernel launches only (no allocation, no memset node); replays with
    # new inputs between eager work must reproduce the eager results bit for bit
    import torch
    import paper_2505_13644_amd as ctm

    dev = torch.device("cuda:0")
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    w = synth.WORKLOADS["c3"]
    N = 64
    arrs = w.build(N)
    mlp = ctm.ctm_create_mlp([t(W) for W in arrs["Ws"]], [t(b) for b in arrs["bs"]])
    x, V = t(arrs["x"]), t(arrs["V"])
    u, op = torch.empty(N, device=dev), torch.empty(N, device=dev)
    print("case static entry point under graph capture, N=64", flush=True)
    ctm.ctm_laplacian_static(mlp, x, V, arrs["scale"], u, op)      # first call on the device: looks up the array's address
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        ctm.ctm_laplacian_static(mlp, x, V, arrs["scale"], u, op)
    for rep in range(3):
        x.copy_(t(synth.make_points(N, 50, seed=200 + rep)))
        u.zero_(); op.zero_()
        g.replay()
        torch.cuda.synchronize()
        gu, go = u.cpu().numpy().copy(), op.cpu().numpy().copy()
        eu, eo = ctm.ctm_laplacian(mlp, x, V, arrs["scale"])        # eager, own workspace
        torch.cuda.synchronize()
        assert np.array_equal(gu, eu.cpu().numpy()) and np.array_equal(go, eo.cpu().numpy()), f"replay {rep}"
        assert np.any(go != 0)
    del g
    mlp.close()
