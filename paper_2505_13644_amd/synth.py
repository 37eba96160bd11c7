"""Seeded synthetic inputs: MLP weights, point batches, direction sets.

This module holds no arithmetic of the method.  It is the one piece that the
test oracle and the GPU path are both fed from, so that they see identical
arrays.  All draws come from numpy's PCG64 with a per-array stream derived
from (seed, tag); values are drawn in fp64 and rounded once to the storage
dtype, and the oracle receives those rounded arrays (widened back to fp64).

The paper's experiments use no dataset (Sec. 4 and its checklist state that
only synthetic inputs are used): a tanh MLP D -> 768 -> 768 -> 512 -> 512 -> 1,
random points, and standard-basis / Gaussian / Rademacher directions or a
sigma matrix.  The five named workloads below follow that recipe.
"""
from __future__ import annotations

import zlib
from dataclasses import dataclass, field

import numpy as np


def _rng(seed: int, tag: str) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, zlib.crc32(tag.encode())])))


def make_mlp(dims, seed=0, bias_std=0.0, dtype=np.float32):
    """Xavier-normal weights W_l ~ N(0, 2/(d_in+d_out)), biases N(0, bias_std^2) (zero if 0)."""
    Ws, bs = [], []
    for l in range(len(dims) - 1):
        d_in, d_out = dims[l], dims[l + 1]
        std = np.sqrt(2.0 / (d_in + d_out))
        Ws.append((_rng(seed, f"W{l}").standard_normal((d_out, d_in)) * std).astype(dtype))
        if bias_std > 0:
            bs.append((_rng(seed, f"b{l}").standard_normal(d_out) * bias_std).astype(dtype))
        else:
            bs.append(np.zeros(d_out, dtype=dtype))
    return Ws, bs


def make_points(N, D, seed=0, dtype=np.float32):
    """x ~ U[0,1)^D."""
    return _rng(seed, "x").random((N, D)).astype(dtype)


def make_directions(kind, shape, seed=0, dtype=np.float32):
    """Direction sets: 'rademacher' (+-1) or 'gaussian' (standard normal); shape [R,D] or [N,R,D]."""
    g = _rng(seed, "V" + kind)
    if kind == "rademacher":
        return (2.0 * g.integers(0, 2, size=shape) - 1.0).astype(dtype)
    if kind == "gaussian":
        return g.standard_normal(shape).astype(dtype)
    raise ValueError(kind)


def make_sigma(D, K, seed=0, dtype=np.float32):
    """sigma in R^{D x K}, i.i.d. N(0, 1/D) entries."""
    return (_rng(seed, "sigma").standard_normal((D, K)) / np.sqrt(D)).astype(dtype)


@dataclass
class Workload:
    name: str
    op: str                      # "laplacian" | "weighted_laplacian" | "biharmonic_rand"
    dims: tuple
    N: int
    dtype: type
    bias_std: float
    tol: float                   # scaled max-norm bound against the fp64 oracle
    directions: str = "basis"    # "basis" | "rademacher" | "gaussian" | "sigma"
    R: int = 0                   # number of directions (S or K); basis => D
    seed: int = 0
    arrays: dict = field(default_factory=dict)

    def build(self, N=None):
        """Materialise the arrays (optionally with another batch size)."""
        N = self.N if N is None else N
        D = self.dims[0]
        Ws, bs = make_mlp(self.dims, self.seed, self.bias_std, self.dtype)
        out = {"Ws": Ws, "bs": bs, "x": make_points(N, D, self.seed, self.dtype)}
        if self.directions in ("basis", "interpolation"):
            out["V"], out["scale"] = None, 1.0
        elif self.directions == "sigma":
            out["sigma"] = make_sigma(D, self.R, self.seed, self.dtype)
        else:
            out["V"] = make_directions(self.directions, (N, self.R, D), self.seed, self.dtype)
            out["scale"] = 1.0 / self.R
        return out


BIG = (50, 768, 768, 512, 512, 1)

WORKLOADS = {
    # exact Laplacian, fp64, tiny: the correctness anchor
    "c1": Workload("c1", "laplacian", (5, 16, 16, 1), 8, np.float64, 0.0, 1e-5, "basis", 5),
    # exact Laplacian, fp32, the configuration the headline metric is quoted on
    "c2": Workload("c2", "laplacian", BIG, 4096, np.float32, 0.01, 2e-4, "basis", 50),
    # randomized Laplacian, per-point Rademacher directions, S = 16
    "c3": Workload("c3", "laplacian", BIG, 4096, np.float32, 0.01, 2e-4, "rademacher", 16),
    # weighted Laplacian, sigma 50 x 10 shared
    "c4": Workload("c4", "weighted_laplacian", BIG, 2048, np.float32, 0.01, 2e-4, "sigma", 10),
    # randomized biharmonic, per-point Gaussian directions, S = 32
    "c5": Workload("c5", "biharmonic_rand", (10, 256, 256, 128, 1), 1024, np.float32, 0.0, 2e-4, "gaussian", 32),
    # beyond the five named configurations: the paper's exact-biharmonic setting (Sec. 4: D = 5, same 768/768/512/512 net),
    # three interpolation families of 5, 20 and 10 directions
    "e1": Workload("e1", "biharmonic_exact", (5, 768, 768, 512, 512, 1), 1024, np.float32, 0.01, 2e-4, "interpolation", 20),
}
