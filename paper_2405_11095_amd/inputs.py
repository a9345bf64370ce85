"""Seeded synthetic gradients for the codec's test and benchmark workloads.

This module holds none of the codec's arithmetic: it only draws fp32 vectors with NumPy's PCG64.
The same arrays are handed to the HIP library (uploaded) and to the CPU oracle (widened to
fp64), so neither side depends on the other for its inputs.

The paper (arXiv 2405.11095) reports no experiment and names no dataset; these generators are the
stand-in workloads: the value laws, sparsity and dynamic range that stress the flattening step
(Sec. 2 motivates sparse gradients; Lemma 3.6 is about heavy concentration in few coordinates).
"""
from __future__ import annotations

import numpy as np

RESNET50_PARAMS = 25_557_032  # parameter count only; no weights or data are involved


def _rng(config: int, worker: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([config, worker])))


def gaussian(d: int, worker: int, config: int = 1) -> np.ndarray:
    """i.i.d. N(0,1) entries (workload c1: d = 2^16, M = 4)."""
    return _rng(config, worker).standard_normal(d, dtype=np.float32)


def sparse_gaussian(d: int, worker: int, density: float = 0.01, config: int = 2) -> np.ndarray:
    """round(density*d) distinct uniformly placed N(0,1) entries, exact +0.0 elsewhere
    (workload c2: d = 2^20, M = 8)."""
    r = _rng(config, worker)
    nnz = int(round(density * d))
    g = np.zeros(d, dtype=np.float32)
    pos = r.choice(d, size=nnz, replace=False)
    g[pos] = r.standard_normal(nnz, dtype=np.float32)
    return g


def heavy_tailed(d: int, worker: int, nu: float = 3.0, scale: float = 1e-3, config: int = 3) -> np.ndarray:
    """scale * Student-t(nu) entries (workload c3: d = 25,557,032, M = 16)."""
    r = _rng(config, worker)
    out = np.empty(d, dtype=np.float32)
    step = 1 << 22
    for s in range(0, d, step):  # chunked to bound the fp64 temporary
        e = min(d, s + step)
        out[s:e] = (scale * r.standard_t(nu, e - s)).astype(np.float32)
    return out


def layered(d: int, worker: int, layers: int = 64, config: int = 4) -> np.ndarray:
    """N(0,1) entries, split into `layers` contiguous groups each scaled by a log-uniform factor
    in [1e-4, 1] that is the same for every worker (workload c4: d = 2^27, M = 8)."""
    factors = 10.0 ** (-4.0 * _rng(config, 1 << 20).random(layers))
    r = _rng(config, worker)
    out = np.empty(d, dtype=np.float32)
    edges = np.linspace(0, d, layers + 1).astype(np.int64)
    for l in range(layers):
        s, e = int(edges[l]), int(edges[l + 1])
        out[s:e] = r.standard_normal(e - s, dtype=np.float32) * np.float32(factors[l])
    return out


def one_sparse(d: int, j: int, c: float = 1.0) -> np.ndarray:
    """c * e_j: the 1-sparse gradient of the paper's motivating example (Sec. 2)."""
    g = np.zeros(d, dtype=np.float32)
    g[j] = c
    return g


WORKLOADS = {
    # name: (d, M, block_log2 list, generator)
    "c1": dict(d=1 << 16, M=4, block_log2=[0], gen=gaussian),
    "c2": dict(d=1 << 20, M=8, block_log2=[0], gen=sparse_gaussian),
    "c3": dict(d=RESNET50_PARAMS, M=16, block_log2=[0], gen=heavy_tailed),
    "c4": dict(d=1 << 27, M=8, block_log2=[10, 12, 14, 16], gen=layered),
}


def workload(name: str, d: int | None = None, M: int | None = None):
    """List of M fp32 gradients for a named workload (optionally at a reduced d or M for tests)."""
    w = WORKLOADS[name]
    d = w["d"] if d is None else d
    M = w["M"] if M is None else M
    return [w["gen"](d, m) for m in range(M)]
