"""Least-squares workload of the paper's problem setup (Sec. 2: f(x) = (1/m) sum_i (<a_i, x> - b_i)^2,
minibatch SGD with rows drawn uniformly with replacement), used as the multi-round test case of the codec.

Harness code, not codec code: it only produces the M fp32 minibatch gradients that a round of FO-SGD
encodes, for whatever iterate it is handed, and evaluates losses.  It holds none of the method's
arithmetic and serves the GPU path and the CPU oracle alike (both are given the gradients it returns).

The design matrix cannot be stored at full size (m = 65536 rows of d = 2^20 fp32 entries are 256 GiB), so
row i is regenerated whenever it is needed: torch.randn from a generator seeded with (seed, i), scaled by
1/sqrt(d).  All rows are produced on one device, so every consumer sees the same numbers.
"""
from __future__ import annotations

import numpy as np
import torch


class LeastSquares:
    def __init__(self, d: int, m: int, M: int, batch: int, seed: int, device, noise: float = 0.01, chunk: int = 256):
        self.d, self.m, self.M, self.batch, self.seed = d, m, M, batch, seed
        self.device = torch.device(device)
        self.gen = torch.Generator(device=self.device)
        self.chunk = min(chunk, batch, m)
        self.buf = torch.empty((self.chunk, d), dtype=torch.float32, device=self.device)
        g = torch.Generator(device="cpu")
        g.manual_seed(seed * 1_000_003 + 17)
        self.x_star = torch.randn(d, generator=g, dtype=torch.float32).to(self.device)
        eta = torch.randn(m, generator=g, dtype=torch.float32).to(self.device) * noise
        self.b = torch.empty(m, dtype=torch.float32, device=self.device)
        for lo in range(0, m, self.chunk):
            idx = np.arange(lo, min(lo + self.chunk, m))
            self.b[lo:lo + idx.size] = self.rows(idx) @ self.x_star
        self.b += eta

    def rows(self, idx) -> torch.Tensor:
        """Rows idx (at most `chunk` of them) of A as a view of an internal buffer."""
        scale = float(self.d) ** -0.5
        out = self.buf[:len(idx)]
        for k, i in enumerate(idx):
            # the CPU generator keeps only the low 32 bits of a seed: mix seed and row index into them
            self.gen.manual_seed(((self.seed * 1_000_003 + int(i)) * 2_654_435_761 + 12_345) % (1 << 63))
            out[k].normal_(0.0, scale, generator=self.gen)
        return out

    def sample(self, rnd: int, worker: int) -> np.ndarray:
        """Row indices of worker `worker` in round `rnd`: i.i.d. uniform on [m], with replacement."""
        rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([5, self.seed, rnd, worker])))
        return rng.integers(0, self.m, size=self.batch)

    def gradients(self, xs, rnd: int):
        """For every iterate in the list xs: the M minibatch gradients (1/batch) sum_i 2 (<a_i, x> - b_i) a_i
        and the mean minibatch loss.  The rows of a round are generated once and serve all iterates, so two
        trajectories (say the GPU's and the oracle's) see the same minibatches."""
        X = torch.stack([x.to(self.device, torch.float32) for x in xs])           # [k, d]
        k = X.shape[0]
        grads = [[] for _ in range(k)]
        loss = [0.0] * k
        for w in range(self.M):
            idx = self.sample(rnd, w)
            g = torch.zeros((k, self.d), dtype=torch.float32, device=self.device)
            for lo in range(0, idx.size, self.chunk):
                part = idx[lo:lo + self.chunk]
                a = self.rows(part)                                                 # [c, d]
                r = a @ X.T - self.b[torch.as_tensor(part, device=self.device)][:, None]  # [c, k]
                g += (2.0 / self.batch) * (r.T @ a)
                sq = (r.double() ** 2).sum(dim=0) / (self.batch * self.M)
                for j in range(k):
                    loss[j] += float(sq[j])
            for j in range(k):
                grads[j].append(g[j].clone())
        return [(grads[j], loss[j]) for j in range(k)]

    def full_loss(self, x: torch.Tensor) -> float:
        x = x.to(self.device, torch.float32)
        acc = 0.0
        for lo in range(0, self.m, self.chunk):
            idx = np.arange(lo, min(lo + self.chunk, self.m))
            r = self.rows(idx) @ x - self.b[lo:lo + idx.size]
            acc += float((r.double() ** 2).sum())
        return acc / self.m

    def proxy(self, x: torch.Tensor) -> float:
        """||x - x*||^2 / d + noise^2: the expected loss when the rows are N(0, I/d)."""
        e = x.to(self.device, torch.float32) - self.x_star
        return float((e.double() ** 2).sum()) / self.d + 1e-4
