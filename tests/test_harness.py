"""CPU checks of the input generators (they hold no codec arithmetic, but the multi-round case depends on them)."""
import numpy as np
import torch

from paper_2405_11095_amd import inputs
from paper_2405_11095_amd.least_squares import LeastSquares


def test_least_squares_gradient_and_losses():
    """Minibatch gradient (1/m') sum_i 2 (<a_i, x> - b_i) a_i of Sec. 2 against an explicit matrix; rows are
    reproducible; sampling is with replacement; the proxy tracks the full loss."""
    d, m, M, batch = 512, 128, 3, 32
    ls = LeastSquares(d=d, m=m, M=M, batch=batch, seed=3, device="cpu")
    A = torch.stack([ls.rows([i])[0].clone() for i in range(m)])
    assert torch.equal(A[5], ls.rows([5])[0])
    assert abs(float(A.var()) * d - 1.0) < 0.05                       # a_i ~ N(0, I/d)
    x = torch.randn(d, generator=torch.Generator().manual_seed(987_654_321))
    (g, loss), (g0, loss0) = ls.gradients([x, torch.zeros(d)], rnd=7)
    tot = 0.0
    for w in range(M):
        idx = ls.sample(7, w)
        assert idx.size == batch and idx.min() >= 0 and idx.max() < m
        r = A[idx] @ x - ls.b[idx]
        want = (2.0 / batch) * (r @ A[idx])
        assert torch.allclose(g[w], want, rtol=1e-4, atol=1e-6)
        tot += float((r * r).mean()) / M
    assert abs(loss - tot) < 1e-5 * tot
    assert len(set(ls.sample(7, 0).tolist())) < batch or batch < 8     # with replacement: repeats are likely
    full = ls.full_loss(x)
    r_all = A @ x - ls.b
    assert abs(full - float((r_all.double() ** 2).mean())) < 1e-6 * full
    assert abs(ls.full_loss(ls.x_star) - 1e-4) < 5e-5                  # only the noise is left at x*
    assert abs(ls.proxy(x) / full - 1.0) < 0.35                        # expectation over rows, m = 128 rows only


def test_workload_generators_are_seeded_and_shaped():
    g1, g2 = inputs.gaussian(1000, 3), inputs.gaussian(1000, 3)
    assert np.array_equal(g1, g2) and g1.dtype == np.float32
    assert not np.array_equal(g1, inputs.gaussian(1000, 4))
    s = inputs.sparse_gaussian(100_000, 0)
    assert np.count_nonzero(s) == round(0.01 * 100_000)
    h = inputs.heavy_tailed(200_000, 1)
    assert 5e-4 < np.median(np.abs(h)) < 1.2e-3 and np.abs(h).max() > 2e-2   # 1e-3 * Student-t(3): heavy tails
    l = inputs.layered(1 << 16, 0)
    stds = l.reshape(64, -1).std(axis=1)
    assert stds.max() / stds.min() > 100                               # log-uniform layer scales over four decades
    e = inputs.one_sparse(10, 4, -2.0)
    assert e[4] == -2.0 and np.count_nonzero(e) == 1
