"""Multi-round case (workload c5): FO-SGD on the least-squares problem of the paper's problem setup (Sec. 2),
the iterate fed back into the next round's minibatch gradients.

Two trajectories run side by side from x_0 = 0: the HIP path (fp32 iterate, fo_step) and the oracle (fp64 iterate,
one full round per step).  Both get their gradients from the same harness (paper_2405_11095_amd/least_squares.py,
which holds no codec arithmetic), each at its own iterate, on the same minibatches.
Gates: (i) teacher-forced, stage-by-stage bit parity of whole rounds at sampled rounds, with the round's real
gradients and iterate; (ii) free running: minibatch loss of every round and full loss at the start, the middle and
the end within 1e-3 relative of the oracle's; the two iterates stay close compared with the distance travelled.
The loss curve is nearly flat by construction: the decoded update has norm alpha alpha^s ln(n) ||g|| whatever the
gradient, and delta is small, so movement is reported as well.
"""
import sys
import time

import numpy as np
import pytest

from tests import parity as P

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env(oracle):
    import torch
    from paper_2405_11095_amd import binding as B
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return oracle, B, torch.device("cuda:0")


def _say(msg):
    print(msg, file=sys.stderr, flush=True)


@pytest.mark.parametrize("name,d,m,M,batch,rounds,every", [
    ("small", 1 << 12, 256, 4, 16, 30, 3),
    ("c5", 1 << 20, 65536, 16, 256, 200, 20),
])
@pytest.mark.timeout(900)
def test_least_squares_rounds(env, name, d, m, M, batch, rounds, every):
    import torch
    from paper_2405_11095_amd.least_squares import LeastSquares
    O, B, dev = env
    delta, seed = 1e-2, 0xF05D + 5
    t0 = time.time()
    ls = LeastSquares(d=d, m=m, M=M, batch=batch, seed=5, device=dev)
    plan = B.Plan(d=d, M=M, seed=seed)
    p = O.params(d=d, M=M, seed=seed)
    x_gpu = torch.zeros(d, dtype=torch.float32, device=dev)
    x_orc = np.zeros(d, dtype=np.float64)
    full = {}
    checked = 0
    _say(f"[{name}] harness ready in {time.time() - t0:.1f}s")
    for t in range(rounds + 1):
        if t in (0, rounds // 2, rounds):
            full[t] = (ls.full_loss(x_gpu), ls.full_loss(torch.from_numpy(x_orc.astype(np.float32))))
            _say(f"[{name}] round {t}: full loss gpu {full[t][0]:.6f} oracle {full[t][1]:.6f} proxy {ls.proxy(x_gpu):.6f}")
            assert abs(full[t][0] - full[t][1]) <= 1e-3 * full[t][1]
        if t == rounds:
            break
        (g_gpu, l_gpu), (g_orc, l_orc) = ls.gradients([x_gpu, torch.from_numpy(x_orc.astype(np.float32))], t)
        assert abs(l_gpu - l_orc) <= 1e-3 * l_orc, (t, l_gpu, l_orc)
        if t % every == 0 or t == rounds - 1:
            rep = P.check_round_trip(O, B, [g.cpu().numpy() for g in g_gpu], d, M, 0, seed, t, delta, dev,
                                     threads=min(M, 16), x0=x_gpu.cpu().numpy())
            P.gates(rep)
            checked += 1
            _say(f"[{name}] round {t}: minibatch loss {l_gpu:.6f}/{l_orc:.6f}; teacher-forced round ok "
                 f"(uplink exempt {rep['uplink_exempt']}, downlink exempt {rep['downlink_exempt']}); {time.time() - t0:.0f}s")
        plan.fo_step(g_gpu, x_gpu, delta, t)
        O.round_trip(p, [g.cpu().numpy() for g in g_orc], x_orc, delta, t, nthreads=min(M, 16))
    assert checked >= 10
    xg = x_gpu.cpu().numpy().astype(np.float64)
    xs = ls.x_star.cpu().numpy().astype(np.float64)
    moved_g, moved_o = np.linalg.norm(xg), np.linalg.norm(x_orc)
    apart = np.linalg.norm(xg - x_orc)
    _say(f"[{name}] |x_T - x_0| gpu {moved_g:.5f} oracle {moved_o:.5f}; apart {apart:.3e}; "
         f"<x_T - x_0, x*> gpu {xg @ xs:.4f} oracle {x_orc @ xs:.4f}; "
         f"f(x_T) - f(x_0) gpu {full[rounds][0] - full[0][0]:+.3e} oracle {full[rounds][1] - full[0][1]:+.3e}")
    assert abs(moved_g - moved_o) <= 1e-3 * moved_o
    assert apart <= 0.1 * moved_o
    plan.close()
