"""A seeded sweep over randomly drawn configurations (length, workers, block size, K, eps mode, server rule, dither,
scale rule, input law): whole rounds against the oracle, stage by stage.  Catches interactions the hand-picked
cases do not list."""
import numpy as np
import pytest

from tests import parity as P

pytestmark = pytest.mark.gpu


def _draw(rng):
    blk = int(rng.choice([0, 0, 0, 6, 7, 8, 9, 11, 13, 15, 16, 17]))
    if blk == 0:
        d = int(rng.choice([rng.integers(1, 200), rng.integers(200, 40_000), rng.integers(40_000, 400_000)]))
    else:
        d = int(rng.integers(1, max(2, min(400_000, 40 * (1 << blk)))))
    M = int(rng.choice([1, 2, 3, 5, 8, 17]))
    K = int(rng.choice([1, 1, 1, 2, 5]))
    eps_mode = int(rng.choice([0, 0, 1, 2]))
    server_scale = int(rng.choice([0, 1]))
    dither = int(rng.choice([0, 0, 0, 1]))
    scale_rule = int(rng.choice([1, 1, 0]))
    kind = str(rng.choice(["gaussian", "heavy", "sparse"]))
    return dict(d=d, M=M, blk=blk, K=K, eps_mode=eps_mode, server_scale=server_scale, dither=dither,
                scale_rule=scale_rule, kind=kind)


CONFIGS = [_draw(np.random.default_rng([2405, 11095, i])) for i in range(60)]


@pytest.mark.parametrize("cfg", CONFIGS, ids=[f"{i:02d}" for i in range(len(CONFIGS))])
def test_random_configuration(oracle, cfg):
    import torch
    from paper_2405_11095_amd import binding as B, inputs
    gen = {"gaussian": inputs.gaussian, "heavy": inputs.heavy_tailed, "sparse": inputs.sparse_gaussian}[cfg["kind"]]
    gs = [gen(cfg["d"], m) for m in range(cfg["M"])]
    bnorm = 1.5 * max(float(np.linalg.norm(g.astype(np.float64))) for g in gs) + 1e-3
    print(cfg, flush=True)
    rep = P.check_round_trip(oracle, B, gs, cfg["d"], cfg["M"], cfg["blk"], seed=0xC0FFEE + cfg["d"], rnd=3, delta=1e-2,
                             device=torch.device("cuda:0"), K=cfg["K"], eps_mode=cfg["eps_mode"],
                             server_scale=cfg["server_scale"], dither=cfg["dither"], scale_rule=cfg["scale_rule"],
                             Bnorm=bnorm)
    P.gates(rep)
