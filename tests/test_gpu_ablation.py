"""The paper's motivating example (Sec. 2, "Communication-efficient SGD": sign compression of 1-sparse gradients)
run through the GPU codec, next to the two baselines it is compared with there.

Every worker holds a 1-sparse gradient c_n e_{j_n}.  Coordinate-wise sign compression with sign(0) = +1 and a
majority vote returns the all-ones vector whatever the c_n and j_n are, so its inner product with the true mean
can have either sign.  FO-SGD's decoded downlink message is an unbiased estimate of the mean (Thm 5.5), so its
average over rounds lines up with the mean.  With the dither switched off (FO_DITHER_NONE, sign of the flattened
gradient only) the estimate is biased but still correlated.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _cos(a, b):
    return float(a @ b / (np.linalg.norm(a) * np.linalg.norm(b)))


def test_one_sparse_gradients_motivating_example(oracle):
    import torch
    from paper_2405_11095_amd import binding as B, inputs
    dev = torch.device("cuda:0")
    d, M, R, K = 1024, 4, 20000, 8   # K = 8 dithers on the downlink cut its variance by 8 (Def. 3.2)
    rng = np.random.default_rng(2024)
    js = rng.choice(d, size=M, replace=False)
    cs = np.array([-3.0, -1.5, -2.0, 0.5])          # the mean points mostly in negative directions
    gs = [inputs.one_sparse(d, int(j), float(c)) for j, c in zip(js, cs)]
    mean = np.mean([g.astype(np.float64) for g in gs], axis=0)

    # baseline: coordinate-wise signs (sign(0) = +1) and majority vote, no flattening
    votes = np.sum([np.where(g >= 0, 1, -1) for g in gs], axis=0)
    majority = np.where(votes >= 0, 1.0, -1.0)
    assert np.all(majority == 1.0)                   # the example's point: the vote ignores the gradients
    assert abs(_cos(majority, mean)) < 0.1           # here: -0.047, and its sign is set by the c_n alone

    gd = [torch.from_numpy(g).to(dev) for g in gs]
    out = {}
    for name, dither in (("fo_sgd", B.DITHER_UNIFORM), ("no_dither", B.DITHER_NONE)):
        plan = B.Plan(d=d, M=M, K=K, seed=31, dither=dither)
        acc = torch.zeros(d, dtype=torch.float64, device=dev)
        x = torch.zeros(d, dtype=torch.float32, device=dev)
        for rnd in range(R):
            x.zero_()
            plan.fo_step(gd, x, 1.0, rnd)             # x = -g^d
            acc -= x.double()
        out[name] = (acc / R).cpu().numpy()
        plan.close()
    cos_fo, cos_nd = _cos(out["fo_sgd"], mean), _cos(out["no_dither"], mean)
    rel = np.linalg.norm(out["fo_sgd"] - mean) / np.linalg.norm(mean)
    print(f"cosine with the true mean: majority vote {_cos(majority, mean):+.3f}, FO-SGD {cos_fo:+.3f} "
          f"(rel. error of the {R}-round average {rel:.3f}), flattened sign without dither {cos_nd:+.3f}")
    assert cos_fo > 0.9
    assert cos_nd > 0.0
    # unbiasedness: the R-round average approaches the mean at the Monte Carlo rate (decoded vectors have norm
    # lambda^s sqrt(n) each, independent over rounds)
    assert rel < 0.5
