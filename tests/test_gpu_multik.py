"""K-fold averaged downlink quantiser (Def. 3.2 with K > 1; Sec. 4, "Server-to-workers encoding") on the GPU:
whole rounds against the oracle stage by stage, the server-party encode on its own, and the 1/K law of the
quantiser's second moment (Lemma "Second moment of the quantizer") measured on the GPU's own output."""
import numpy as np
import pytest

from tests import parity as P

pytestmark = pytest.mark.gpu
SERVER = 0xFFFFFFFF


@pytest.fixture(scope="module")
def env(oracle):
    import torch
    from paper_2405_11095_amd import binding as B, inputs
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return oracle, B, inputs, torch.device("cuda:0")


@pytest.mark.parametrize("name,d,M,blk,K,kw", [
    ("single_pass_K2", 20_000, 3, 0, 2, {}),
    ("two_pass_K3", 100_000, 3, 0, 3, {}),
    ("small_blocks_K5", 5_000, 2, 7, 5, {}),
    ("blocks_4096_K8", 300_000, 2, 12, 8, {}),
    ("eight_planes_K255", 70_000, 2, 0, 255, {}),
    ("no_dither_K3", 40_000, 2, 0, 3, dict(dither=1)),
    ("three_pass_K3", (1 << 25) + 5, 1, 0, 3, {}),
    ("shared_eps_two_pass_K2", 90_000, 3, 0, 2, dict(eps_mode=1)),
    ("shared_eps_single_pass_K6", 9_000, 3, 0, 6, dict(eps_mode=1)),
    ("all_shared_two_pass_K4", 90_000, 3, 0, 4, dict(eps_mode=2)),
])
def test_round_trip_with_averaged_downlink(env, name, d, M, blk, K, kw):
    O, B, inputs, dev = env
    gs = [inputs.gaussian(d, m) for m in range(M)]
    rep = P.check_round_trip(O, B, gs, d, M, blk, seed=0xF05D + 40 + K, rnd=6, delta=1e-3, device=dev, K=K, **kw)
    print(name, rep)
    P.gates(rep)


@pytest.mark.parametrize("d,blk,K", [(50_000, 0, 4), (9_000, 8, 6), (150_000, 16, 3), (60_000, 0, 1), (3_000, 10, 1)])
def test_server_party_encode_and_decode(env, d, blk, K):
    """fo_encode / fo_decode for the server party use the K-fold quantiser on their own as well."""
    import torch
    O, B, inputs, dev = env
    plan = B.Plan(d=d, M=1, block_log2=blk, K=K, seed=77, alpha=2.0, alpha_s=2.5)
    p = O.params(d=d, M=1, block_log2=blk, K=K, seed=77, alpha=2.0, alpha_s=2.5)
    b, nb, nt = O.geometry(p)
    x = np.zeros(nt, dtype=np.float32)
    x[:d] = inputs.gaussian(d, 1)
    planes = torch.zeros((plan.planes, plan.W), dtype=torch.int64, device=dev)
    lam = torch.zeros(nb, dtype=torch.float32, device=dev)
    plan.fo_encode(torch.from_numpy(x).to(dev), 3, SERVER, planes, lam)
    out = torch.zeros(d, dtype=torch.float32, device=dev)
    plan.fo_decode(planes, lam, 3, SERVER, out)
    torch.cuda.synchronize()
    h_lam = lam.cpu().numpy()
    r = O.encode(p, x[:d].astype(np.float64), 3, SERVER, K=K, lam=h_lam.astype(np.float64), want_margin=True)
    q_gpu = P.planes_to_code(planes.cpu().numpy().view(np.uint64), nt, K)
    bad, exempt, raw = P.compare_codes(q_gpu, r["q"], r["margin"], h_lam, b)
    assert bad == 0, (bad, exempt, raw)
    # the server party's own measured-norm amplitude carries alpha_s: the encoder's rule with that factor
    p_s = O.params(d=d, M=1, block_log2=blk, K=K, seed=77, alpha=2.5, alpha_s=2.5)
    free = O.encode(p_s, x[:d].astype(np.float64), 3, SERVER, K=K)["lam"]
    assert np.max(np.abs(h_lam - free) / np.where(free > 0, free, 1.0)) <= 1e-6
    dec = O.decode(p, q_gpu, h_lam.astype(np.float64), 3, SERVER, K=K)[:d]
    assert P.rel_l2(out.cpu().numpy(), dec) <= 1e-5
    plan.close()


def test_second_moment_falls_as_one_over_K(env):
    """E ||Z_{lambda,K}(x) - x||^2 = (lambda^2 n - ||x||^2) / K when ||H_eps x||_inf <= lambda: measured on the GPU
    for K = 1, 4, 16 over a few rounds (n = 2^16 coordinates average the dither well)."""
    import torch
    O, B, inputs, dev = env
    d = 1 << 16
    x = inputs.gaussian(d, 2)
    xd = torch.from_numpy(x).to(dev)
    nx2 = float(np.sum(x.astype(np.float64) ** 2))
    for K in (1, 4, 16):
        plan = B.Plan(d=d, M=1, K=K, seed=123)
        planes = torch.zeros((plan.planes, plan.W), dtype=torch.int64, device=dev)
        lam = torch.zeros(1, dtype=torch.float32, device=dev)
        out = torch.zeros(d, dtype=torch.float32, device=dev)
        errs = []
        for rnd in range(8):
            plan.fo_encode(xd, rnd, SERVER, planes, lam)
            plan.fo_decode(planes, lam, rnd, SERVER, out)
            errs.append(float(((out - xd).double() ** 2).sum()))
        l = float(lam[0])
        want = (l * l * d - nx2) / K
        got = float(np.mean(errs))
        assert abs(got - want) <= 0.02 * want, (K, got, want)
        plan.close()


@pytest.mark.parametrize("name,d,M,blk,kw", [
    ("single_pass", 20_000, 3, 0, {}),
    ("blocked_small", 6_000, 2, 7, {}),
    ("blocked_4096", 300_000, 3, 12, {}),
    ("two_pass", 100_000, 4, 0, {}),
    ("two_pass_K3", 100_000, 3, 0, dict(K=3)),
    ("blocked_65536", (1 << 18) + 9, 2, 16, {}),
    ("shared_eps_two_pass", 90_000, 3, 0, dict(eps_mode=1)),
    ("shared_eps_single_pass", 9_000, 3, 0, dict(eps_mode=1)),
    ("three_pass", (1 << 25) + 5, 1, 0, {}),
    ("n2p25", 25_557_032, 2, 0, {}),
    ("all_shared_single_pass", 9_000, 3, 0, dict(eps_mode=2)),
    ("all_shared_blocked_small", 7_000, 5, 6, dict(eps_mode=2)),
    ("all_shared_blocked_128", 7_000, 4, 7, dict(eps_mode=2)),
    ("all_shared_blocked_512", 70_000, 3, 9, dict(eps_mode=2)),
    ("all_shared_two_pass_K2", 200_000, 16, 0, dict(eps_mode=2, K=2)),
])
def test_measured_norm_server_amplitude(env, name, d, M, blk, kw):
    """FO_SERVER_SCALE_L2: lambda^s = alpha_s sqrt(ln b / b) ||gbar_block|| from the mean the server has just formed."""
    O, B, inputs, dev = env
    gs = [inputs.heavy_tailed(d, m) for m in range(M)]
    rep = P.check_round_trip(O, B, gs, d, M, blk, seed=0xABC + M, rnd=5, delta=1e-3, device=dev, server_scale=1, **kw)
    print(name, rep)
    P.gates(rep)


def test_measured_norm_rule_shrinks_the_downlink_error(env):
    """Same uplink messages, two server rules.  E||decode - gbar||^2 = (lambda^s)^2 n - ||gbar||^2 (K = 1).  The mean
    of M independently quantised vectors has ||gbar||^2 of about lambda^2 n / M (quantisation noise dominates), so
    the theorem's rule, which allows for ||gbar|| = lambda sqrt(n), is about M times the measured-norm rule."""
    import torch
    O, B, inputs, dev = env
    d, M = 1 << 16, 4
    gs = [torch.from_numpy(inputs.gaussian(d, m)).to(dev) for m in range(M)]
    err, lam_s_of = {}, {}
    for rule in (0, 1):
        plan = B.Plan(d=d, M=M, seed=5, server_scale=rule)
        bits = torch.zeros((M, plan.W), dtype=torch.int64, device=dev)
        lam = torch.zeros((M, 1), dtype=torch.float32, device=dev)
        for m in range(M):
            plan.fo_encode(gs[m], 1, m, bits[m], lam[m])
        down = torch.zeros((plan.planes, plan.W), dtype=torch.int64, device=dev)
        lam_s = torch.zeros(1, dtype=torch.float32, device=dev)
        gbar = torch.zeros(plan.ntot, dtype=torch.float32, device=dev)
        out = torch.zeros(d, dtype=torch.float32, device=dev)
        plan.fo_server_aggregate(bits, lam, 1, down, lam_s, gbar)
        plan.fo_decode(down, lam_s, 1, SERVER, out)
        torch.cuda.synchronize()
        nb2 = float((gbar.double() ** 2).sum())
        err[rule] = float(((out - gbar[:d]).double() ** 2).sum())
        lam_s_of[rule] = float(lam_s[0])
        # the identity above holds exactly for every draw: the decoded vector has norm lambda^s sqrt(n) and the
        # cross term <decode, gbar> has mean ||gbar||^2; check it loosely on this one draw
        want = lam_s_of[rule] ** 2 * d - nb2
        assert abs(err[rule] - want) < 0.1 * want, (rule, err[rule], want)
        plan.close()
    ratio = err[0] / err[1]
    assert 0.6 * M < ratio < 1.6 * M, (err, lam_s_of, ratio)
