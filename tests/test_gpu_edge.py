"""GPU edge cases and full-size workloads, through the C ABI, against the CPU oracle."""
import numpy as np
import pytest

from tests.parity import SERVER, check_round_trip, check_sampled_blocks, gates

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env(oracle):
    import torch
    from paper_2405_11095_amd import binding, inputs
    assert torch.cuda.is_available()
    binding.load_library()
    return oracle, binding, inputs, torch.device("cuda:0")


def _encode(B, torch, dev, plan, g, rnd, party, flags=0, scales=None):
    bits = torch.zeros(plan.W, dtype=torch.int64, device=dev)
    lam = torch.zeros(plan.nblocks, dtype=torch.float32, device=dev) if scales is None else scales
    plan.fo_encode(torch.from_numpy(g).to(dev), rnd, party, bits, lam, flags)
    torch.cuda.synchronize()
    return bits, lam


@pytest.mark.parametrize("d,blk", [(1 << 15, 0), (1 << 16, 0), (3 << 16, 16), (1 << 18, 0), (1 << 14, 10), (1000, 6)])
def test_decode_of_walsh_rows_is_a_spike(env, d, blk):
    """A message that is row j of the Walsh matrix decodes to lambda sqrt(b) eps_j e_j: the largest value an inverse
    transform can produce (all b signs add up), elsewhere exact zeros.  j = 0 is the all-ones message.  Exercises
    the integer decode paths at the end of their range (2^14, 2^15 and 2^16 in half values) and their offsets."""
    import torch
    O, B, inputs, dev = env
    plan = B.Plan(d=d, M=2, block_log2=blk, seed=19)
    p = O.params(d=d, M=2, block_log2=blk, seed=19)
    b, nb, nt = O.geometry(p)
    lam = np.linspace(1.0, 2.0, nb).astype(np.float32)
    i = np.arange(b, dtype=np.uint64)
    rs = np.random.default_rng(5)
    for j in [0, 1, 31, 32, 33, b // 2, b - 1, int(rs.integers(0, b)), int(rs.integers(0, b))]:
        par = np.zeros(b, dtype=np.uint64)
        x = i & np.uint64(j)
        for sh in (32, 16, 8, 4, 2, 1):                        # parity of popcount(i & j)
            x ^= x >> np.uint64(sh)
        q_blk = 1 - 2 * (x & np.uint64(1)).astype(np.int32)    # (-1)^popcount(i & j)
        q = np.tile(q_blk, nb)
        bits = O.pack(q)
        for party in (1, SERVER):
            out = torch.zeros(d, dtype=torch.float32, device=dev)
            plan.fo_decode(torch.from_numpy(bits.view(np.int64)).to(dev), torch.from_numpy(lam).to(dev), 4, party, out)
            torch.cuda.synchronize()
            want = O.decode(p, q, lam.astype(np.float64), 4, party)[:d]
            got = out.cpu().numpy().astype(np.float64)
            spikes = np.arange(nb) * b + j
            spikes = spikes[spikes < d]
            assert np.count_nonzero(want) == spikes.size and np.all(np.abs(want[spikes]) > 0)
            assert np.array_equal(got != 0, want != 0), (j, party)
            assert np.allclose(got[spikes], want[spikes], rtol=1e-6, atol=0), (j, party)
    plan.close()


@pytest.mark.parametrize("d,blk", [(1 << 25, 0), (1 << 17, 15), (1 << 16, 12), (1 << 18, 16)])
def test_extreme_messages_through_the_server(env, d, blk):
    """Both workers send the all-ones message: the inverse transform's value at the first coordinate of a block is
    b, the largest integer the decode side ever holds (for n = 2^25: 2^24 in half values in the fp32 stages of the
    server pass, still exact).  Mean, downlink bits and one worker decode against the oracle, for the two-pass
    server, the single-tile mean kernel and blocks of two tiles."""
    import torch
    O, B, inputs, dev = env
    M, rnd = 2, 6
    plan = B.Plan(d=d, M=M, block_log2=blk, seed=23)
    p = O.params(d=d, M=M, block_log2=blk, seed=23)
    b, nb, nt = O.geometry(p)
    W = nt // 64
    bits_up = torch.full((M, W), -1, dtype=torch.int64, device=dev)
    lam_up = torch.tensor([[1.0] * nb, [0.5] * nb], dtype=torch.float32, device=dev)
    bits_down = torch.zeros(W, dtype=torch.int64, device=dev)
    lam_s = torch.zeros(nb, dtype=torch.float32, device=dev)
    gbar = torch.zeros(nt, dtype=torch.float32, device=dev)
    out = torch.zeros(d, dtype=torch.float32, device=dev)
    plan.fo_server_aggregate(bits_up, lam_up, rnd, bits_down, lam_s, gbar)
    plan.fo_decode(bits_up[1], lam_up[1], rnd, 1, out)
    torch.cuda.synchronize()
    h_up = bits_up.cpu().numpy().view(np.uint64)
    s = O.server(p, h_up, lam_up.cpu().numpy().astype(np.float64), rnd, lam_s=lam_s.cpu().numpy().astype(np.float64),
                 want_margin=True)
    h_gbar = gbar.cpu().numpy().astype(np.float64)
    first = np.arange(nb) * b
    assert np.count_nonzero(s["gbar"]) == nb and np.count_nonzero(h_gbar) == nb
    assert np.all(np.abs(h_gbar[first] - s["gbar"][first]) <= 1e-6 * np.abs(s["gbar"][first]))
    from tests.parity import compare_bits
    bad, exempt, raw = compare_bits(bits_down.cpu().numpy().view(np.uint64), s["margin"], lam_s.cpu().numpy(), b)
    assert bad == 0, (bad, exempt, raw)
    dec = O.decode(p, O.unpack(h_up[1], nt), lam_up[1].cpu().numpy().astype(np.float64), rnd, 1)[:d]
    h_out = out.cpu().numpy().astype(np.float64)
    assert np.count_nonzero(h_out) == nb and np.all(np.abs(h_out[first] - dec[first]) <= 1e-6 * np.abs(dec[first]))
    plan.close()


@pytest.mark.parametrize("d,blk", [(1000, 0), (70_000, 0), (5000, 7), (50_000, 0), (200_000, 16)])
def test_zero_gradient(env, d, blk):
    """sign(0) = +1: every bit is set, lambda = 0, the decoded vector and the update are exactly 0."""
    import torch
    O, B, inputs, dev = env
    plan = B.Plan(d=d, M=2, block_log2=blk, seed=9)
    g = np.zeros(d, dtype=np.float32)
    g[1::2] = -0.0
    bits, lam = _encode(B, torch, dev, plan, g, 3, 0)
    assert torch.all(lam == 0)
    assert np.all(bits.cpu().numpy().view(np.uint64) == np.uint64(0xFFFFFFFFFFFFFFFF))
    out = torch.full((d,), 7.0, dtype=torch.float32, device=dev)
    plan.fo_decode(bits, lam, 3, 0, out)
    x = torch.ones(d, dtype=torch.float32, device=dev)
    gz = torch.from_numpy(g).to(dev)
    plan.fo_step([gz, gz], x, 0.5, 3)
    torch.cuda.synchronize()
    assert torch.all(out == 0) and torch.all(x == 1)


def test_nan_input_is_defined(env):
    """A NaN entry makes the norm, hence lambda, NaN: every comparison is false (all bits 0) and the
    decoded vector is NaN; nothing faults."""
    import torch
    O, B, inputs, dev = env
    d = 4096
    plan = B.Plan(d=d, M=1, seed=1)
    g = inputs.gaussian(d, 0)
    g[17] = np.nan
    bits, lam = _encode(B, torch, dev, plan, g, 0, 0)
    assert torch.isnan(lam).all()
    assert np.all(bits.cpu().numpy() == 0)
    out = torch.zeros(d, dtype=torch.float32, device=dev)
    plan.fo_decode(bits, lam, 0, 0, out)
    torch.cuda.synchronize()
    assert torch.isnan(out).all()


def test_determinism_and_seed_sensitivity(env):
    import torch
    O, B, inputs, dev = env
    d = 100_000
    g = inputs.heavy_tailed(d, 0)
    p1, p2, p3 = B.Plan(d=d, M=1, seed=5), B.Plan(d=d, M=1, seed=5), B.Plan(d=d, M=1, seed=6)
    b1, l1 = _encode(B, torch, dev, p1, g, 4, 0)
    b2, l2 = _encode(B, torch, dev, p2, g, 4, 0)
    b3, _ = _encode(B, torch, dev, p3, g, 4, 0)
    b4, _ = _encode(B, torch, dev, p1, g, 5, 0)
    assert torch.equal(b1, b2) and torch.equal(l1, l2)
    for other in (b3, b4):
        diff = (b1 ^ other).cpu().numpy().view(np.uint64)
        frac = sum(bin(int(w)).count("1") for w in diff[:2000]) / (2000 * 64)
        assert 0.3 < frac < 0.7


@pytest.mark.parametrize("d,blk", [(100_000, 0), (40_000, 0), (300_000, 12), (200_000, 16)])
def test_scaling_by_a_power_of_two_changes_only_the_amplitude(env, d, blk):
    """The codec is homogeneous: g -> 2^k g scales every fp32 intermediate exactly, so the message is the same bit
    for bit and the amplitude is 2^k times the old one (k = +-40: well inside the fp32 range of the norms)."""
    import torch
    O, B, inputs, dev = env
    g = inputs.gaussian(d, 4)
    plan = B.Plan(d=d, M=1, block_log2=blk, seed=29)
    ref, lref = _encode(B, torch, dev, plan, g, 2, 0)
    for k in (-40, 40):
        b, l = _encode(B, torch, dev, plan, np.ldexp(g, k).astype(np.float32), 2, 0)
        assert torch.equal(b, ref)
        assert torch.equal(l, torch.ldexp(lref, torch.tensor(k, device=dev)))
    plan.close()


@pytest.mark.parametrize("blk", [0, 12, 16])
def test_repeat_encodes_agree_large(env, blk):
    """Ten encodes of one 2^22-coordinate vector give the same 65536 words every time (the packed words
    travel through scalar registers and lane writes, where a missed wait state shows up as rare stale words).
    Block lengths: one long transform, single-tile blocks, and blocks of two tiles (two groups of a workgroup
    that must agree on the amplitude to the bit)."""
    import torch
    O, B, inputs, dev = env
    d = 1 << 22
    g = inputs.gaussian(d, 3)
    plan = B.Plan(d=d, M=1, seed=11, block_log2=blk)
    ref, lref = _encode(B, torch, dev, plan, g, 9, 0)
    for _ in range(9):
        b, l = _encode(B, torch, dev, plan, g, 9, 0)
        assert torch.equal(b, ref) and torch.equal(l, lref)


@pytest.mark.parametrize("name,kw", [
    ("bound_rule", dict(scale_rule=0, Bnorm=400.0)),
    ("no_dither", dict(dither=1)),
    ("alpha3", dict(alpha=3.0, alpha_s=2.5)),
    ("bound_rule_b65536", dict(scale_rule=0, Bnorm=400.0, block_log2=16)),
    ("no_dither_b65536", dict(dither=1, block_log2=16)),
])
def test_parameter_variants(env, name, kw):
    O, B, inputs, dev = env
    d, M = 150_000, 3
    gs = [inputs.gaussian(d, m) for m in range(M)]
    kw = dict(kw)
    rep = check_round_trip(O, B, gs, d=d, M=M, block_log2=kw.pop("block_log2", 0), seed=77, rnd=2, delta=0.1, device=dev, **kw)
    print(name, rep, flush=True)
    gates(rep)


@pytest.mark.parametrize("name,d,M,blk,K", [
    ("single_pass", 30_000, 5, 0, 1),
    ("blocked_small", 7_000, 3, 7, 1),
    ("blocked", 200_003, 4, 12, 3),
    ("two_pass", (1 << 18) + 11, 7, 0, 1),
    ("blocked_b65536", (1 << 18) + 11, 3, 16, 2),
    ("n2p25", 25_557_032, 3, 0, 1),
    ("three_pass", (1 << 25) + 5, 2, 0, 1),
])
def test_all_shared_eps_zero_transform_server(env, name, d, M, blk, K):
    """The server shares the workers' eps: its pre-quantisation vector is (lambda / M)(2 c - M) and the kernel
    applies no transform.  The oracle takes the long way (M decodes, mean, forward transform with the same eps),
    so this checks the identity H D_eps D_eps H^T = I the shortcut rests on, to the bit."""
    O, B, inputs, dev = env
    gs = [inputs.heavy_tailed(d, m) for m in range(M)]
    rep = check_round_trip(O, B, gs, d=d, M=M, block_log2=blk, seed=0x77 + M, rnd=13, delta=0.02, device=dev,
                           eps_mode=B.EPS_SHARED_ALL, K=K)
    print(name, rep, flush=True)
    gates(rep)


@pytest.mark.parametrize("name,d,M,blk,K", [
    ("single_pass", 30_000, 5, 0, 1),
    ("blocked", 200_003, 4, 12, 3),
    ("two_pass", (1 << 18) + 11, 7, 0, 1),
    ("blocked_b65536", (1 << 18) + 11, 3, 16, 2),
])
def test_all_shared_eps_with_the_workers_amplitude_for_the_server(env, name, d, M, blk, K):
    """FO_SERVER_SCALE_SUP: with the server sharing the workers' eps its vector is bounded by lambda in every
    coordinate, so lambda^s = lambda is admissible (Def. 3.2's first-moment lemma); amplitudes, downlink bits, decode
    and update against the oracle's long way round, and the coordinates that sit at the bound included."""
    O, B, inputs, dev = env
    gs = [inputs.heavy_tailed(d, m) for m in range(M)]
    rep = check_round_trip(O, B, gs, d=d, M=M, block_log2=blk, seed=0x99 + M, rnd=17, delta=0.02, device=dev,
                           eps_mode=B.EPS_SHARED_ALL, K=K, server_scale=B.SERVER_SCALE_SUP)
    print(name, rep, flush=True)
    gates(rep)


@pytest.mark.parametrize("d,blk,eps_mode", [(20_000, 0, 0), (50_000, 0, 0), (300_000, 0, 0), (70_000, 10, 0),
                                            (200_000, 16, 1), (5_000, 7, 2)])
def test_worker_message_decode(env, d, blk, eps_mode):
    """fo_decode of a worker's own message (the call a hand-rolled server would make): D_{eps_n,lambda_n}(q_n)
    against the oracle's decoder, for a worker other than 0 (its own eps stream unless the mode shares it)."""
    import torch
    O, B, inputs, dev = env
    M, m, rnd = 3, 2, 5
    plan = B.Plan(d=d, M=M, block_log2=blk, seed=91, eps_mode=eps_mode)
    p = O.params(d=d, M=M, block_log2=blk, seed=91, eps_mode=eps_mode)
    b, nb, nt = O.geometry(p)
    g = inputs.heavy_tailed(d, m)
    bits = torch.zeros(plan.W, dtype=torch.int64, device=dev)
    lam = torch.zeros(nb, dtype=torch.float32, device=dev)
    out = torch.zeros(d, dtype=torch.float32, device=dev)
    plan.fo_encode(torch.from_numpy(g).to(dev), rnd, m, bits, lam)
    plan.fo_decode(bits, lam, rnd, m, out)
    torch.cuda.synchronize()
    h_lam = lam.cpu().numpy().astype(np.float64)
    q = O.unpack(bits.cpu().numpy().view(np.uint64), nt)      # +-1
    dec = O.decode(p, q, h_lam, rnd, m)[:d]
    from tests.parity import rel_l2
    assert rel_l2(out.cpu().numpy(), dec) <= 1e-5
    # and the round trip is the paper's estimator: norm lambda sqrt(b) per block (every entry of q is +-1)
    full = np.zeros(nt)
    full[:d] = out.cpu().numpy()
    if d == nt:
        assert np.allclose(np.linalg.norm(full.reshape(nb, b), axis=1), h_lam * np.sqrt(b), rtol=1e-5)
    plan.close()


def test_forced_scale_is_used(env):
    import torch
    O, B, inputs, dev = env
    d = 50_000
    plan = B.Plan(d=d, M=1, seed=3)
    g = inputs.gaussian(d, 0)
    forced = torch.full((1,), 0.123, dtype=torch.float32, device=dev)
    bits, lam = _encode(B, torch, dev, plan, g, 1, 0, flags=B.FORCE_SCALE, scales=forced)
    assert float(lam[0]) == np.float32(0.123)
    p = O.params(d=d, M=1, seed=3)
    r = O.encode(p, g.astype(np.float64), 1, 0, lam=np.array([float(np.float32(0.123))]), want_margin=True)
    from tests.parity import compare_bits
    bad, exempt, _ = compare_bits(bits.cpu().numpy().view(np.uint64), r["margin"], [0.123], plan.b)
    assert bad == 0


def test_argument_errors(env):
    import torch
    O, B, inputs, dev = env
    plan = B.Plan(d=1000, M=2, seed=1)
    g = torch.zeros(1004, dtype=torch.float32, device=dev)
    bits = torch.zeros(plan.W, dtype=torch.int64, device=dev)
    lam = torch.zeros(1, dtype=torch.float32, device=dev)
    with pytest.raises(B.FoError) as e:
        plan.fo_encode(g, 0, 2, bits, lam)            # party out of range
    assert e.value.code == B.EINVAL
    with pytest.raises(B.FoError) as e:
        plan.fo_encode(g[1:], 0, 0, bits, lam)        # gradient not 16-byte aligned
    assert e.value.code == B.EALIGN
    with pytest.raises(B.FoError) as e:
        plan.fo_encode(g, 0, 0, bits, lam, flags=8)   # unknown flag
    assert e.value.code == B.EINVAL


def test_single_worker_and_odd_worker_counts(env):
    O, B, inputs, dev = env
    for M in (1, 5):
        d = (1 << 20) + 3
        gs = [inputs.gaussian(d, m) for m in range(M)]
        rep = check_round_trip(O, B, gs, d=d, M=M, block_log2=0, seed=31 + M, rnd=9, delta=0.1, device=dev)
        print(M, rep, flush=True)
        gates(rep)


def test_three_pass_transform(env):
    """n = 2^26: two strided passes around the contiguous one."""
    O, B, inputs, dev = env
    d, M = (1 << 26) - 12345, 1
    gs = [inputs.gaussian(d, 0)]
    rep = check_round_trip(O, B, gs, d=d, M=M, block_log2=0, seed=5, rnd=1, delta=0.1, device=dev)
    print(rep, flush=True)
    gates(rep)


def test_c2_sparse_workload(env):
    """1 % dense gradients are flattened: no coordinate of H_eps g exceeds lambda (event A of Thm 5.5)."""
    O, B, inputs, dev = env
    d, M = 1 << 20, 8
    gs = inputs.workload("c2")
    rep = check_round_trip(O, B, gs, d=d, M=M, block_log2=0, seed=0xF05D + 2, rnd=0, delta=0.01, device=dev)
    print(rep, flush=True)
    gates(rep)
    p = O.params(d=d, M=M, seed=0xF05D + 2)
    r = O.encode(p, gs[0].astype(np.float64), 0, 0, want_z=True)
    assert np.max(np.abs(r["z"])) <= r["lam"][0]
    assert np.max(np.abs(gs[0])) / np.sqrt(np.mean(gs[0].astype(np.float64) ** 2)) > 5 * np.max(np.abs(r["z"])) / np.sqrt(np.mean(r["z"] ** 2))


@pytest.mark.parametrize("blk", [10, 12, 14, 16])
def test_c4_full_size_sampled_blocks(env, blk):
    """d = 2^27, M = 8, layered dynamic range: the whole round on the GPU, oracle on sampled blocks."""
    O, B, inputs, dev = env
    d, M = 1 << 27, 8
    gs = inputs.workload("c4")
    nb = d >> blk
    nj = max(1, (1 << 17) >> blk)                      # 2^17 coordinates per sampled range
    ranges = [(0, nj), (nb // 2 + 3, nj), (nb - nj, nj)]
    rep = check_sampled_blocks(O, B, gs, d=d, M=M, block_log2=blk, seed=0xF05D + 4, rnd=0, device=dev, block_ranges=ranges)
    print(rep, flush=True)
    assert rep["uplink_mismatch"] == 0 and rep["downlink_mismatch"] == 0, rep
    assert rep["lam_rel_err"] <= 1e-6 and rep["lam_s_rel_err"] <= 1e-6, rep
    assert rep["decode_rel_l2"] <= 1e-5, rep


@pytest.mark.parametrize("name,d,M,blk", [
    ("single_pass", 30_000, 5, 0),
    ("blocked", 200_003, 4, 12),
    ("two_pass", (1 << 18) + 11, 7, 0),
    ("blocked_b65536", (1 << 18) + 11, 5, 16),
    ("n2p25", 25_557_032, 3, 0),
    ("three_pass", (1 << 25) + 5, 2, 0),
])
def test_shared_worker_eps_popcount_server(env, name, d, M, blk):
    """One eps and one amplitude for all workers: the server sums the packed sign vectors per
    coordinate and runs a single inverse transform.  The oracle forms the mean the long way (M
    decodes), so this checks the shortcut against the unshortened formula."""
    O, B, inputs, dev = env
    gs = [inputs.heavy_tailed(d, m) for m in range(M)]
    rep = check_round_trip(O, B, gs, d=d, M=M, block_log2=blk, seed=0x5A + M, rnd=11, delta=0.02, device=dev,
                           eps_mode=B.EPS_SHARED_WORKERS)
    print(name, rep, flush=True)
    gates(rep)


def test_diagnostic_counters(env):
    """fo_stats: coordinates where the flattening failed (|z_i| > lambda, expected none for alpha = 2 on dense
    inputs, some when lambda is forced small) and near-tie coordinates, against counts made from the oracle's
    flattened vector."""
    import torch
    O, B, inputs, dev = env
    d, M = 200_000, 2
    plan = B.Plan(d=d, M=M, seed=21)
    p = O.params(d=d, M=M, seed=21)
    stats = torch.zeros(2 * (B.MAX_WORKERS + 1), dtype=torch.int64, device=dev)
    plan.fo_set_stats(stats)
    gs = [inputs.gaussian(d, m) for m in range(M)]
    x = torch.zeros(d, dtype=torch.float32, device=dev)
    plan.fo_step([torch.from_numpy(g).to(dev) for g in gs], x, 0.1, 2)
    torch.cuda.synchronize()
    h = stats.cpu().numpy()
    assert np.all(h[:B.MAX_WORKERS + 1] == 0)                       # nothing clipped: alpha = 2 flattens
    assert h[B.MAX_WORKERS + 1:].sum() < 50                         # a handful of near ties out of 3 * 2^18
    # force a small amplitude on worker 1: now a known share of the coordinates exceeds it
    stats.zero_()
    lam_free = torch.zeros(1, dtype=torch.float32, device=dev)
    bits = torch.zeros(plan.W, dtype=torch.int64, device=dev)
    g1 = torch.from_numpy(gs[1]).to(dev)
    plan.fo_encode(g1, 2, 1, bits, lam_free)
    lam_small = lam_free * 0.25
    stats.zero_()
    plan.fo_encode(g1, 2, 1, bits, lam_small, flags=B.FORCE_SCALE)
    torch.cuda.synchronize()
    h = stats.cpu().numpy()
    r = O.encode(p, gs[1].astype(np.float64), 2, 1, lam=lam_small.cpu().numpy().astype(np.float64), want_margin=True, want_z=True)
    lam = float(lam_small[0])
    want_clipped = int(np.count_nonzero(np.abs(r["z"]) > lam))
    want_near = int(np.count_nonzero(np.abs(r["margin"]) < 1e-6 * lam))
    assert want_clipped > 1000
    assert abs(int(h[1]) - want_clipped) <= 3, (h[1], want_clipped)
    assert abs(int(h[B.MAX_WORKERS + 1 + 1]) - want_near) <= 3, (h[B.MAX_WORKERS + 2], want_near)
    assert h[0] == 0 and h[B.MAX_WORKERS] == 0
    plan.fo_set_stats(None)
    plan.close()
    # the counting variants of the K-fold server encode and of the single-tile path: same messages as without counters
    for dd, blk, K in ((70_000, 0, 3), (20_000, 9, 1), (20_000, 0, 2)):
        gs2 = [torch.from_numpy(inputs.gaussian(dd, m)).to(dev) for m in range(M)]
        got = []
        for attach in (False, True):
            pl = B.Plan(d=dd, M=M, block_log2=blk, K=K, seed=33)
            if attach:
                stats.zero_()
                pl.fo_set_stats(stats)
            xx = torch.zeros(dd, dtype=torch.float32, device=dev)
            pl.fo_step(gs2, xx, 0.1, 4)
            torch.cuda.synchronize()
            got.append(xx.clone())
            pl.close()
        assert torch.equal(got[0], got[1])
        assert int(stats[:B.MAX_WORKERS + 1].sum()) == 0
    # blocks of 2^16: with counters the encode takes the two-pass kernels, without them the one-pass kernel.  The two
    # add up the block norms in different orders, so the amplitudes may differ in the last place: same step up to that.
    gs2 = [torch.from_numpy(inputs.gaussian(150_000, m)).to(dev) for m in range(M)]
    got = []
    for attach in (False, True):
        pl = B.Plan(d=150_000, M=M, block_log2=16, seed=34)
        if attach:
            stats.zero_()
            pl.fo_set_stats(stats)
        xx = torch.zeros(150_000, dtype=torch.float32, device=dev)
        pl.fo_step(gs2, xx, 0.1, 4)
        torch.cuda.synchronize()
        got.append(xx.clone())
        pl.close()
    assert float((got[0] - got[1]).norm() / got[0].norm()) < 1e-3  # a near-tie bit may flip with the amplitude's last place
    assert int(stats[:B.MAX_WORKERS + 1].sum()) == 0


def test_caller_streams_and_two_plans(env):
    """All work goes to the caller's stream: two plans driven from two (default-priority) streams at the same time
    give what each gives alone on the default stream."""
    import torch
    O, B, inputs, dev = env
    d, M = 300_000, 3
    gs = [torch.from_numpy(inputs.gaussian(d, m)).to(dev) for m in range(M)]

    def run(plan, stream, rounds):
        x = torch.zeros(d, dtype=torch.float32, device=dev)
        with torch.cuda.stream(stream):
            for r in range(rounds):
                plan.fo_step(gs, x, 0.01, r)
        return x

    p0 = B.Plan(d=d, M=M, seed=3)
    ref = run(p0, torch.cuda.default_stream(), 6)
    torch.cuda.synchronize()
    p1, p2 = B.Plan(d=d, M=M, seed=3), B.Plan(d=d, M=M, seed=3)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    x1 = run(p1, s1, 6)
    x2 = run(p2, s2, 6)
    torch.cuda.synchronize()
    assert torch.equal(x1, ref) and torch.equal(x2, ref)
    for p in (p0, p1, p2):
        p.close()


def test_per_kernel_timing(env):
    """fo_profile_begin / fo_profile_end: every kernel of the step is reported with its launch count and a positive
    time; the times add up to no more than the wall time of the steps."""
    import time
    import torch
    O, B, inputs, dev = env
    d, M = 1 << 18, 4
    gs = [torch.from_numpy(inputs.gaussian(d, m)).to(dev) for m in range(M)]
    x = torch.zeros(d, dtype=torch.float32, device=dev)
    plan = B.Plan(d=d, M=M, seed=8)
    plan.fo_step(gs, x, 0.01, 0)
    torch.cuda.synchronize()
    plan.fo_profile_begin()
    t0 = time.perf_counter()
    for r in range(5):
        plan.fo_step(gs, x, 0.01, r + 1)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    prof = plan.fo_profile_end()
    assert {"k_strided<ENC_FIRST>", "k_contig<IN_F32,OUT_PACK>", "k_declow", "k_strided<SERVER>", "k_strided<DEC_LAST>",
            "scale kernels"} <= set(prof)
    assert prof["k_strided<ENC_FIRST>"][0] == 5 and prof["k_contig<IN_F32,OUT_PACK>"][0] == 10
    assert all(ms > 0 for _, ms in prof.values())
    assert sum(ms for _, ms in prof.values()) <= wall_ms
    with pytest.raises(B.FoError):
        plan.fo_profile_end()          # not recording any more
    plan.close()


def test_resume_needs_only_x_and_the_round(env):
    """The codec keeps no state between rounds (eps and dither are functions of seed, round, party, coordinate):
    a run that is cut after round 3 and continued by a fresh plan from the saved iterate and round number ends where
    the uninterrupted run ends."""
    import torch
    O, B, inputs, dev = env
    d, M = 200_000, 3
    gs = [torch.from_numpy(inputs.gaussian(d, m)).to(dev) for m in range(M)]
    whole = B.Plan(d=d, M=M, seed=17)
    x = torch.zeros(d, dtype=torch.float32, device=dev)
    for r in range(7):
        whole.fo_step(gs, x, 0.01, r)
    first = B.Plan(d=d, M=M, seed=17)
    y = torch.zeros(d, dtype=torch.float32, device=dev)
    for r in range(4):
        first.fo_step(gs, y, 0.01, r)
    torch.cuda.synchronize()
    saved = y.cpu()                       # the checkpoint: iterate and round number
    first.close()
    second = B.Plan(d=d, M=M, seed=17)
    z = saved.to(dev)
    for r in range(4, 7):
        second.fo_step(gs, z, 0.01, r)
    torch.cuda.synchronize()
    assert torch.equal(z, x)
    whole.close()
    second.close()


@pytest.mark.parametrize("d,blk,M", [(50_000, 12, 3), (30_000, 0, 2), ((1 << 17) + 9, 16, 2), (300_000, 0, 3),
                                     ((1 << 24) + 3, 0, 2), ((1 << 25) + 3, 0, 2)])
def test_negative_amplitudes_flip_the_decoded_vector(env, d, blk, M):
    """The decoder is linear in the amplitude, D = lambda D_eps H^T q (Def. 3.8): a caller-supplied negative
    amplitude gives minus the vector of the positive one on every kernel path (single tile, pair, two-pass, the
    matrix-core server pass of n = 2^25, three-pass), and in
    the server's mean a worker with a negated amplitude enters with the opposite sign."""
    import torch
    O, B, inputs, dev = env
    plan = B.Plan(d=d, M=M, block_log2=blk, seed=99)
    W, nb, nt = plan.W, plan.nblocks, plan.ntot
    bits = torch.zeros((M, W), dtype=torch.int64, device=dev)
    lam = torch.zeros((M, nb), dtype=torch.float32, device=dev)
    for m in range(M):
        plan.fo_encode(torch.from_numpy(inputs.gaussian(d, m)).to(dev), 4, m, bits[m], lam[m])
    out_p = torch.zeros(d, dtype=torch.float32, device=dev)
    out_n = torch.zeros(d, dtype=torch.float32, device=dev)
    plan.fo_decode(bits[0], lam[0], 4, 0, out_p)
    plan.fo_decode(bits[0], -lam[0], 4, 0, out_n)
    torch.cuda.synchronize()
    assert float(out_p.abs().max()) > 0 and torch.equal(out_n, -out_p)
    # server: negating worker 1's amplitudes moves the mean by -2/M times that worker's decoded vector
    bd = torch.zeros((plan.planes, W), dtype=torch.int64, device=dev)
    ls = torch.zeros(nb, dtype=torch.float32, device=dev)
    g1 = torch.zeros(nt, dtype=torch.float32, device=dev)
    g2 = torch.zeros(nt, dtype=torch.float32, device=dev)
    plan.fo_server_aggregate(bits, lam, 4, bd, ls, g1)
    lam2 = lam.clone()
    lam2[1] = -lam2[1]
    plan.fo_server_aggregate(bits, lam2, 4, bd, ls, g2)
    torch.cuda.synchronize()
    p = O.params(d=d, M=M, block_log2=blk, seed=99)
    dec1 = O.decode(p, O.unpack(bits[1].cpu().numpy().view(np.uint64), nt), lam[1].cpu().numpy().astype(np.float64), 4, 1)
    want = g1.cpu().numpy().astype(np.float64) - 2.0 * dec1 / M
    from tests.parity import rel_l2
    assert rel_l2(g2.cpu().numpy(), want) < 1e-5
    plan.close()


@pytest.mark.gpu
@pytest.mark.parametrize("d,M,blk,server_scale", [
    ((1 << 24) + 12_345, 3, 0, 0),            # n = 2^25, ragged, the theorem's server amplitude
    ((1 << 25) + 70_001, 2, 25, 1),           # two blocks of 2^25, server amplitude from the measured norm of the mean
    ((1 << 24) + 5, 33, 0, 0),                # an odd, larger number of workers (both parities of the doubled buffers)
])
def test_matrix_core_server_pass_equals_the_vector_unit_one(env, monkeypatch, d, M, blk, server_scale):
    """Blocks of 2^25: the server pass runs its ten inverse stages on the matrix cores (fp16 pieces of exact integers).
    With FO_SERVER_VECTOR_UNIT=1 a plan keeps the vector-unit kernel.  Every product and sum of the matrix-core form is
    exact, so the mean, the downlink amplitudes and the downlink bits of the two plans are identical to the bit."""
    import torch
    O, B, inputs, dev = env
    gs = [torch.from_numpy(inputs.heavy_tailed(d, m)).to(dev) for m in range(M)]
    out = []
    for vector_unit in (False, True):
        if vector_unit:
            monkeypatch.setenv("FO_SERVER_VECTOR_UNIT", "1")
        else:
            monkeypatch.delenv("FO_SERVER_VECTOR_UNIT", raising=False)
        plan = B.Plan(d=d, M=M, block_log2=blk, seed=77, server_scale=server_scale)
        W, nb, nt = plan.W, plan.nblocks, plan.ntot
        bits_up = torch.zeros((M, W), dtype=torch.int64, device=dev)
        lam_up = torch.zeros((M, nb), dtype=torch.float32, device=dev)
        for m in range(M):
            plan.fo_encode(gs[m], 3, m, bits_up[m], lam_up[m])
        bits_down = torch.zeros(W, dtype=torch.int64, device=dev)
        lam_down = torch.zeros(nb, dtype=torch.float32, device=dev)
        gbar = torch.zeros(nt, dtype=torch.float32, device=dev)
        plan.fo_server_aggregate(bits_up, lam_up, 3, bits_down, lam_down, gbar)
        torch.cuda.synchronize()
        plan.fo_profile_begin()
        plan.fo_server_aggregate(bits_up, lam_up, 3, bits_down, lam_down, gbar)
        torch.cuda.synchronize()
        kernels = set(plan.fo_profile_end())
        assert ("k_strided<SERVER>" in kernels) == vector_unit and ("k_server_mfma" in kernels) == (not vector_unit), kernels
        out.append((bits_down.cpu().numpy(), lam_down.cpu().numpy(), gbar.cpu().numpy().view(np.uint32)))
        plan.close()
    assert np.isfinite(out[0][2].view(np.float32)).all() and np.count_nonzero(out[0][2]) > 0.9 * out[0][2].size
    assert np.array_equal(out[0][1], out[1][1])
    assert np.array_equal(out[0][2], out[1][2])
    assert np.array_equal(out[0][0], out[1][0])


@pytest.mark.gpu
@pytest.mark.parametrize("d,blk", [(100_000, 0), (40_000, 9)])
def test_unanimous_workers_pass_the_bound_exactly(env, d, blk):
    """FO_SERVER_SCALE_SUP puts unanimous coordinates exactly at the quantiser's bound: (lambda / M)(2 c - M) = +-lambda
    with lambda^s = lambda.  The dither is an odd multiple of 2^-24 inside (-1, 1), so such a coordinate keeps its
    sign for every draw: all-ones messages come back all ones, all-zero messages all zero, in every round."""
    import torch
    O, B, inputs, dev = env
    M = 5
    plan = B.Plan(d=d, M=M, block_log2=blk, seed=31, eps_mode=B.EPS_SHARED_ALL, server_scale=B.SERVER_SCALE_SUP)
    W, nb = plan.W, plan.nblocks
    lam = torch.rand(nb, dtype=torch.float32, device=dev) + 0.25
    lam_up = lam.repeat(M, 1).contiguous()
    for fill in (-1, 0):
        bits_up = torch.full((M, W), fill, dtype=torch.int64, device=dev)
        for rnd in range(40):
            bits_down = torch.full((W,), 0x5555, dtype=torch.int64, device=dev)
            lam_s = torch.zeros(nb, dtype=torch.float32, device=dev)
            plan.fo_server_aggregate(bits_up, lam_up, rnd, bits_down, lam_s)
            torch.cuda.synchronize()
            assert torch.equal(lam_s, lam)
            assert bool((bits_down == fill).all()), (fill, rnd)
    plan.close()
