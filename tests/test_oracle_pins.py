"""Pins for the CPU oracle: every check compares the oracle with something other than itself --
the paper's identities and closed forms (arXiv 2405.11095), dense definitions built here with
NumPy, brute force on tiny inputs, or published known-answer vectors.  No GPU is used."""
import math
import os

import numpy as np
import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden")
SERVER = 0xFFFFFFFF


def kron_hadamard(k):
    """Def. 3.4's recursion H_k = [[1,1],[1,-1]] (x) H_{k-1}, built with numpy.kron."""
    H = np.array([[1.0]])
    for _ in range(k):
        H = np.kron(np.array([[1.0, 1.0], [1.0, -1.0]]), H)
    return H


def eps_vec(O, p, rnd, party, n):
    return O.eps(p.seed, rnd, O.eps_party(p.eps_mode, party), np.arange(n))


# ------------------------------------------------------------------ generator
def test_philox_known_answers(oracle):
    rows = [l.split() for l in open(os.path.join(GOLD, "philox4x32_10_kat.txt")) if l[0] != "#"]
    assert len(rows) == 3
    for r in rows:
        v = [int(t, 16) for t in r]
        out = oracle.philox4x32_10(v[0:4], v[4:6])
        assert [int(o) for o in out] == v[6:10]


def test_rng_key_separation(oracle):
    """Distinct (seed, domain, round, party, k, counter) tuples give unrelated blocks."""
    base = dict(seed=7, domain=1, rnd=3, party=2, k=0, counter=5)
    ref = oracle.rng(**base)
    for key, val in [("seed", 8), ("seed", 7 + (1 << 32)), ("domain", 2), ("rnd", 4),
                     ("rnd", 3 + (1 << 32)), ("party", 3), ("party", SERVER), ("k", 1), ("counter", 6)]:
        o = oracle.rng(**{**base, key: val})
        assert not np.array_equal(o, ref)
        # about half of the 128 bits differ
        diff = sum(bin(int(a) ^ int(b)).count("1") for a, b in zip(o, ref))
        assert 32 <= diff <= 96


def test_eps_balance_and_independence(oracle):
    n = 1 << 14
    e0 = oracle.eps(11, 0, 0, np.arange(n))
    e1 = oracle.eps(11, 0, 1, np.arange(n))
    e2 = oracle.eps(11, 1, 0, np.arange(n))
    assert set(np.unique(e0)) == {-1.0, 1.0}
    s = 4.5 * math.sqrt(n)
    for a in (e0, e1, e2):
        assert abs(a.sum()) < s
    for a, b in ((e0, e1), (e0, e2), (e1, e2), (e0[:-1], e0[1:]), (e0[:-64], e0[64:])):
        assert abs((a * b).sum()) < s


def test_dither_grid_and_uniformity(oracle):
    n = 1 << 15
    u = oracle.dither_u(5, 9, 3, 0, np.arange(n))
    m = u * 2.0 ** 24
    assert np.all(m == np.round(m)) and np.all(np.abs(m) % 2 == 1)      # odd multiples of 2^-24
    assert np.all(np.abs(u) < 1.0) and not np.any(u == 0.0)
    assert abs(u.mean()) < 4.5 / math.sqrt(3 * n)
    assert abs((u * u).mean() - 1.0 / 3.0) < 4.5 * math.sqrt(4.0 / 45.0 / n)
    # Kolmogorov-Smirnov distance from U(-1,1)
    us = np.sort(u)
    cdf = (us + 1.0) / 2.0
    ks = np.max(np.abs(cdf - (np.arange(n) + 0.5) / n))
    assert ks < 1.95 / math.sqrt(n)
    # different dither index k, party or round: uncorrelated streams
    for other in (oracle.dither_u(5, 9, 3, 1, np.arange(n)), oracle.dither_u(5, 9, 4, 0, np.arange(n)),
                  oracle.dither_u(5, 10, 3, 0, np.arange(n))):
        assert abs((u * other).mean()) < 4.5 / 3.0 / math.sqrt(n)
    # neighbouring coordinates (which share a generator call) and stride-64 neighbours
    assert abs((u[:-1] * u[1:]).mean()) < 4.5 / 3.0 / math.sqrt(n)
    assert abs((u[:-64] * u[64:]).mean()) < 4.5 / 3.0 / math.sqrt(n)


# ------------------------------------------------------------------ transform (Def. 3.4)
@pytest.mark.parametrize("k", [0, 1, 2, 3, 4])
def test_sylvester_matches_entry_formula_and_kron(oracle, k):
    n = 1 << k
    H = oracle.sylvester(k)
    F = np.array([[(-1.0) ** bin(i & j).count("1") for j in range(n)] for i in range(n)])
    assert np.array_equal(H, F)
    assert np.array_equal(H, kron_hadamard(k))
    assert np.array_equal(H @ H, n * np.eye(n))              # calH calH = n I: H/sqrt(n) orthonormal
    assert np.all(np.abs(H / math.sqrt(n)) == 1 / math.sqrt(n))  # universal sensing basis


@pytest.mark.parametrize("k", [1, 4, 7, 12])
def test_fast_transform_equals_dense(oracle, k):
    n = 1 << k
    x = np.random.default_rng(k).standard_normal(n)
    y = oracle.fwht(x)
    yd = oracle.wht_dense(x)
    assert np.allclose(y, yd, rtol=0, atol=1e-12 * np.abs(yd).max() * k)
    if k <= 10:
        assert np.allclose(y, kron_hadamard(k) @ x, rtol=0, atol=1e-12 * np.abs(y).max() * k)
    assert np.allclose(oracle.fwht(y), n * x, rtol=0, atol=1e-11 * n)
    assert abs(np.linalg.norm(y) - math.sqrt(n) * np.linalg.norm(x)) < 1e-11 * np.linalg.norm(y)


# ------------------------------------------------------------------ randomised basis (Def. 3.5)
def test_encoder_flattens_with_H_eps(oracle):
    """z = H D_eps x (flip BEFORE the transform), checked against a dense numpy product."""
    d = 256
    p = oracle.params(d=d, seed=21)
    x = np.random.default_rng(0).standard_normal(d)
    r = oracle.encode(p, x, rnd=4, party=2, want_z=True)
    e = eps_vec(oracle, p, 4, 2, d)
    H = kron_hadamard(8) / 16.0
    assert np.allclose(r["z"], H @ (e * x), atol=1e-13)
    assert not np.allclose(r["z"], e * (H @ x), atol=1e-3)           # the other order differs
    assert abs(np.linalg.norm(r["z"]) - np.linalg.norm(x)) < 1e-12   # orthogonality (Remark 5.2)
    # H_eps^{-1} = D_eps H^T recovers x
    assert np.allclose(e * (H.T @ r["z"]), x, atol=1e-13)


def test_decoder_is_lambda_D_eps_Ht(oracle):
    d = 128
    p = oracle.params(d=d, seed=3)
    q = np.random.default_rng(1).choice([-1, 1], size=d).astype(np.int32)
    lam = np.array([0.37])
    out = oracle.decode(p, q, lam, rnd=8, party=5)
    e = eps_vec(oracle, p, 8, 5, d)
    H = kron_hadamard(7) / math.sqrt(d)
    assert np.allclose(out, 0.37 * e * (H.T @ q), atol=1e-14)
    # K-averaged code: divide by K (Def. 3.8)
    q3 = np.random.default_rng(2).choice([-3, -1, 1, 3], size=d).astype(np.int32)
    out3 = oracle.decode(p, q3, lam, rnd=8, party=5, K=3)
    assert np.allclose(out3, (0.37 / 3) * e * (H.T @ q3), atol=1e-14)


def test_one_sparse_is_perfectly_flat(oracle):
    """x = c e_j  =>  |z_i| = |c|/sqrt(n) for all i, sign = eps_j (-1)^{popcount(i&j)} sgn(c)."""
    d, j, c = 512, 77, -2.5
    p = oracle.params(d=d, seed=99)
    x = np.zeros(d); x[j] = c
    r = oracle.encode(p, x, rnd=0, party=0, want_z=True)
    e = eps_vec(oracle, p, 0, 0, d)
    walsh = np.array([(-1.0) ** bin(i & j).count("1") for i in range(d)])
    assert np.allclose(r["z"], c * e[j] * walsh / math.sqrt(d), atol=1e-15)


# ------------------------------------------------------------------ quantizer moments (Lemma A.4-A.6)
def test_quantizer_mean_is_clip(oracle):
    lam = 0.8
    x = np.array([-1.5, -0.8, -0.79, -0.4, 0.0, 0.1, 0.5, 0.8, 1.2]) * 1.0
    R = 20000
    acc = np.zeros_like(x)
    for rnd in range(R):
        acc += lam * oracle.quantize(x, lam, seed=1, rnd=rnd, party=0)
    mean = acc / R
    clip = np.clip(x, -lam, lam)
    sd = np.sqrt(np.maximum(lam * lam - clip * clip, 0.0) / R)
    assert np.all(np.abs(mean - clip) <= 4.5 * sd + 1e-12)
    # saturation is deterministic; the residual is the soft threshold (statement 2)
    assert abs(mean[0] + lam) < 1e-9 and abs(mean[-1] - lam) < 1e-9
    soft = np.sign(x) * np.maximum(np.abs(x) - lam, 0.0)
    assert np.all(np.abs((x - mean) - soft) <= 4.5 * sd + 1e-12)


@pytest.mark.parametrize("K", [1, 3, 8])
def test_quantizer_mse_identity(oracle, K):
    """E || Q_{lam,K}(x) - x ||^2 = (lam^2 n - ||x||^2) / K for ||x||_inf <= lam."""
    n, lam, R = 64, 1.0, 4000
    x = np.random.default_rng(5).uniform(-1, 1, n)
    errs = np.empty(R)
    for rnd in range(R):
        q = oracle.quantize(x, lam, K=K, seed=2, rnd=rnd, party=1)
        assert set(np.unique(q)) <= set(range(-K, K + 1, 2))            # Remark 3.3
        errs[rnd] = np.sum((lam / K * q - x) ** 2)
    want = (lam * lam * n - x @ x) / K
    assert abs(errs.mean() - want) < 4.5 * errs.std() / math.sqrt(R)


def test_quantizer_inner_product_identity(oracle):
    """E <x, Q_lam(y)>^2 = <x,y>^2 + ||x||^2 lam^2 - sum x_i^2 y_i^2  (||y||_inf <= lam)."""
    n, lam, R = 32, 0.5, 20000
    g = np.random.default_rng(6)
    x, y = g.standard_normal(n), g.uniform(-lam, lam, n)
    vals = np.empty(R)
    for rnd in range(R):
        vals[rnd] = (x @ (lam * oracle.quantize(y, lam, seed=3, rnd=rnd, party=0))) ** 2
    want = (x @ y) ** 2 + (x @ x) * lam * lam - np.sum(x * x * y * y)
    assert abs(vals.mean() - want) < 4.5 * vals.std() / math.sqrt(R)


def test_bit_probability_brute_force(oracle):
    """P(bit = +1) = clip((z + lam) / (2 lam), 0, 1): frequency over dither draws, n = 16."""
    lam, R = 1.0, 30000
    z = np.linspace(-1.2, 1.2, 16)
    cnt = np.zeros(16)
    for rnd in range(R):
        cnt += oracle.quantize(z, lam, seed=4, rnd=rnd, party=7) > 0
    pr = np.clip((z + lam) / (2 * lam), 0, 1)
    assert np.all(np.abs(cnt / R - pr) <= 4.5 * np.sqrt(pr * (1 - pr) / R) + 1e-12)


def test_sign_of_zero_is_plus_one(oracle):
    q = oracle.quantize(np.array([0.0, -0.0, 1e-300, -1e-300]), 1.0, dither=oracle.DITHER_NONE)
    assert list(q) == [1, 1, 1, -1]
    # zero gradient: lam = 0, every bit is 1, the decoded vector is exactly 0
    p = oracle.params(d=200, seed=1)
    r = oracle.encode(p, np.zeros(200), rnd=0, party=0)
    assert r["lam"][0] == 0.0 and np.all(r["bits"] == np.uint64(0xFFFFFFFFFFFFFFFF))
    assert np.all(oracle.decode(p, r["q"], r["lam"], 0, 0) == 0.0)


# ------------------------------------------------------------------ flattening (Lemma 3.6)
def test_flattening_tail_bound(oracle):
    n, alpha, R = 64, 2.0, 3000
    x = np.zeros(n); x[:3] = [3.0, -2.0, 1.0]           # a sparse, hard-to-flatten vector
    p = oracle.params(d=n, seed=77)
    thr = alpha * math.sqrt(math.log(n) / n) * np.linalg.norm(x)
    bad = 0
    for rnd in range(R):
        z = oracle.encode(p, x, rnd=rnd, party=0, want_z=True)["z"]
        bad += np.max(np.abs(z)) > thr
    bound = 2.0 * math.exp(-0.25 * alpha * alpha * math.log(n))
    assert bad / R <= bound + 4.5 * math.sqrt(bound / R)


# ------------------------------------------------------------------ codec (Def. 3.7, 3.8, 5.1, Remark 5.2)
@pytest.mark.parametrize("K", [1, 4])
def test_round_trip_norm(oracle, K):
    d = 1024
    p = oracle.params(d=d, seed=5)
    for x in (np.random.default_rng(3).standard_normal(d), np.zeros(d)):
        lam = np.array([0.3])
        r = oracle.encode(p, x, rnd=1, party=0, K=K, lam=lam)
        out = oracle.decode(p, r["q"], lam, 1, 0, K=K)
        if K == 1:
            assert abs(np.linalg.norm(out) - 0.3 * math.sqrt(d)) < 1e-12
        else:
            assert np.linalg.norm(out) <= 0.3 * math.sqrt(d) + 1e-12


def test_lambda_rule(oracle):
    """lam = alpha B sqrt(log n / n) with natural log (Thm 5.5); L2 rule takes B = ||g||_2."""
    d = 4096
    x = np.random.default_rng(8).standard_normal(d)
    p = oracle.params(d=d, alpha=2.5, scale_rule=oracle.SCALE_L2)
    lam = oracle.encode(p, x, 0, 0)["lam"][0]
    assert math.isclose(lam, 2.5 * np.linalg.norm(x) * math.sqrt(math.log(d) / d), rel_tol=1e-14)
    p = oracle.params(d=d, alpha=3.0, B=7.0, scale_rule=oracle.SCALE_BOUND)
    lam = oracle.encode(p, x, 0, 0)["lam"][0]
    assert math.isclose(lam, 3.0 * 7.0 * math.sqrt(math.log(d) / d), rel_tol=1e-14)
    # hypothesis the analysis uses: on the flattening event ||H_eps g||_inf <= lam
    r = oracle.encode(oracle.params(d=d, seed=2), x, 0, 0, want_z=True)
    assert np.max(np.abs(r["z"])) <= r["lam"][0]


def test_transform_mse_matches_lemma_on_flat_event(oracle):
    """E_tau ||Z_{lam,K}(x) - x||^2 = (lam^2 n - ||x||^2)/K when ||H_eps x||_inf <= lam, and the
    upper bound alpha^2 B^2 log n / K + 8 B^2 exp(-alpha^2 log n / 8) of Lemma A.9 holds."""
    d, R = 256, 1500
    x = np.random.default_rng(9).standard_normal(d)
    B = np.linalg.norm(x)
    for K in (1, 4):
        p = oracle.params(d=d, seed=10, eps_mode=oracle.EPS_SHARED_ALL)
        errs = np.empty(R)
        for rnd in range(R):
            # dither keyed by round; eps also changes with the round, the identity holds for each
            r = oracle.encode(p, x, rnd, 0, K=K, want_z=True)
            assert np.max(np.abs(r["z"])) <= r["lam"][0]
            out = oracle.decode(p, r["q"], r["lam"], rnd, 0, K=K)
            errs[rnd] = np.sum((out - x) ** 2)
        lam = r["lam"][0]
        want = (lam * lam * d - B * B) / K
        assert abs(errs.mean() - want) < 4.5 * errs.std() / math.sqrt(R)
        a = 2.0
        assert errs.mean() <= a * a * B * B * math.log(d) / K + 8 * B * B * math.exp(-a * a * math.log(d) / 8)


# ------------------------------------------------------------------ server (Sec. 4) and full round
def _uplink(O, p, gs, rnd, lam=None):
    enc = [O.encode(p, g.astype(np.float64), rnd, m, lam=lam) for m, g in enumerate(gs)]
    return np.stack([e["bits"] for e in enc]), np.stack([e["lam"] for e in enc])


def test_server_mean_is_average_of_decodes(oracle):
    d, M = 300, 3                      # padded to 512
    p = oracle.params(d=d, M=M, seed=12)
    gs = [np.random.default_rng(20 + m).standard_normal(d).astype(np.float32) for m in range(M)]
    bits, lams = _uplink(oracle, p, gs, 2)
    s = oracle.server(p, bits, lams, 2, want_margin=True)
    n = 512
    H = kron_hadamard(9) / math.sqrt(n)
    want = np.zeros(n)
    for m in range(M):
        q = oracle.unpack(bits[m], n).astype(np.float64)
        want += lams[m, 0] * eps_vec(oracle, p, 2, m, n) * (H.T @ q)
    want /= M
    assert np.allclose(s["gbar"], want, atol=1e-13)
    # server amplitude: lam_s = alpha_s * max lam * sqrt(log n); the analysis needs
    # lam_s >= alpha_s sqrt(log n / n) ||gbar||, which follows from ||gbar|| <= lam sqrt(n)
    assert math.isclose(s["lam_s"][0], 2.0 * lams.max() * math.sqrt(math.log(n)), rel_tol=1e-14)
    assert s["lam_s"][0] >= 2.0 * math.sqrt(math.log(n) / n) * np.linalg.norm(s["gbar"])
    # downlink bits are the (eps_s, lam_s)-encoder of gbar
    es = eps_vec(oracle, p, 2, SERVER, n)
    zs = H @ (es * s["gbar"])
    us = oracle.dither_u(p.seed, 2, SERVER, 0, np.arange(n))
    assert np.allclose(s["margin"], zs + s["lam_s"][0] * us, atol=1e-12)
    assert np.array_equal(oracle.unpack(s["bits_down"], n) > 0, s["margin"] >= 0)


def test_identical_workers_average_to_one_decode(oracle):
    """Same bits from every worker (shared eps, no dither): the mean equals a single decode, and
    lam_s = alpha_s sqrt(log n / n) ||gbar|| holds with equality (||gbar|| = lam sqrt(n))."""
    d, M = 256, 5
    p = oracle.params(d=d, M=M, seed=1, eps_mode=oracle.EPS_SHARED_WORKERS, dither=oracle.DITHER_NONE)
    g = np.random.default_rng(30).standard_normal(d).astype(np.float32)
    bits, lams = _uplink(oracle, p, [g] * M, 0)
    assert all(np.array_equal(bits[0], b) for b in bits)
    s = oracle.server(p, bits, lams, 0)
    one = oracle.decode(p, oracle.unpack(bits[0], d), lams[0], 0, 0)
    assert np.allclose(s["gbar"], one, atol=1e-14)
    assert math.isclose(s["lam_s"][0], 2.0 * math.sqrt(math.log(d) / d) * np.linalg.norm(s["gbar"]), rel_tol=1e-12)


def test_shared_eps_mean_equals_popcount_formula(oracle):
    """With one eps for all workers and a common lam, linearity of H^T gives
    gbar = (lam / M) D_eps H^T (sum_n q_n) = (lam / M) D_eps H^T (2 c - M), c = per-coordinate popcount."""
    d, M = 512, 7
    p = oracle.params(d=d, M=M, seed=40, eps_mode=oracle.EPS_SHARED_WORKERS)
    gs = [np.random.default_rng(50 + m).standard_normal(d).astype(np.float32) for m in range(M)]
    lam = np.array([0.9])
    bits, lams = _uplink(oracle, p, gs, 3, lam=lam)
    s = oracle.server(p, bits, lams, 3)
    c = sum((oracle.unpack(b, d) > 0).astype(np.int64) for b in bits)
    H = kron_hadamard(9) / math.sqrt(d)
    e = eps_vec(oracle, p, 3, 0, d)
    assert np.array_equal(e, eps_vec(oracle, p, 3, 4, d))
    assert np.allclose(s["gbar"], (0.9 / M) * e * (H.T @ (2 * c - M)), atol=1e-13)


def test_average_of_M_dithers_is_K_equals_M_quantizer(oracle):
    """Same g and eps on all M workers, independent dithers: E||gbar - g||^2 = (lam^2 n - ||g||^2)/M."""
    d, M, R = 128, 4, 1500
    p = oracle.params(d=d, M=M, seed=60, eps_mode=oracle.EPS_SHARED_WORKERS)
    g = np.random.default_rng(61).standard_normal(d).astype(np.float32)
    errs = np.empty(R)
    for rnd in range(R):
        bits, lams = _uplink(oracle, p, [g] * M, rnd)
        errs[rnd] = np.sum((oracle.server(p, bits, lams, rnd)["gbar"] - g) ** 2)
    lam = lams[0, 0]
    want = (lam * lam * d - float(g.astype(np.float64) @ g.astype(np.float64))) / M
    assert abs(errs.mean() - want) < 4.5 * errs.std() / math.sqrt(R)


def test_all_shared_eps_server_identity_and_unbiasedness(oracle):
    """Server sharing the workers' eps (a variant outside the paper): (i) its pre-quantisation vector is
    (lam / M)(2 c - M) exactly, because H D_eps D_eps H^T = I; (ii) the decoded downlink message stays an unbiased
    estimate of the workers' mean over rounds (the quantiser-moment lemma needs |z| <= lam^s, which holds surely
    here since |2 c - M| <= M and lam <= lam^s)."""
    d, M = 64, 3
    p = oracle.params(d=d, M=M, seed=90, eps_mode=oracle.EPS_SHARED_ALL)
    gs = [np.random.default_rng(91 + m).standard_normal(d).astype(np.float32) for m in range(M)]
    lam = np.array([1.3])
    bits, lams = _uplink(oracle, p, gs, 5, lam=lam)
    s = oracle.server(p, bits, lams, 5, want_margin=True)
    c = sum((oracle.unpack(b, d) > 0).astype(np.int64) for b in bits)
    u = np.asarray(oracle.dither_u(p.seed, 5, 0xFFFFFFFF, 0, np.arange(d))).reshape(d)
    assert np.allclose(s["margin"], (1.3 / M) * (2 * c - M) + s["lam_s"][0] * u, atol=1e-12)
    # unbiasedness of the whole round over fresh eps and dithers
    R = 6000
    mean = np.zeros(d)
    want = np.mean([g.astype(np.float64) for g in gs], axis=0)
    lam_s = None
    for rnd in range(R):
        x = np.zeros(d)
        o = oracle.round_trip(p, gs, x, 1.0, rnd, want=True)
        mean += o["gd"] / R
        lam_s = o["lam_s"][0]
    # every decoded coordinate has second moment (lam^s)^2 (the decoded vector has norm lam^s sqrt(n))
    assert np.max(np.abs(mean - want)) < 5.0 * lam_s / math.sqrt(R)


def test_all_shared_eps_admits_the_workers_amplitude_for_the_server(oracle):
    """Rule SUP (all-shared eps only): lambda^s = lambda.  The server's vector (lam / M)(2 c - M) is bounded by lam
    in every coordinate, so (i) nothing is ever clipped, (ii) the quantiser stays unbiased (first-moment lemma of
    Def. 3.2: E Q = z whenever ||z||_inf <= lambda^s), checked by Monte Carlo over rounds, and (iii) the decoded
    message's error drops by the factor alpha_s^2 ln n of the theorem's rule: with K = 1 every decoded coordinate
    has magnitude lambda^s, so E ||g^d - mean||^2 = n (lambda^s)^2 - ||w||^2 (second-moment lemma)."""
    d, M = 64, 3
    ps = oracle.params(d=d, M=M, seed=190, eps_mode=oracle.EPS_SHARED_ALL, server_scale=oracle.SERVER_SCALE_SUP)
    pt = oracle.params(d=d, M=M, seed=190, eps_mode=oracle.EPS_SHARED_ALL)
    gs = [np.random.default_rng(191 + m).standard_normal(d).astype(np.float32) for m in range(M)]
    lam = np.array([0.9])
    bits, lams = _uplink(oracle, ps, gs, 7, lam=lam)
    s, st = oracle.server(ps, bits, lams, 7, want_margin=True), oracle.server(pt, bits, lams, 7)
    assert s["lam_s"][0] == 0.9 and np.isclose(st["lam_s"][0], 2.0 * 0.9 * math.sqrt(math.log(d)), rtol=1e-13)
    assert np.array_equal(s["gbar"], st["gbar"])
    c = sum((oracle.unpack(b, d) > 0).astype(np.int64) for b in bits)
    w = (0.9 / M) * (2 * c - M)
    assert np.max(np.abs(w)) <= 0.9
    u = np.asarray(oracle.dither_u(ps.seed, 7, 0xFFFFFFFF, 0, np.arange(d))).reshape(d)
    assert np.allclose(s["margin"], w + 0.9 * u, atol=1e-12)
    # coordinates at the bound are quantised deterministically: |u| < 1, so sign(w + lam u) = sign(w)
    at_bound = np.abs(w) == 0.9
    assert np.array_equal(np.sign(s["margin"][at_bound]), np.sign(w[at_bound]))
    R = 4000
    want = np.mean([g.astype(np.float64) for g in gs], axis=0)
    mean_s, err_s, err_t = np.zeros(d), 0.0, 0.0
    for rnd in range(R):
        o = oracle.round_trip(ps, gs, np.zeros(d), 1.0, rnd, want=True)
        mean_s += o["gd"] / R
        err_s += float(np.sum((o["gd"] - o["gbar"][:d]) ** 2)) / R
        lam_s = o["lam_s"][0]
        if rnd < 400:
            ot = oracle.round_trip(pt, gs, np.zeros(d), 1.0, rnd, want=True)
            err_t += float(np.sum((ot["gd"] - ot["gbar"][:d]) ** 2)) / 400
    assert np.max(np.abs(mean_s - want)) < 5.0 * lam_s / math.sqrt(R)
    # downlink error: n lam_s^2 - ||w||^2 on average, against n (alpha_s^2 ln n) lam^2 - ||w||^2 for the theorem's rule
    assert err_s < d * lam_s ** 2 and err_t > 0.5 * (4.0 * math.log(d)) * err_s


def test_measured_norm_server_amplitude(oracle):
    """Server rule L2: lambda^s = alpha_s sqrt(ln n / n) ||gbar||, per block; it is the smallest amplitude the
    server lemma of Thm 5.5 admits, never larger than the theorem's rule (||gbar|| <= lambda sqrt(n)), and the
    flattening event ||H_eps^s gbar||_inf <= lambda^s it is chosen for fails with probability <= 2 n^(-alpha_s^2/4)
    over eps^s (Lemma 3.6), here <= 2/n per round."""
    d, M, blk = 600, 3, 8                       # three blocks of 256, the last one padded
    p = oracle.params(d=d, M=M, block_log2=blk, seed=70, server_scale=oracle.SERVER_SCALE_L2)
    pt = oracle.params(d=d, M=M, block_log2=blk, seed=70)
    gs = [np.random.default_rng(80 + m).standard_normal(d).astype(np.float32) for m in range(M)]
    b, nb, nt = oracle.geometry(p)
    bits, lams = _uplink(oracle, p, gs, 4)
    s, st = oracle.server(p, bits, lams, 4, want_margin=True), oracle.server(pt, bits, lams, 4)
    assert np.array_equal(s["gbar"], st["gbar"])
    norms = np.linalg.norm(s["gbar"].reshape(nb, b), axis=1)
    assert np.allclose(s["lam_s"], 2.0 * math.sqrt(math.log(b) / b) * norms, rtol=1e-13)
    assert np.all(s["lam_s"] <= st["lam_s"])
    # the downlink message is the (eps^s, lambda^s)-encoding of gbar with that amplitude
    us = oracle.dither_u(p.seed, 4, SERVER, 0, np.arange(nt))
    r = oracle.encode(oracle.params(d=nt, M=M, block_log2=blk, seed=70), s["gbar"], 4, SERVER, lam=s["lam_s"], want_margin=True, want_z=True)
    assert np.allclose(s["margin"], r["z"] + np.repeat(s["lam_s"], b) * us, atol=1e-12)
    # flattening event over rounds (fresh eps^s each round)
    fails, R = 0, 400
    for rnd in range(R):
        bits, lams = _uplink(oracle, p, gs, rnd)
        sr = oracle.server(p, bits, lams, rnd)
        z = oracle.encode(oracle.params(d=nt, M=M, block_log2=blk, seed=70), sr["gbar"], rnd, SERVER, lam=sr["lam_s"], want_z=True)["z"]
        fails += int(np.count_nonzero(np.abs(z) > np.repeat(sr["lam_s"], b)))
    assert fails <= 50                      # Lemma 3.6 allows up to 2 R nb = 2400 in expectation; observed: 1


def test_padding_and_blocking(oracle):
    d = 200
    x = np.random.default_rng(70).standard_normal(d)
    xp = np.concatenate([x, np.zeros(56)])
    p, pp = oracle.params(d=d, seed=9), oracle.params(d=256, seed=9)
    a, b = oracle.encode(p, x, 1, 0, want_z=True), oracle.encode(pp, xp, 1, 0, want_z=True)
    assert oracle.geometry(p) == (256, 1, 256)
    assert np.array_equal(a["bits"], b["bits"]) and np.array_equal(a["z"], b["z"]) and a["lam"][0] == b["lam"][0]
    # a single block of the full length is the unblocked codec
    pb = oracle.params(d=256, seed=9, block_log2=8)
    c = oracle.encode(pb, xp, 1, 0)
    assert np.array_equal(c["bits"], b["bits"]) and c["lam"][0] == b["lam"][0]
    # blocks are independent transforms with their own amplitude, indexed by global coordinate
    pb = oracle.params(d=256, seed=9, block_log2=6)
    c = oracle.encode(pb, xp, 1, 0, want_z=True)
    assert oracle.geometry(pb) == (64, 4, 256)
    H = kron_hadamard(6) / 8.0
    e = eps_vec(oracle, pb, 1, 0, 256)
    u = oracle.dither_u(9, 1, 0, 0, np.arange(256))
    for j in range(4):
        sl = slice(64 * j, 64 * j + 64)
        assert np.allclose(c["z"][sl], H @ (e[sl] * xp[sl]), atol=1e-14)
        assert math.isclose(c["lam"][j], 2.0 * np.linalg.norm(xp[sl]) * math.sqrt(math.log(64) / 64), rel_tol=1e-13)
        assert np.array_equal(c["q"][sl] > 0, c["z"][sl] + c["lam"][j] * u[sl] >= 0)
    out = oracle.decode(pb, c["q"], c["lam"], 1, 0)
    for j in range(4):
        sl = slice(64 * j, 64 * j + 64)
        assert np.allclose(out[sl], c["lam"][j] * e[sl] * (H.T @ c["q"][sl]), atol=1e-14)


def test_full_round_is_the_composition(oracle):
    """x_{t+1} = x_t - delta * D^s(E^s((1/M) sum_n D_n(E_n(g_n)))), first d coordinates."""
    d, M, delta = 700, 4, 0.25
    p = oracle.params(d=d, M=M, seed=80)
    gs = [np.random.default_rng(90 + m).standard_normal(d).astype(np.float32) for m in range(M)]
    x0 = np.random.default_rng(99).standard_normal(d)
    x = x0.copy()
    o = oracle.round_trip(p, gs, x, delta, rnd=6, nthreads=2, want=True)
    bits, lams = _uplink(oracle, p, gs, 6)
    assert np.array_equal(o["bits_up"], bits) and np.array_equal(o["lam_up"], lams)
    s = oracle.server(p, bits, lams, 6)
    assert np.array_equal(o["bits_down"], s["bits_down"]) and np.array_equal(o["gbar"], s["gbar"])
    gd = oracle.decode(p, s["q_down"], s["lam_s"], 6, SERVER)[:d]
    assert np.array_equal(o["gd"], gd)
    assert np.array_equal(x, x0 - delta * gd)
    # the decoded update correlates positively with the true mean gradient
    gm = np.mean([g.astype(np.float64) for g in gs], axis=0)
    assert gd @ gm > 0


def test_dither_and_eps_streams_do_not_collide(oracle):
    """Distinct coordinates must draw distinct generator outputs: the number of equal 24-bit
    values among n draws stays at the birthday level n^2 / 2^25, and lags that are natural
    collision candidates of a wrong counter mapping (32, 128, 256, 4096) are uncorrelated."""
    n = 1 << 15
    u = oracle.dither_u(5, 9, 3, 0, np.arange(n))
    dup = n - np.unique(u).size
    assert dup < 4 * n * n / 2 ** 25 + 20
    e = oracle.eps(5, 9, 3, np.arange(n))
    for lag in (1, 2, 32, 64, 128, 256, 4096):
        assert abs((u[:-lag] * u[lag:]).mean()) < 4.5 / 3.0 / math.sqrt(n - lag)
        assert abs((e[:-lag] * e[lag:]).mean()) < 4.5 / math.sqrt(n - lag)


def test_stream_layout_matches_the_stated_mapping(oracle):
    """The coordinate -> (generator call, word, bits) mapping stated in the oracle's comments,
    recomputed here from raw generator blocks: eps: call i>>7, word (i>>5)&3, bit i&31, set = -1;
    dither: call ((i>>8)<<6)|(i&63), word (i>>6)&3, top 24 bits."""
    seed, rnd, party = 0xABCDEF0123, 17, 6
    for i in (0, 1, 31, 32, 63, 64, 127, 128, 255, 256, 1000, 65535, 65536, (1 << 25) + 12345):
        w = oracle.rng(seed, oracle.DOMAIN_EPS, rnd, party, 0, i >> 7)
        bit = (int(w[(i >> 5) & 3]) >> (i & 31)) & 1
        assert oracle.eps(seed, rnd, party, [i])[0] == (-1.0 if bit else 1.0)
        for k in (0, 2):
            w = oracle.rng(seed, oracle.DOMAIN_DITHER, rnd, party, k, ((i >> 8) << 6) | (i & 63))
            r = int(w[(i >> 6) & 3]) >> 8
            assert oracle.dither_u(seed, rnd, party, k, [i])[0] == (2 * r + 1 - 2 ** 24) / 2 ** 24


def test_block_range_equals_full(oracle):
    """Encoding / decoding a range of blocks alone gives the same result as the whole vector."""
    d = 1000                                 # 16 blocks of 64 -> 1024
    p = oracle.params(d=d, seed=3, block_log2=6)
    x = np.random.default_rng(4).standard_normal(d)
    full = oracle.encode(p, x, 2, 1, want_margin=True)
    part = oracle.encode_blocks(p, x[64 * 13:], 2, 1, j0=13, nj=3, want_margin=True)
    assert np.array_equal(part["q"], full["q"][64 * 13:]) and np.array_equal(part["lam"], full["lam"][13:])
    assert np.array_equal(part["margin"], full["margin"][64 * 13:]) and np.array_equal(part["bits"], full["bits"][13:])
    dec = oracle.decode(p, full["q"], full["lam"], 2, 1)
    decp = oracle.decode_blocks(p, full["q"][64 * 5:64 * 9], full["lam"][5:9], 2, 1, j0=5, nj=4)
    assert np.array_equal(decp, dec[64 * 5:64 * 9])


def test_encoder_is_homogeneous(oracle):
    """E(c x) = E(x) with amplitude c lambda for c > 0 (the rule lambda = alpha ||x|| sqrt(ln n / n) scales with x and
    the quantiser only looks at signs of z + lambda u): exact for c a power of two, where no rounding changes."""
    d = 3000
    x = np.random.default_rng(21).standard_normal(d)
    for blk in (0, 8):
        p = oracle.params(d=d, seed=8, block_log2=blk)
        ref = oracle.encode(p, x, 3, 1)
        for k in (-20, 7):
            r = oracle.encode(p, np.ldexp(x, k), 3, 1)
            assert np.array_equal(r["bits"], ref["bits"])
            assert np.array_equal(r["lam"], np.ldexp(ref["lam"], k))


def test_single_entries_of_the_transform_and_bulk_eps(oracle):
    """The helpers behind the sampled checks of transforms too long to run whole: single entries of H x against
    the Kronecker-built matrix, and the bulk eps draw against the per-coordinate one."""
    k = 9
    n = 1 << k
    x = np.random.default_rng(12).standard_normal(n)
    idx = np.array([0, 1, 2, 77, 255, 256, n - 1], dtype=np.uint64)
    want = kron_hadamard(k) @ x
    got = oracle.wht_rows(np.ascontiguousarray(x), idx)
    assert np.allclose(got, want[idx.astype(int)], rtol=0, atol=1e-11)
    e = oracle.eps_fill(11, 5, 3, 1000, 700)                     # straddles generator blocks of 128
    assert np.array_equal(e, oracle.eps(11, 5, 3, np.arange(1000, 1700)))
    assert set(np.unique(e)) == {-1.0, 1.0}


def test_oracle_is_clean_under_host_sanitizers(tmp_path):
    """The oracle, driven through whole rounds on exactly sized arrays, under AddressSanitizer and
    UndefinedBehaviorSanitizer (host only): no out-of-bounds access, no undefined operation."""
    import os
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = str(tmp_path / "orc_selftest")
    cc = subprocess.run(["gcc", "-std=c11", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                         "-static-libasan", "-static-libubsan", "-o", exe, os.path.join(root, "oracle", "selftest.c"), "-lm", "-lpthread"],
                        capture_output=True, text=True)
    if cc.returncode != 0 and "sanitize" in cc.stderr:
        pytest.skip("this gcc has no sanitizer runtime")
    assert cc.returncode == 0, cc.stderr
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert run.stdout.count("checksum") == 5


def test_pack_layout_against_numpy_little_endian_bits(oracle):
    """Packing format: word w, bit j <-> coordinate 64 w + j, set bit = +1.  Pinned to NumPy's own little-endian
    bit (un)packing of the same bytes and to single-coordinate spikes, so that a slip on one side or a consistent
    one on both sides of pack / unpack (bit order inside a word, word order, polarity) fails here."""
    rng = np.random.default_rng(77)
    n = 64 * 37
    q = (2 * rng.integers(0, 2, n) - 1).astype(np.int32)
    bits = oracle.pack(q)
    assert bits.dtype == np.uint64 and bits.size == n // 64
    want = np.packbits((q > 0).astype(np.uint8), bitorder="little").view("<u8")
    assert np.array_equal(bits, want)
    got = np.unpackbits(bits.view(np.uint8), bitorder="little")[:n]
    assert np.array_equal(got.astype(bool), q > 0)
    assert np.array_equal(oracle.unpack(want, n), q)
    for i in (0, 1, 31, 32, 63, 64, 65, 127, 64 * 36 + 63):
        e = -np.ones(n, dtype=np.int32)
        e[i] = 1
        b = oracle.pack(e)
        assert int(b[i // 64]) == 1 << (i % 64) and np.count_nonzero(b) == 1
        w = np.zeros(n // 64, dtype=np.uint64)
        w[i // 64] = np.uint64(1) << np.uint64(i % 64)
        assert np.array_equal(oracle.unpack(w, n), e)
