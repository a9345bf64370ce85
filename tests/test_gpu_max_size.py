"""The largest vector the C ABI accepts: d = n = 2^30 (three-pass transform, 4 GiB of gradient), one worker.

The oracle cannot run a 2^30-point transform whole inside a test, so every stage is checked on sampled
coordinates that it computes one by one from the definition: entry i of H x is sum_j (-1)^popcount(i & j) x_j
(Def. 3.4 unrolled), an O(n) sum per coordinate in fp64.  Stages are teacher-forced like the full-size tests:
the uplink check uses the GPU's fp32 amplitude, the server check the GPU's uplink bits and mean, the decode
check the GPU's downlink bits."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

SERVER = 0xFFFFFFFF
TIE = 1e-6


def _rows(O, x64, idx, threads=12):
    with ThreadPoolExecutor(max_workers=threads) as ex:
        return np.array(list(ex.map(lambda i: O.wht_rows(x64, [i])[0], idx)))


def _bit(bits, i):
    return int((int(bits[i >> 6]) >> (i & 63)) & 1)


def _signs(bits, n):
    """Packed bits -> +-1 as fp64 (bit 1 <-> +1)."""
    b = np.unpackbits(np.ascontiguousarray(bits).view(np.uint8), bitorder="little")[:n]
    q = b.astype(np.float64)
    q *= 2.0
    q -= 1.0
    return q


def test_sampled_check_on_a_small_ragged_vector(oracle):
    """The same sampled check where the whole-vector tests also run (three passes need n >= 2^26; this is two)."""
    _sampled_check(oracle, (1 << 22) + 77)


@pytest.mark.timeout(900)
def test_largest_vector_on_sampled_coordinates(oracle):
    _sampled_check(oracle, 1 << 30)


def _sampled_check(O, d):
    import torch
    from paper_2405_11095_amd import binding as B, inputs
    dev = torch.device("cuda:0")
    seed, rnd, delta = 0xF05D + 30, 9, 0.25
    plan = B.Plan(d=d, M=1, seed=seed)
    p = O.params(d=d, M=1, seed=seed)
    b, nb, n = O.geometry(p)
    assert (plan.b, plan.nblocks, plan.ntot) == (b, nb, n) and nb == 1 and n >= d
    W = n // 64
    rootn = float(np.sqrt(float(n)))

    g = inputs.gaussian(d, 0)
    g[: d // 4] *= 8.0                                   # a quarter of the coordinates carries most of the norm
    print(f"sampled check: d = {d}, n = {n}, scratch {plan.scratch_bytes / 2**30:.1f} GiB", flush=True)
    gd = torch.from_numpy(g).to(dev)
    bits_up = torch.zeros((1, W), dtype=torch.int64, device=dev)
    lam_up = torch.zeros((1, 1), dtype=torch.float32, device=dev)
    bits_down = torch.zeros((1, W), dtype=torch.int64, device=dev)
    lam_s = torch.zeros(1, dtype=torch.float32, device=dev)
    gbar = torch.zeros(n, dtype=torch.float32, device=dev)
    out = torch.zeros(d, dtype=torch.float32, device=dev)
    plan.fo_encode(gd, rnd, 0, bits_up[0], lam_up[0])
    plan.fo_server_aggregate(bits_up, lam_up, rnd, bits_down, lam_s, gbar)
    plan.fo_decode(bits_down, lam_s, rnd, SERVER, out)
    torch.cuda.synchronize()
    h_bits_up = bits_up[0].cpu().numpy().view(np.uint64)
    h_bits_down = bits_down[0].cpu().numpy().view(np.uint64)
    lam = float(lam_up[0, 0])
    lams = float(lam_s[0])
    print("gpu stages done", flush=True)

    rs = np.random.default_rng(30)
    idx = np.concatenate([[0, 1, n - 1, n // 2, (1 << 15) - 1, 1 << 15, n >> 5, d - 1],
                          rs.integers(0, n, size=4)]).astype(np.uint64)
    idx_int = [int(i) for i in idx]

    # ---- uplink: amplitude rule and sampled sign bits
    x64 = np.zeros(n, dtype=np.float64)
    x64[:d] = g
    del g
    lam_free = O.lam_rule(2.0, float(np.linalg.norm(x64)), n)
    assert abs(lam - lam_free) <= 1e-6 * lam_free, (lam, lam_free)
    e = O.eps_fill(seed, rnd, O.eps_party(0, 0), 0, n)
    x64 *= e
    del e
    z = _rows(O, x64, idx_int) / rootn
    del x64
    u = O.dither_u(seed, rnd, 0, 0, idx)
    margin = z + lam * u
    assert np.max(np.abs(z)) <= lam                      # flattened (Lemma 3.6 at alpha = 2)
    checked = 0
    for i, m in zip(idx_int, margin):
        if abs(m) >= TIE * lam:
            assert _bit(h_bits_up, i) == (1 if m >= 0 else 0), ("uplink", i, m)
            checked += 1
    assert checked >= len(idx_int) - 1
    print("uplink ok", flush=True)

    # ---- server: the mean (one worker: its decode), the amplitude rule, the re-encode of the GPU's mean
    q64 = _signs(h_bits_up, n)
    s_up = _rows(O, q64, idx_int)
    del q64
    e_i = O.eps(seed, rnd, O.eps_party(0, 0), idx)
    want_gbar = lam / rootn * e_i * s_up
    h_gbar = gbar.cpu().numpy()
    got_gbar = h_gbar[idx.astype(np.int64)].astype(np.float64)
    assert np.max(np.abs(got_gbar - want_gbar)) <= 1e-5 * np.max(np.abs(want_gbar)), (got_gbar, want_gbar)
    lams_free = float(O.server_lambda(p, np.array([[lam]], dtype=np.float64))[0])
    assert abs(lams - lams_free) <= 1e-6 * lams_free, (lams, lams_free)
    y64 = h_gbar.astype(np.float64)
    del h_gbar
    # ||gbar|| = lambda sqrt(n) exactly for one worker (every entry of H^T q / sqrt(n) ... has unit mean square)
    assert abs(float(np.linalg.norm(y64)) - lam * rootn) <= 1e-5 * lam * rootn
    e = O.eps_fill(seed, rnd, O.eps_party(0, SERVER), 0, n)
    y64 *= e
    del e
    zs = _rows(O, y64, idx_int) / rootn
    del y64
    us = O.dither_u(seed, rnd, SERVER, 0, idx)
    margin_s = zs + lams * us
    checked = 0
    for i, m in zip(idx_int, margin_s):
        if abs(m) >= TIE * lams:
            assert _bit(h_bits_down, i) == (1 if m >= 0 else 0), ("downlink", i, m)
            checked += 1
    assert checked >= len(idx_int) - 1
    print("server ok", flush=True)

    # ---- decode of the GPU's downlink message, and the update
    qd64 = _signs(h_bits_down, n)
    s_dn = _rows(O, qd64, idx_int)
    del qd64
    es_i = O.eps(seed, rnd, O.eps_party(0, SERVER), idx)
    want_out = lams / rootn * es_i * s_dn
    inside = idx < d                                     # the decoder keeps the first d coordinates
    got_out = out[torch.from_numpy(idx[inside].astype(np.int64)).to(dev)].cpu().numpy().astype(np.float64)
    assert np.max(np.abs(got_out - want_out[inside])) <= 1e-5 * np.max(np.abs(want_out)), (got_out, want_out)
    if d == n:  # ||decode|| = lambda^s sqrt(n) whatever the message (every entry of q is +-1)
        nrm = float(torch.linalg.vector_norm(out.double()))
        assert abs(nrm - lams * rootn) <= 1e-5 * lams * rootn
    print("decode ok", flush=True)

    x = torch.zeros(d, dtype=torch.float32, device=dev)
    plan.fo_step([gd], x, delta, rnd)
    torch.cuda.synchronize()
    assert torch.allclose(x, -delta * out, rtol=1e-6, atol=0.0)
    plan.close()
