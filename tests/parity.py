"""Staged parity harness: the HIP codec against the CPU oracle on the same seeded inputs.

Stages are teacher-forced: each stage's oracle is fed the GPU's own upstream output (uplink bits
and fp32 amplitudes), because one legitimately exempt near-tie flip upstream would otherwise move
every downstream value.  Gates (from the paper's arithmetic and the build's target):
  - packed sign bits equal the oracle's except at coordinates whose pre-quantisation value
    |z_i + tau_i| is below 1e-6 * lambda (counted and reported);
  - amplitudes within 1e-6 relative of the oracle's own rule;
  - mean gradient, decoded vector and updated iterate within 1e-5 relative l2.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor

import numpy as np

TIE = 1e-6
SERVER = 0xFFFFFFFF


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / den) if den > 0 else float(np.linalg.norm(a - b))


def bits_to_bool(bits, n):
    return np.unpackbits(np.ascontiguousarray(bits).view(np.uint8), bitorder="little")[:n].astype(bool)


def compare_bits(gpu_bits, margin, lam, b):
    """(mismatches outside the near-tie exemption, exempt coordinates, raw mismatches)."""
    n = margin.size
    want = margin >= 0.0
    got = bits_to_bool(gpu_bits, n)
    lam_c = np.repeat(np.asarray(lam, dtype=np.float64), b)[:n]
    exempt = np.abs(margin) < TIE * lam_c
    diff = want != got
    return int(np.count_nonzero(diff & ~exempt)), int(np.count_nonzero(exempt)), int(np.count_nonzero(diff))


def planes_to_code(planes, n, K):
    """Bit planes [P][W] of the counts c_i -> the code q_i = 2 c_i - K (Def. 3.2 scaled by K / lambda)."""
    planes = np.ascontiguousarray(planes, dtype=np.uint64).reshape(-1, n // 64)
    c = np.zeros(n, dtype=np.int64)
    for p in range(planes.shape[0]):
        c += bits_to_bool(planes[p], n).astype(np.int64) << p
    return (2 * c - K).astype(np.int32)


def compare_codes(q_gpu, q_oracle, margin, lam, b):
    """As compare_bits, for K >= 1: margin is the pre-quantisation value closest to zero over the K dithers."""
    n = margin.size
    lam_c = np.repeat(np.asarray(lam, dtype=np.float64), b)[:n]
    exempt = np.abs(margin) < TIE * lam_c
    diff = np.asarray(q_gpu) != np.asarray(q_oracle)
    return int(np.count_nonzero(diff & ~exempt)), int(np.count_nonzero(exempt)), int(np.count_nonzero(diff))


def check_round_trip(O, B, gs, d, M, block_log2, seed, rnd, delta, device, alpha=2.0, alpha_s=2.0,
                     scale_rule=1, dither=0, Bnorm=1.0, threads=8, check_step=True, eps_mode=0, x0=None, K=1,
                     server_scale=0):
    """Runs encode x M, server, decode and fo_step on the GPU and compares every stage with the
    oracle.  Returns a report dict; asserts nothing (callers apply the gates)."""
    import torch

    plan = B.Plan(d=d, M=M, block_log2=block_log2, K=K, dither=dither, scale_rule=scale_rule, alpha=alpha,
                  alpha_s=alpha_s, B=Bnorm, seed=seed, eps_mode=eps_mode, server_scale=server_scale)
    p = O.params(d=d, M=M, block_log2=block_log2, K=K, dither=dither, scale_rule=scale_rule, alpha=alpha,
                 alpha_s=alpha_s, B=Bnorm, seed=seed, eps_mode=eps_mode, server_scale=server_scale)
    b, nb, nt = O.geometry(p)
    assert (plan.b, plan.nblocks, plan.ntot) == (b, nb, nt)
    W = nt // 64
    PL = plan.planes
    assert PL == max(1, int(K).bit_length())
    gd = [torch.from_numpy(g).to(device) for g in gs]
    bits_up = torch.zeros((M, W), dtype=torch.int64, device=device)
    lam_up = torch.zeros((M, nb), dtype=torch.float32, device=device)
    for m in range(M):
        plan.fo_encode(gd[m], rnd, m, bits_up[m], lam_up[m])
    torch.cuda.synchronize()
    h_lam_free = lam_up.cpu().numpy().copy()         # each worker's own amplitude (the rule's value)
    if eps_mode >= 1:
        # shared worker eps: everybody quantises with the largest amplitude, per block (what fo_step does)
        lam_up[:] = lam_up.max(dim=0, keepdim=True).values.expand(M, nb)
        for m in range(M):
            plan.fo_encode(gd[m], rnd, m, bits_up[m], lam_up[m], flags=B.FORCE_SCALE)
    bits_down = torch.zeros((PL, W), dtype=torch.int64, device=device)
    lam_s = torch.zeros(nb, dtype=torch.float32, device=device)
    gbar = torch.zeros(nt, dtype=torch.float32, device=device)
    plan.fo_server_aggregate(bits_up, lam_up, rnd, bits_down, lam_s, gbar)
    out = torch.zeros(d, dtype=torch.float32, device=device)
    plan.fo_decode(bits_down, lam_s, rnd, SERVER, out)
    torch.cuda.synchronize()
    h_bits_up = bits_up.cpu().numpy().view(np.uint64)
    h_lam_up = lam_up.cpu().numpy()
    h_bits_down = bits_down.cpu().numpy().view(np.uint64)
    h_lam_s = lam_s.cpu().numpy()
    h_gbar = gbar.cpu().numpy()
    h_out = out.cpu().numpy()

    rep = dict(d=d, M=M, b=b, nblocks=nb)

    # ---- stage (i): uplink, oracle forced to the GPU's fp32 amplitudes
    def uplink(m):
        x = gs[m].astype(np.float64)
        free = O.encode(p, x, rnd, m)["lam"]
        r = O.encode(p, x, rnd, m, lam=h_lam_up[m].astype(np.float64), want_margin=True)
        bad, exempt, raw = compare_bits(h_bits_up[m], r["margin"], h_lam_up[m], b)
        den = np.where(free > 0, free, 1.0)
        lam_err = float(np.max(np.abs(h_lam_free[m] - free) / den))
        return bad, exempt, raw, lam_err

    with ThreadPoolExecutor(max_workers=threads) as ex:
        res = list(ex.map(uplink, range(M)))
    rep["uplink_mismatch"] = sum(r[0] for r in res)
    rep["uplink_exempt"] = sum(r[1] for r in res)
    rep["uplink_raw_diff"] = sum(r[2] for r in res)
    rep["lam_rel_err"] = max(r[3] for r in res)

    # ---- stage (ii): server, oracle fed the GPU's uplink messages and the GPU's lambda^s
    if server_scale == 0:
        free_s = O.server_lambda(p, h_lam_up.astype(np.float64))
    else:   # measured-norm rule: the oracle's own amplitude comes with its own mean
        free_s = O.server(p, h_bits_up, h_lam_up.astype(np.float64), rnd)["lam_s"]
    den = np.where(free_s > 0, free_s, 1.0)
    rep["lam_s_rel_err"] = float(np.max(np.abs(h_lam_s - free_s) / den))
    s = O.server(p, h_bits_up, h_lam_up.astype(np.float64), rnd, lam_s=h_lam_s.astype(np.float64), want_margin=True)
    rep["gbar_rel_l2"] = rel_l2(h_gbar, s["gbar"])
    q_gpu = planes_to_code(h_bits_down, nt, K)
    assert q_gpu.min() >= -K and q_gpu.max() <= K
    bad, exempt, raw = compare_codes(q_gpu, s["q_down"], s["margin"], h_lam_s, b)
    rep["downlink_mismatch"], rep["downlink_exempt"], rep["downlink_raw_diff"] = bad, exempt, raw

    # ---- stage (iii): worker decode of the GPU's downlink message
    dec = O.decode(p, q_gpu, h_lam_s.astype(np.float64), rnd, SERVER, K=K)[:d]
    rep["decode_rel_l2"] = rel_l2(h_out, dec)

    # ---- fo_step: same messages as the calls made by hand, and the SGD update
    if check_step:
        if x0 is None:
            x0 = np.random.default_rng(12345).standard_normal(d).astype(np.float32)
        x = torch.from_numpy(x0.copy()).to(device)
        plan.fo_step(gd, x, delta, rnd)
        torch.cuda.synchronize()
        pb_up, ps_up, pb_dn, ps_dn = plan.fo_step_messages()
        step_bits_up = _peek(torch, pb_up, M * W, torch.int64, device).view(np.uint64).reshape(M, W)
        step_lam_up = _peek(torch, ps_up, M * nb, torch.float32, device).reshape(M, nb)
        step_bits_dn = _peek(torch, pb_dn, PL * W, torch.int64, device).view(np.uint64).reshape(PL, W)
        step_lam_s = _peek(torch, ps_dn, nb, torch.float32, device)
        rep["step_messages_equal"] = bool(
            np.array_equal(step_bits_up, h_bits_up) and np.array_equal(step_lam_up, h_lam_up)
            and np.array_equal(step_bits_dn, h_bits_down) and np.array_equal(step_lam_s, h_lam_s))
        want_x = x0.astype(np.float64) - delta * dec
        # x is stored in fp32: besides the 1e-5 budget on the update itself, allow half an ulp of x
        # (2^-24 ~ 6e-8 relative, written 1.2e-7 for the two roundings of a read-modify-write)
        err = np.linalg.norm(x.cpu().numpy().astype(np.float64) - want_x)
        rep["x_rel_l2"] = float(err / (np.linalg.norm(delta * dec) + 0.012 * np.linalg.norm(x0)))
    plan.close()
    return rep


def _peek(torch, addr, count, dtype, device):
    """Copy `count` elements at device address `addr` (plan scratch) to a NumPy array."""
    import ctypes as C
    itemsize = torch.empty(0, dtype=dtype).element_size()
    dst = torch.empty(count, dtype=dtype, device=device)
    hip = C.CDLL("libamdhip64.so")
    hip.hipMemcpy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int]
    rc = hip.hipMemcpy(dst.data_ptr(), addr, count * itemsize, 3)  # device to device
    assert rc == 0
    return dst.cpu().numpy()


def gates(rep, tol=1e-5):
    assert rep["uplink_mismatch"] == 0, rep
    assert rep["downlink_mismatch"] == 0, rep
    assert rep["lam_rel_err"] <= 1e-6 and rep["lam_s_rel_err"] <= 1e-6, rep
    assert rep["gbar_rel_l2"] <= tol and rep["decode_rel_l2"] <= tol, rep
    if "x_rel_l2" in rep:
        assert rep["step_messages_equal"], rep
        assert rep["x_rel_l2"] <= tol, rep


def check_sampled_blocks(O, B, gs, d, M, block_log2, seed, rnd, device, block_ranges, threads=8):
    """Full-size blocked workloads: the GPU runs the whole round through fo_step; the oracle checks
    the stages on sampled ranges of blocks only (blocks are independent transforms), teacher-forced
    as in check_round_trip.  block_ranges: list of (j0, nj)."""
    import torch

    plan = B.Plan(d=d, M=M, block_log2=block_log2, seed=seed)
    p = O.params(d=d, M=M, block_log2=block_log2, seed=seed)
    b, nb, nt = O.geometry(p)
    W = nt // 64
    gd = [torch.from_numpy(g).to(device) for g in gs]
    x0 = np.zeros(d, dtype=np.float32)
    x = torch.from_numpy(x0.copy()).to(device)
    delta = 1.0                                  # x becomes minus the decoded downlink vector
    plan.fo_step(gd, x, delta, rnd)
    torch.cuda.synchronize()
    pb_up, ps_up, pb_dn, ps_dn = plan.fo_step_messages()
    bits_up = _peek(torch, pb_up, M * W, torch.int64, device).view(np.uint64).reshape(M, W)
    lam_up = _peek(torch, ps_up, M * nb, torch.float32, device).reshape(M, nb)
    bits_dn = _peek(torch, pb_dn, W, torch.int64, device).view(np.uint64)
    lam_s = _peek(torch, ps_dn, nb, torch.float32, device)
    hx = x.cpu().numpy()
    del gd, x
    rep = dict(d=d, M=M, b=b, nblocks=nb, blocks_checked=0, uplink_mismatch=0, uplink_exempt=0, lam_rel_err=0.0,
               lam_s_rel_err=0.0, downlink_mismatch=0, downlink_exempt=0, decode_rel_l2=0.0)
    ps = O.params(d=nt, M=M, block_log2=block_log2, seed=seed)   # the server encodes a vector of length ntot
    for (j0, nj) in block_ranges:
        lo, hi = j0 * b, min(d, (j0 + nj) * b)
        wlo, whi = j0 * b // 64, (j0 + nj) * b // 64

        def uplink(m):
            xs = gs[m][lo:hi].astype(np.float64)
            free = O.encode_blocks(p, xs, rnd, m, j0, nj)["lam"]
            r = O.encode_blocks(p, xs, rnd, m, j0, nj, lam=lam_up[m, j0:j0 + nj].astype(np.float64), want_margin=True)
            bad, exempt, _ = compare_bits(bits_up[m, wlo:whi], r["margin"], lam_up[m, j0:j0 + nj], b)
            den = np.where(free > 0, free, 1.0)
            return bad, exempt, float(np.max(np.abs(lam_up[m, j0:j0 + nj] - free) / den))

        with ThreadPoolExecutor(max_workers=threads) as ex:
            res = list(ex.map(uplink, range(M)))
        rep["uplink_mismatch"] += sum(r[0] for r in res)
        rep["uplink_exempt"] += sum(r[1] for r in res)
        rep["lam_rel_err"] = max(rep["lam_rel_err"], max(r[2] for r in res))
        # server on the sampled blocks: decode every worker's GPU bits, average, re-encode
        gbar = np.zeros(nj * b)
        for m in range(M):
            q = O.unpack(bits_up[m, wlo:whi], nj * b)
            gbar += O.decode_blocks(p, q, lam_up[m, j0:j0 + nj].astype(np.float64), rnd, m, j0, nj)
        gbar /= M
        free_s = 2.0 * lam_up[:, j0:j0 + nj].astype(np.float64).max(axis=0) * np.sqrt(np.log(b))
        den = np.where(free_s > 0, free_s, 1.0)
        rep["lam_s_rel_err"] = max(rep["lam_s_rel_err"], float(np.max(np.abs(lam_s[j0:j0 + nj] - free_s) / den)))
        r = O.encode_blocks(ps, gbar, rnd, SERVER, j0, nj, lam=lam_s[j0:j0 + nj].astype(np.float64), want_margin=True)
        bad, exempt, _ = compare_bits(bits_dn[wlo:whi], r["margin"], lam_s[j0:j0 + nj], b)
        rep["downlink_mismatch"] += bad
        rep["downlink_exempt"] += exempt
        dec = O.decode_blocks(p, O.unpack(bits_dn[wlo:whi], nj * b), lam_s[j0:j0 + nj].astype(np.float64), rnd, SERVER, j0, nj)
        rep["decode_rel_l2"] = max(rep["decode_rel_l2"], rel_l2(-hx[lo:hi].astype(np.float64), dec[:hi - lo]))
        rep["blocks_checked"] += nj
    plan.close()
    return rep
