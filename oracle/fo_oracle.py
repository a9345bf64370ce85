"""ctypes front end of the plain CPU oracle (oracle/fo_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg.  Nothing in the product package may import this module, and this module
imports nothing from the product package.  All values cross as NumPy arrays; the arithmetic is
entirely in the C file, so that it can be read against the paper in one place.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fo_oracle.c")
_LIB = os.path.join(_HERE, "libfo_oracle.so")

PARTY_SERVER = 0xFFFFFFFF
DITHER_UNIFORM, DITHER_NONE = 0, 1
SCALE_BOUND, SCALE_L2 = 0, 1
EPS_INDEPENDENT, EPS_SHARED_WORKERS, EPS_SHARED_ALL = 0, 1, 2
SERVER_SCALE_THM, SERVER_SCALE_L2, SERVER_SCALE_SUP = 0, 1, 2
DOMAIN_EPS, DOMAIN_DITHER = 1, 2


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (plain -O2, no vectorisation flags)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-std=c11", "-O2", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC,
             "-lm", "-lpthread"])
        # the self-test driver (run under sanitizers by the CPU tests) must at least compile with the library
        out_dir = os.path.join(os.path.dirname(_SRC), "_build")
        os.makedirs(out_dir, exist_ok=True)
        subprocess.check_call(
            ["gcc", "-std=c11", "-O2", "-Wall", "-Wextra", "-o", os.path.join(out_dir, "orc_selftest"),
             os.path.join(os.path.dirname(_SRC), "selftest.c"), "-lm", "-lpthread"])
    return _LIB


class Params(C.Structure):
    _fields_ = [("d", C.c_uint64), ("M", C.c_uint32), ("block_log2", C.c_uint32),
                ("K", C.c_uint32), ("dither", C.c_uint32), ("scale_rule", C.c_uint32),
                ("eps_mode", C.c_uint32), ("alpha", C.c_double), ("alpha_s", C.c_double),
                ("B", C.c_double), ("seed", C.c_uint64), ("server_scale", C.c_uint32)]


def params(d, M=1, block_log2=0, K=1, dither=DITHER_UNIFORM, scale_rule=SCALE_L2,
           eps_mode=EPS_INDEPENDENT, alpha=2.0, alpha_s=2.0, B=1.0, seed=0, server_scale=SERVER_SCALE_THM) -> Params:
    return Params(int(d), int(M), int(block_log2), int(K), int(dither), int(scale_rule),
                  int(eps_mode), float(alpha), float(alpha_s), float(B), int(seed), int(server_scale))


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_lambda.restype = C.c_double
        _lib.orc_lambda.argtypes = [C.c_double, C.c_double, C.c_uint64]
        _lib.orc_dither_u.restype = C.c_double
        _lib.orc_dither_u.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint64]
        _lib.orc_eps.restype = C.c_int
        _lib.orc_eps.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint64]
        _lib.orc_eps_party.restype = C.c_uint32
        _lib.orc_eps_party.argtypes = [C.c_uint32, C.c_uint32]
    return _lib


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t)) if a is not None else None


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


# ---------------------------------------------------------------- random numbers
def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    out = np.zeros(4, dtype=np.uint32)
    lib().orc_philox4x32_10(_p(c, C.c_uint32), _p(k, C.c_uint32), _p(out, C.c_uint32))
    return out


def rng(seed, domain, rnd, party, k, counter):
    out = np.zeros(4, dtype=np.uint32)
    lib().orc_rng(C.c_uint64(seed), C.c_uint32(domain), C.c_uint64(rnd), C.c_uint32(party),
                  C.c_uint32(k), C.c_uint32(counter), _p(out, C.c_uint32))
    return out


def eps(seed, rnd, eps_party, idx):
    """eps_i for every i in idx (array of coordinates)."""
    L = lib()
    return np.array([L.orc_eps(seed, rnd, eps_party, int(i)) for i in np.atleast_1d(idx)],
                    dtype=np.float64)


def eps_fill(seed, rnd, eps_party, i0, n):
    """eps_i for i = i0 .. i0 + n - 1 as an fp64 array of +-1."""
    out = np.empty(int(n), dtype=np.float64)
    lib().orc_eps_fill(C.c_uint64(seed), C.c_uint64(rnd), C.c_uint32(eps_party), C.c_uint64(i0), C.c_uint64(n),
                       _p(out, C.c_double))
    return out


def dither_u(seed, rnd, party, k, idx):
    L = lib()
    return np.array([L.orc_dither_u(seed, rnd, party, k, int(i)) for i in np.atleast_1d(idx)],
                    dtype=np.float64)


def eps_party(eps_mode, party):
    return lib().orc_eps_party(eps_mode, party)


# ---------------------------------------------------------------- transform
def sylvester(k):
    n = 1 << k
    H = np.zeros((n, n), dtype=np.float64)
    lib().orc_sylvester(C.c_uint32(k), _p(H, C.c_double))
    return H


def wht_dense(x):
    x = _f64(x)
    y = np.zeros_like(x)
    lib().orc_wht_dense(_p(x, C.c_double), _p(y, C.c_double), C.c_uint64(x.size))
    return y


def wht_rows(x, idx):
    """Entries idx of the unnormalised transform H x, each by the entry formula (O(n) per entry).  x must be
    a contiguous fp64 array (it is not copied: it may be large)."""
    assert x.dtype == np.float64 and x.flags["C_CONTIGUOUS"]
    idx = np.ascontiguousarray(np.atleast_1d(idx), dtype=np.uint64)
    y = np.zeros(idx.size, dtype=np.float64)
    lib().orc_wht_rows(_p(x, C.c_double), C.c_uint64(x.size), _p(idx, C.c_uint64), C.c_uint64(idx.size),
                       _p(y, C.c_double))
    return y


def fwht(x):
    y = _f64(x).copy()
    lib().orc_fwht(_p(y, C.c_double), C.c_uint64(y.size))
    return y


# ---------------------------------------------------------------- geometry
def geometry(p: Params):
    b, nb, nt = C.c_uint64(), C.c_uint64(), C.c_uint64()
    lib().orc_geometry(C.byref(p), C.byref(b), C.byref(nb), C.byref(nt))
    return b.value, nb.value, nt.value


def lam_rule(alpha, B, n):
    return lib().orc_lambda(alpha, B, n)


# ---------------------------------------------------------------- quantizer
def quantize(z, lam, K=1, dither=DITHER_UNIFORM, seed=0, rnd=0, party=0, i0=0, want_margin=False):
    z = _f64(z)
    q = np.zeros(z.size, dtype=np.int32)
    m = np.zeros(z.size, dtype=np.float64) if want_margin else None
    lib().orc_quantize(_p(z, C.c_double), C.c_uint64(z.size), C.c_uint64(i0), C.c_double(lam),
                       C.c_uint32(K), C.c_uint32(dither), C.c_uint64(seed), C.c_uint64(rnd),
                       C.c_uint32(party), _p(q, C.c_int32), _p(m, C.c_double))
    return (q, m) if want_margin else q


def pack(q):
    q = np.ascontiguousarray(q, dtype=np.int32)
    bits = np.zeros(q.size // 64, dtype=np.uint64)
    lib().orc_pack(_p(q, C.c_int32), C.c_uint64(q.size), _p(bits, C.c_uint64))
    return bits


def unpack(bits, n):
    bits = np.ascontiguousarray(bits, dtype=np.uint64)
    q = np.zeros(n, dtype=np.int32)
    lib().orc_unpack(_p(bits, C.c_uint64), C.c_uint64(n), _p(q, C.c_int32))
    return q


# ---------------------------------------------------------------- codec
def encode(p: Params, x, rnd, party, K=1, lam=None, want_margin=False, want_z=False):
    """Returns dict(q, bits (K == 1), lam, margin?, z?).  lam given => forced amplitudes."""
    b, nb, nt = geometry(p)
    x = _f64(x)
    assert x.size == p.d
    force = lam is not None
    lam_a = _f64(lam).copy() if force else np.zeros(nb, dtype=np.float64)
    assert lam_a.size == nb
    q = np.zeros(nt, dtype=np.int32)
    bits = np.zeros(nt // 64, dtype=np.uint64) if K == 1 else None
    margin = np.zeros(nt, dtype=np.float64) if want_margin else None
    z = np.zeros(nt, dtype=np.float64) if want_z else None
    lib().orc_encode(C.byref(p), _p(x, C.c_double), C.c_uint64(rnd), C.c_uint32(party),
                     C.c_uint32(K), C.c_int(1 if force else 0), _p(lam_a, C.c_double),
                     _p(q, C.c_int32), _p(bits, C.c_uint64), _p(margin, C.c_double),
                     _p(z, C.c_double))
    return dict(q=q, bits=bits, lam=lam_a, margin=margin, z=z)


def encode_blocks(p: Params, xs, rnd, party, j0, nj, K=1, lam=None, want_margin=False):
    """Encode blocks j0 .. j0+nj-1 only; xs is the input slice starting at coordinate j0*b."""
    b, nb, nt = geometry(p)
    xs = _f64(xs)
    assert j0 + nj <= nb and xs.size == min(p.d, (j0 + nj) * b) - j0 * b
    force = lam is not None
    lam_a = _f64(lam).copy() if force else np.zeros(nj, dtype=np.float64)
    q = np.zeros(nj * b, dtype=np.int32)
    bits = np.zeros(nj * b // 64, dtype=np.uint64) if K == 1 else None
    margin = np.zeros(nj * b, dtype=np.float64) if want_margin else None
    lib().orc_encode_blocks(C.byref(p), _p(xs, C.c_double), C.c_uint64(rnd), C.c_uint32(party),
                            C.c_uint32(K), C.c_int(1 if force else 0), C.c_uint64(j0), C.c_uint64(nj),
                            _p(lam_a, C.c_double), _p(q, C.c_int32), _p(bits, C.c_uint64),
                            _p(margin, C.c_double), None)
    return dict(q=q, bits=bits, lam=lam_a, margin=margin)


def decode_blocks(p: Params, q, lam, rnd, party, j0, nj, K=1):
    b, nb, nt = geometry(p)
    q = np.ascontiguousarray(q, dtype=np.int32)
    lam = _f64(lam)
    assert q.size == nj * b and lam.size == nj
    out = np.zeros(nj * b, dtype=np.float64)
    lib().orc_decode_blocks(C.byref(p), _p(q, C.c_int32), _p(lam, C.c_double), C.c_uint32(K),
                            C.c_uint64(rnd), C.c_uint32(party), C.c_uint64(j0), C.c_uint64(nj),
                            _p(out, C.c_double))
    return out


def decode(p: Params, q, lam, rnd, party, K=1):
    """Decoded vector of padded length ntot (fp64); callers truncate to d."""
    b, nb, nt = geometry(p)
    q = np.ascontiguousarray(q, dtype=np.int32)
    lam = _f64(lam)
    assert q.size == nt and lam.size == nb
    out = np.zeros(nt, dtype=np.float64)
    lib().orc_decode(C.byref(p), _p(q, C.c_int32), _p(lam, C.c_double), C.c_uint32(K),
                     C.c_uint64(rnd), C.c_uint32(party), _p(out, C.c_double))
    return out


def server_lambda(p: Params, lam_up):
    b, nb, nt = geometry(p)
    lam_up = _f64(lam_up).reshape(p.M, nb)
    out = np.zeros(nb, dtype=np.float64)
    lib().orc_server_lambda(C.byref(p), _p(lam_up, C.c_double), _p(out, C.c_double))
    return out


def server(p: Params, bits_up, lam_up, rnd, lam_s=None, want_margin=False):
    """Returns dict(gbar [ntot], lam_s, q_down, bits_down (K == 1), margin?)."""
    b, nb, nt = geometry(p)
    bits_up = np.ascontiguousarray(bits_up, dtype=np.uint64).reshape(p.M, nt // 64)
    lam_up = _f64(lam_up).reshape(p.M, nb)
    force = lam_s is not None
    lam_s_a = _f64(lam_s).copy() if force else np.zeros(nb, dtype=np.float64)
    gbar = np.zeros(nt, dtype=np.float64)
    qd = np.zeros(nt, dtype=np.int32)
    bd = np.zeros(nt // 64, dtype=np.uint64) if p.K == 1 else None
    margin = np.zeros(nt, dtype=np.float64) if want_margin else None
    lib().orc_server(C.byref(p), _p(bits_up, C.c_uint64), _p(lam_up, C.c_double), C.c_uint64(rnd),
                     _p(gbar, C.c_double), C.c_int(1 if force else 0), _p(lam_s_a, C.c_double),
                     _p(qd, C.c_int32), _p(bd, C.c_uint64), _p(margin, C.c_double))
    return dict(gbar=gbar, lam_s=lam_s_a, q_down=qd, bits_down=bd, margin=margin)


def round_trip(p: Params, g_list, x, delta, rnd, nthreads=1, want=False):
    """One FO-SGD iteration on fp32 gradients g_list (M arrays of length d); x fp64 in place.
    With want=True also returns the intermediate messages."""
    b, nb, nt = geometry(p)
    gs = [np.ascontiguousarray(g, dtype=np.float32) for g in g_list]
    assert len(gs) == p.M and all(g.size == p.d for g in gs)
    ptrs = (C.POINTER(C.c_float) * p.M)(*[_p(g, C.c_float) for g in gs])
    assert x.dtype == np.float64 and x.flags["C_CONTIGUOUS"] and x.size == p.d
    W = nt // 64
    o = {}
    if want:
        o = dict(bits_up=np.zeros((p.M, W), np.uint64), lam_up=np.zeros((p.M, nb), np.float64),
                 gbar=np.zeros(nt, np.float64), bits_down=np.zeros(W, np.uint64),
                 lam_s=np.zeros(nb, np.float64), gd=np.zeros(p.d, np.float64))
    lib().orc_round(C.byref(p), ptrs, _p(x, C.c_double), C.c_double(delta), C.c_uint64(rnd),
                    C.c_int(nthreads), _p(o.get("bits_up"), C.c_uint64),
                    _p(o.get("lam_up"), C.c_double), _p(o.get("gbar"), C.c_double),
                    _p(o.get("bits_down"), C.c_uint64), _p(o.get("lam_s"), C.c_double),
                    _p(o.get("gd"), C.c_double))
    return o
