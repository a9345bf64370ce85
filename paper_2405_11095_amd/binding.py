"""Thin ctypes binding of the C-ABI codec library (include/fo.h): argument marshalling only.

Every step of the codec runs in the HIP kernels behind `libfo.so`; this module passes device
pointers (from torch tensors, or plain integers) and the current HIP stream across the boundary
and raises on a nonzero return code.  There is no CPU fallback: if the library has not been
built the first call raises.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfo.so")

OK, EINVAL, EALIGN, EHIP, ENOMEM, ESIZE = 0, -1, -2, -3, -4, -5
DITHER_UNIFORM, DITHER_NONE = 0, 1
SCALE_BOUND, SCALE_L2 = 0, 1
EPS_INDEPENDENT, EPS_SHARED_WORKERS, EPS_SHARED_ALL = 0, 1, 2
SERVER_SCALE_THM, SERVER_SCALE_L2, SERVER_SCALE_SUP = 0, 1, 2
PARTY_SERVER = 0xFFFFFFFF
FORCE_SCALE = 1
MAX_WORKERS = 64
NOALLOC_MAX_N = 1 << 22

EXPORTS = ("fo_plan_create", "fo_plan_destroy", "fo_padded_len", "fo_packed_words", "fo_num_scales",
           "fo_block_len", "fo_downlink_planes", "fo_scratch_bytes", "fo_last_hip_error", "fo_encode", "fo_decode",
           "fo_server_aggregate", "fo_step", "fo_encode_noalloc", "fo_step_dev_round", "fo_step_messages", "fo_set_stats", "fo_profile_begin", "fo_profile_begin_kernel", "fo_profile_end")


class FoError(RuntimeError):
    def __init__(self, code, where):
        names = {EINVAL: "FO_EINVAL", EALIGN: "FO_EALIGN", EHIP: "FO_EHIP", ENOMEM: "FO_ENOMEM", ESIZE: "FO_ESIZE"}
        detail = ""
        if code in (EHIP, ESIZE):
            detail = ": " + load_library().fo_last_hip_error().decode()
        super().__init__(f"{where} failed with {names.get(code, code)}{detail}")
        self.code = code


class Params(C.Structure):
    _fields_ = [("d", C.c_uint64), ("M", C.c_uint32), ("block_log2", C.c_uint32), ("K", C.c_uint32),
                ("dither", C.c_uint32), ("scale_rule", C.c_uint32), ("eps_mode", C.c_uint32),
                ("alpha", C.c_float), ("alpha_s", C.c_float), ("B", C.c_float), ("seed", C.c_uint64),
                ("server_scale", C.c_uint32)]


class KernelTime(C.Structure):
    _fields_ = [("name", C.c_char * 48), ("launches", C.c_uint32), ("total_ms", C.c_float)]


_lib = None


def load_library():
    """Load libfo.so (built by __graft_entry__.build()); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build the HIP library first (python -c 'import __graft_entry__ as g; g.build()')")
        lib = C.CDLL(LIB_PATH)
        vp, u64, u32 = C.c_void_p, C.c_uint64, C.c_uint32
        lib.fo_plan_create.argtypes = [C.POINTER(Params), C.POINTER(vp)]
        lib.fo_plan_destroy.argtypes = [vp]
        lib.fo_plan_destroy.restype = None
        for f in ("fo_padded_len", "fo_packed_words", "fo_num_scales", "fo_block_len", "fo_downlink_planes",
                  "fo_scratch_bytes"):
            getattr(lib, f).argtypes = [vp]
            getattr(lib, f).restype = C.c_size_t
        lib.fo_last_hip_error.restype = C.c_char_p
        lib.fo_encode.argtypes = [vp, vp, u64, u32, u32, vp, vp, vp]
        lib.fo_decode.argtypes = [vp, vp, vp, u64, u32, vp, vp]
        lib.fo_encode_noalloc.argtypes = [C.POINTER(Params), vp, u64, u32, u32, vp, vp, vp]
        lib.fo_server_aggregate.argtypes = [vp, vp, vp, u64, vp, vp, vp, vp]
        lib.fo_step.argtypes = [vp, C.POINTER(vp), vp, C.c_float, u64, vp]
        lib.fo_step_dev_round.argtypes = [vp, C.POINTER(vp), vp, C.c_float, vp, vp]
        lib.fo_step_messages.argtypes = [vp, C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), C.POINTER(vp)]
        lib.fo_set_stats.argtypes = [vp, vp]
        lib.fo_profile_begin.argtypes = [vp]
        lib.fo_profile_begin_kernel.argtypes = [vp, C.c_char_p]
        lib.fo_profile_end.argtypes = [vp, C.POINTER(KernelTime), C.c_size_t, C.POINTER(C.c_size_t)]
        _lib = lib
    return _lib


def _ptr(x):
    """Device pointer of a torch tensor (or an int / None passed through)."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _stream(stream):
    if stream is not None:
        return stream
    import torch
    return torch.cuda.current_stream().cuda_stream


def fo_encode_noalloc(params, g, rnd, party, bits, scales, flags=0, stream=None):
    """fo_encode without a plan and without any allocation (static device scratch); params is a Params."""
    rc = load_library().fo_encode_noalloc(C.byref(params), _ptr(g), rnd, party, flags, _ptr(bits), _ptr(scales),
                                          _stream(stream))
    if rc:
        raise FoError(rc, "fo_encode_noalloc")


class Plan:
    """Owner of an fo_plan.  Methods mirror the C entry points one to one."""

    def __init__(self, d, M=1, block_log2=0, K=1, dither=DITHER_UNIFORM, scale_rule=SCALE_L2,
                 eps_mode=EPS_INDEPENDENT, alpha=2.0, alpha_s=2.0, B=1.0, seed=0, server_scale=SERVER_SCALE_THM):
        lib = load_library()
        self.params = Params(int(d), int(M), int(block_log2), int(K), int(dither), int(scale_rule),
                             int(eps_mode), float(alpha), float(alpha_s), float(B), int(seed), int(server_scale))
        h = C.c_void_p()
        rc = lib.fo_plan_create(C.byref(self.params), C.byref(h))
        if rc:
            raise FoError(rc, "fo_plan_create")
        self._h = h
        self.d, self.M = int(d), int(M)
        self.ntot = lib.fo_padded_len(h)
        self.W = lib.fo_packed_words(h)
        self.nblocks = lib.fo_num_scales(h)
        self.b = lib.fo_block_len(h)
        self.planes = lib.fo_downlink_planes(h)
        self.scratch_bytes = lib.fo_scratch_bytes(h)

    def close(self):
        if getattr(self, "_h", None):
            load_library().fo_plan_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def fo_encode(self, g, rnd, party, bits, scales, flags=0, stream=None):
        rc = load_library().fo_encode(self._h, _ptr(g), rnd, party, flags, _ptr(bits), _ptr(scales), _stream(stream))
        if rc:
            raise FoError(rc, "fo_encode")

    def fo_decode(self, bits, scales, rnd, party, out, stream=None):
        rc = load_library().fo_decode(self._h, _ptr(bits), _ptr(scales), rnd, party, _ptr(out), _stream(stream))
        if rc:
            raise FoError(rc, "fo_decode")

    def fo_server_aggregate(self, bits_up, scales_up, rnd, bits_down, scales_down, gbar=None, stream=None):
        rc = load_library().fo_server_aggregate(self._h, _ptr(bits_up), _ptr(scales_up), rnd, _ptr(bits_down),
                                                _ptr(scales_down), _ptr(gbar), _stream(stream))
        if rc:
            raise FoError(rc, "fo_server_aggregate")

    def fo_step(self, g_list, x, delta, rnd, stream=None):
        arr = (C.c_void_p * self.M)(*[_ptr(g) for g in g_list])
        rc = load_library().fo_step(self._h, arr, _ptr(x), delta, rnd, _stream(stream))
        if rc:
            raise FoError(rc, "fo_step")

    def fo_step_dev_round(self, g_list, x, delta, round_dev, stream=None):
        """fo_step with the round read from a device uint64 (a one-element int64 tensor) at kernel run time."""
        arr = (C.c_void_p * self.M)(*[_ptr(g) for g in g_list])
        rc = load_library().fo_step_dev_round(self._h, arr, _ptr(x), delta, _ptr(round_dev), _stream(stream))
        if rc:
            raise FoError(rc, "fo_step_dev_round")

    def fo_step_messages(self):
        """Device addresses (ints) of the last fo_step's messages inside plan scratch."""
        a, b, c, d = C.c_void_p(), C.c_void_p(), C.c_void_p(), C.c_void_p()
        rc = load_library().fo_step_messages(self._h, C.byref(a), C.byref(b), C.byref(c), C.byref(d))
        if rc:
            raise FoError(rc, "fo_step_messages")
        return a.value, b.value, c.value, d.value

    def fo_set_stats(self, stats):
        """Attach (or, with None, detach) a device block of 2 * (MAX_WORKERS + 1) uint64 counters: first the
        `clipped` counts per worker and for the server, then the `near_tie` counts (struct fo_stats)."""
        rc = load_library().fo_set_stats(self._h, _ptr(stats))
        if rc:
            raise FoError(rc, "fo_set_stats")

    def fo_profile_begin(self):
        rc = load_library().fo_profile_begin(self._h)
        if rc:
            raise FoError(rc, "fo_profile_begin")

    def fo_profile_begin_kernel(self, name):
        rc = load_library().fo_profile_begin_kernel(self._h, name.encode())
        if rc:
            raise FoError(rc, "fo_profile_begin_kernel")

    def fo_profile_end(self):
        """{kernel name: (launches, total_ms)} for the kernels that ran since fo_profile_begin."""
        out = (KernelTime * 32)()
        n = C.c_size_t()
        rc = load_library().fo_profile_end(self._h, out, 32, C.byref(n))
        if rc:
            raise FoError(rc, "fo_profile_end")
        return {out[i].name.decode(): (out[i].launches, out[i].total_ms) for i in range(n.value)}
