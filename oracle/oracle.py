"""ctypes loader for the CPU oracle (comp_ams_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the
benchmark's CPU-baseline leg.  The HIP package never imports this module, and
this module never imports the HIP package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "comp_ams_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

TOPK = 0
BLOCKSIGN = 1
RANDK = 2   # Appendix A, "Rand-k"
EF = 0      # error feedback (Section 4)
CD = 1      # CD-Adam, Algorithm 1
NAIVE = 2   # naive compression (Section 4), no memory
NONE = 3    # no compression: vanilla distributed AMSGrad (Section 3)


_SWEEP_SRC = os.path.join(_HERE, "sanitize_sweep.c")
_SWEEP = os.path.join(_HERE, "sanitize_sweep.bin")


def build(force: bool = True) -> str:
    """Compile the oracle with gcc: -O2, no FMA contraction, no fast-math.  A forced build also compiles the
    sweep driver (oracle/sanitize_sweep.c) with the same flags, as a check that it builds; the sanitizer run
    itself is tests/test_sanitizers.py's, with its own instrumented binary."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        flags = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-Wall", "-Wextra"]
        subprocess.run(flags + ["-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"], check=True)
        if force:
            subprocess.run(flags + ["-o", _SWEEP, _SWEEP_SRC, _SRC, "-lm"], check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build(force=False)
        L = C.CDLL(_LIB)
        fp = C.POINTER(C.c_float)
        u32p = C.POINTER(C.c_uint32)
        i64p = C.POINTER(C.c_int64)
        L.oracle_create.restype = C.c_void_p
        L.oracle_create.argtypes = [C.c_int64, C.c_int32, C.c_int32, C.c_int64, C.c_float, C.c_float,
                                    C.c_float, C.c_float]
        L.oracle_set_blocks.argtypes = [C.c_void_p, i64p, C.c_int32]
        L.oracle_set_theta.argtypes = [C.c_void_p, fp]
        L.oracle_set_lr.argtypes = [C.c_void_p, C.c_float]
        L.oracle_set_eps_mode.argtypes = [C.c_void_p, C.c_int32]
        L.oracle_set_method.argtypes = [C.c_void_p, C.c_int32]
        L.oracle_set_rand.argtypes = [C.c_void_p, C.c_uint64, C.c_uint32]
        L.oracle_mix32.restype = C.c_uint32
        L.oracle_mix32.argtypes = [C.c_uint32]
        L.oracle_randk_score.restype = C.c_uint32
        L.oracle_randk_score.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32]
        L.oracle_randk.argtypes = [fp, C.c_int64, C.c_int64, C.c_uint64, C.c_uint32, C.c_uint32, fp, u32p]
        L.oracle_step.argtypes = [C.c_void_p, fp]
        for name in ("theta", "m", "v", "vhat", "gbar", "error", "compressed", "scales", "ghat_workers",
                     "ghat_server", "gtilde", "server_compressed", "server_scales"):
            f = getattr(L, "oracle_" + name)
            f.restype = fp
            f.argtypes = [C.c_void_p]
        L.oracle_selected.restype = u32p
        L.oracle_selected.argtypes = [C.c_void_p]
        L.oracle_server_selected.restype = u32p
        L.oracle_server_selected.argtypes = [C.c_void_p]
        L.oracle_n_blocks.restype = C.c_int32
        L.oracle_n_blocks.argtypes = [C.c_void_p]
        L.oracle_destroy.argtypes = [C.c_void_p]
        L.oracle_topk.argtypes = [fp, C.c_int64, C.c_int64, fp, u32p]
        L.oracle_blocksign.argtypes = [fp, i64p, C.c_int32, fp, fp]
        L.oracle_amsgrad.argtypes = [fp, fp, fp, fp, fp, C.c_int64, C.c_float, C.c_float, C.c_float,
                                     C.c_float, C.c_int32]
        _lib = L
    return _lib


def _fp(a):
    return a.ctypes.data_as(C.POINTER(C.c_float))


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def topk(x, k):
    """C_top(x): returns (c, selected indices ascending)."""
    x = _f32(x)
    c = np.empty_like(x)
    sel = np.empty(k, dtype=np.uint32)
    lib().oracle_topk(_fp(x), x.size, k, _fp(c), sel.ctypes.data_as(C.POINTER(C.c_uint32)))
    return c, sel


def randk(x, k, seed, draw, who):
    """C_rand(x) for the draw (seed, draw, who): returns (c, selected indices ascending)."""
    x = _f32(x)
    c = np.empty_like(x)
    sel = np.empty(k, dtype=np.uint32)
    lib().oracle_randk(_fp(x), x.size, k, seed, draw, who, _fp(c), sel.ctypes.data_as(C.POINTER(C.c_uint32)))
    return c, sel


def randk_score(seed, draw, who, j):
    return lib().oracle_randk_score(seed, draw, who, j)


def mix32(h):
    return lib().oracle_mix32(h)


def blocksign(x, offsets):
    """Scaled sign per block: returns (c, scales)."""
    x = _f32(x)
    off = np.ascontiguousarray(offsets, dtype=np.int64)
    c = np.empty_like(x)
    s = np.empty(off.size - 1, dtype=np.float32)
    lib().oracle_blocksign(_fp(x), off.ctypes.data_as(C.POINTER(C.c_int64)), off.size - 1, _fp(c), _fp(s))
    return c, s


def amsgrad(theta, m, v, vhat, gbar, beta1, beta2, eps, lr, eps_mode=0):
    """One AMSGrad update; returns new (theta, m, v, vhat) without touching the inputs."""
    th, m, v, vh = (_f32(a).copy() for a in (theta, m, v, vhat))
    g = _f32(gbar)
    lib().oracle_amsgrad(_fp(th), _fp(m), _fp(v), _fp(vh), _fp(g), g.size, beta1, beta2, eps, lr, eps_mode)
    return th, m, v, vh


class Oracle:
    """Stateful compressed AMSGrad on n simulated workers (CPU, fp32): error feedback (default)
    or, with method=CD, CD-Adam (Algorithm 1)."""

    def __init__(self, d, n, compressor, k_or_block, beta1, beta2, eps, lr, method=EF):
        self.d, self.n, self.compressor = int(d), int(n), int(compressor)
        self.k = int(k_or_block) if compressor != BLOCKSIGN else 0
        self.method = int(method)
        self._h = lib().oracle_create(d, n, compressor, k_or_block, beta1, beta2, eps, lr)
        if self.method != EF:
            lib().oracle_set_method(self._h, self.method)

    def close(self):
        if self._h:
            lib().oracle_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:      # interpreter shutdown: the library may already be gone
            pass

    def set_blocks(self, offsets):
        off = np.ascontiguousarray(offsets, dtype=np.int64)
        lib().oracle_set_blocks(self._h, off.ctypes.data_as(C.POINTER(C.c_int64)), off.size - 1)

    def set_theta(self, theta):
        t = _f32(theta)
        assert t.size == self.d
        lib().oracle_set_theta(self._h, _fp(t))

    def set_lr(self, lr):
        lib().oracle_set_lr(self._h, lr)

    def set_eps_mode(self, mode):
        lib().oracle_set_eps_mode(self._h, mode)

    def set_rand(self, seed, draw=0):
        """Rand-k: the generator's seed and the number of the next draw (= steps taken so far)."""
        lib().oracle_set_rand(self._h, seed, draw)

    def step(self, grads):
        g = _f32(grads)
        assert g.shape == (self.n, self.d)
        lib().oracle_step(self._h, _fp(g))

    def _view(self, name, shape):
        p = getattr(lib(), "oracle_" + name)(self._h)
        return np.ctypeslib.as_array(p, shape=shape)

    @property
    def n_blocks(self):
        return lib().oracle_n_blocks(self._h)

    # views into the oracle's own memory (copy if you need them past the next step)
    theta = property(lambda s: s._view("theta", (s.d,)))
    m = property(lambda s: s._view("m", (s.d,)))
    v = property(lambda s: s._view("v", (s.d,)))
    vhat = property(lambda s: s._view("vhat", (s.d,)))
    gbar = property(lambda s: s._view("gbar", (s.d,)))
    error = property(lambda s: s._view("error", (s.n, s.d)))
    compressed = property(lambda s: s._view("compressed", (s.n, s.d)))
    selected = property(lambda s: s._view("selected", (s.n, s.k)))
    scales = property(lambda s: s._view("scales", (s.n, s.n_blocks)))
    # CD-Adam state
    ghat_workers = property(lambda s: s._view("ghat_workers", (s.n, s.d)))
    ghat_server = property(lambda s: s._view("ghat_server", (s.d,)))
    gtilde = property(lambda s: s._view("gtilde", (s.d,)))
    server_compressed = property(lambda s: s._view("server_compressed", (s.d,)))
    server_selected = property(lambda s: s._view("server_selected", (s.k,)))
    server_scales = property(lambda s: s._view("server_scales", (s.n_blocks,)))
