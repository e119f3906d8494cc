"""ctypes front end of the CPU oracle (``regtopk_oracle.cpp``).

TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the ``cpu_baseline``
leg of the benchmark may import this module; the product path never does.  It
holds no arithmetic of the method: it compiles the C++ file with g++, loads it
and moves numpy arrays across.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "regtopk_oracle.cpp")
_LIB = os.path.join(_HERE, "libregtopk_oracle.so")
# tests/test_oracle_mutations.py points this at a deliberately broken build to show that the pins notice
_LIB_OVERRIDE = os.environ.get("REGTOPK_ORACLE_LIB")
_lib = None

# No FMA contraction, no fast-math: every operation is a single IEEE rounding.
CXXFLAGS = ["-O2", "-std=c++17", "-ffp-contract=off", "-fno-fast-math",
            "-shared", "-fPIC"]


def build(force: bool = False) -> str:
    """Compile the oracle into ``oracle/libregtopk_oracle.so``."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    tmp = _LIB + ".tmp.%d" % os.getpid()
    subprocess.check_call(["g++", *CXXFLAGS, _SRC, "-o", tmp])
    os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    lib = ctypes.CDLL(_LIB_OVERRIDE or build())
    c = ctypes
    lib.rtk_oracle_create.restype = c.c_void_p
    lib.rtk_oracle_create.argtypes = [c.c_int32, c.c_int64, c.c_int64, c.c_float]
    lib.rtk_oracle_destroy.argtypes = [c.c_void_p]
    lib.rtk_oracle_step.argtypes = [c.c_void_p] + [c.c_void_p] * 5
    lib.rtk_oracle_step_global.argtypes = [c.c_void_p] + [c.c_void_p] * 4
    for name in ("e", "a", "score", "mask"):
        f = getattr(lib, "rtk_oracle_" + name)
        f.restype = c.c_void_p
        f.argtypes = [c.c_void_p]
    lib.rtk_oracle_round.restype = c.c_int64
    lib.rtk_oracle_round.argtypes = [c.c_void_p]
    lib.rtk_oracle_set_weights.argtypes = [c.c_void_p, c.c_void_p]
    lib.rtk_oracle_mask_overlap.argtypes = [c.c_void_p, c.c_void_p]
    lib.rtk_oracle_sgd_update.argtypes = [c.c_void_p, c.c_void_p, c.c_float, c.c_int64]
    lib.rtk_oracle_set_worker_k.restype = c.c_int
    lib.rtk_oracle_set_worker_k.argtypes = [c.c_void_p, c.c_void_p]
    lib.rtk_oracle_set_score_variant.restype = c.c_int
    lib.rtk_oracle_set_score_variant.argtypes = [c.c_void_p, c.c_int, c.c_int]
    lib.rtk_oracle_likelihood_sent_kind.restype = c.c_float
    lib.rtk_oracle_likelihood_sent_kind.argtypes = [c.c_float] * 5 + [c.c_int]
    lib.rtk_oracle_set_prior_exponent.restype = c.c_int
    lib.rtk_oracle_set_prior_exponent.argtypes = [c.c_void_p, c.c_float]
    lib.rtk_oracle_prior_pow.restype = c.c_float
    lib.rtk_oracle_prior_pow.argtypes = [c.c_float, c.c_float]
    lib.rtk_oracle_prior_pow_array.argtypes = [c.c_void_p, c.c_float, c.c_void_p, c.c_int64]
    lib.rtk_oracle_prior.restype = c.c_float
    lib.rtk_oracle_prior.argtypes = [c.c_float, c.c_int]
    lib.rtk_oracle_tanh32.restype = c.c_float
    lib.rtk_oracle_tanh32.argtypes = [c.c_float]
    lib.rtk_oracle_likelihood_sent.restype = c.c_float
    lib.rtk_oracle_likelihood_sent.argtypes = [c.c_float] * 5
    lib.rtk_oracle_topk_mask.argtypes = [c.c_void_p, c.c_int64, c.c_int64, c.c_void_p]
    lib.rtk_oracle_tanh32_array.argtypes = [c.c_void_p, c.c_void_p, c.c_int64]
    lib.rtk_oracle_erf32.restype = c.c_float
    lib.rtk_oracle_erf32.argtypes = [c.c_float]
    lib.rtk_oracle_erf32_array.argtypes = [c.c_void_p, c.c_void_p, c.c_int64]
    _lib = lib
    return lib


def _f32(x) -> np.ndarray:
    return np.ascontiguousarray(x, dtype=np.float32)


class Oracle:
    """N workers, model size d, k kept entries, temperature mu (0 = plain Top-k)."""

    def __init__(self, N: int, d: int, k: int, mu: float):
        self._lib = _load()
        self.N, self.d, self.k, self.mu = int(N), int(d), int(k), float(mu)
        self._h = self._lib.rtk_oracle_create(self.N, self.d, self.k, self.mu)
        if not self._h:
            raise ValueError("invalid oracle arguments N=%r d=%r k=%r mu=%r" % (N, d, k, mu))

    def close(self):
        if self._h:
            self._lib.rtk_oracle_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def step(self, grads, gprev=None):
        """One round. Returns (idx [N,k] int32, val [N,k] f32, agg [d] f32)."""
        g = _f32(grads)
        if g.shape != (self.N, self.d):
            raise ValueError("grads must be [N,d]")
        if gprev is None:
            if self.round != 0 and self.mu != 0.0:
                raise ValueError("gprev is required after round 0")
            gp = np.zeros(self.d, dtype=np.float32)
        else:
            gp = _f32(gprev)
            if gp.shape != (self.d,):
                raise ValueError("gprev must be [d]")
        idx = np.empty((self.N, self.k), dtype=np.int32)
        val = np.empty((self.N, self.k), dtype=np.float32)
        agg = np.empty(self.d, dtype=np.float32)
        self._lib.rtk_oracle_step(self._h, g.ctypes.data, gp.ctypes.data,
                                  idx.ctypes.data, val.ctypes.data, agg.ctypes.data)
        return idx, val, agg

    def step_global(self, grads):
        """One round of the genie-aided global Top-k (all workers share the mask
        of the k largest entries of the unsparsified aggregate).  Returns like step."""
        g = _f32(grads)
        if g.shape != (self.N, self.d):
            raise ValueError("grads must be [N,d]")
        idx = np.empty((self.N, self.k), dtype=np.int32)
        val = np.empty((self.N, self.k), dtype=np.float32)
        agg = np.empty(self.d, dtype=np.float32)
        self._lib.rtk_oracle_step_global(self._h, g.ctypes.data, idx.ctypes.data, val.ctypes.data,
                                         agg.ctypes.data)
        return idx, val, agg

    def set_weights(self, w):
        """Aggregation weights omega_n, one per worker (default 1/N each)."""
        ws = _f32(w)
        if ws.shape != (self.N,):
            raise ValueError("weights must be [N]")
        self._lib.rtk_oracle_set_weights(self._h, ws.ctypes.data)

    def set_worker_k(self, kn):
        """Entries kept by each worker, k_n in [1, k]; the rest of a worker's output row is (-1, 0)."""
        ks = np.ascontiguousarray(kn, dtype=np.int64)
        if ks.shape != (self.N,):
            raise ValueError("need N values")
        if self._lib.rtk_oracle_set_worker_k(self._h, ks.ctypes.data) != 0:
            raise ValueError("every k_n must be in [1, k]")

    def set_score_variant(self, sqrt_steps: int = 0, likelihood: int = 0):
        """Prior |a|^(2^-sqrt_steps) and likelihood kind (0 tanh, 1 clipped linear, 2 erf)."""
        if self._lib.rtk_oracle_set_score_variant(self._h, int(sqrt_steps), int(likelihood)) != 0:
            raise ValueError("sqrt_steps must be 0..3 and likelihood 0, 1 or 2")

    def set_prior_exponent(self, y: float):
        """Prior |a|^y with a general exponent 0 < y <= 1 (replaces the square-root variant)."""
        if self._lib.rtk_oracle_set_prior_exponent(self._h, float(np.float32(y))) != 0:
            raise ValueError("the exponent must be in (0, 1]")

    def mask_overlap(self) -> np.ndarray:
        """counts[c] = number of entries selected by exactly c workers in the last round."""
        counts = np.zeros(self.N + 1, dtype=np.int64)
        self._lib.rtk_oracle_mask_overlap(self._h, counts.ctypes.data)
        return counts

    def _view(self, name, dtype):
        p = getattr(self._lib, "rtk_oracle_" + name)(self._h)
        n = self.N * self.d
        buf = (ctypes.c_char * (n * np.dtype(dtype).itemsize)).from_address(p)
        return np.frombuffer(buf, dtype=dtype).reshape(self.N, self.d).copy()

    @property
    def round(self) -> int:
        return int(self._lib.rtk_oracle_round(self._h))

    @property
    def e(self):
        return self._view("e", np.float32)

    @property
    def a(self):
        return self._view("a", np.float32)

    @property
    def score(self):
        return self._view("score", np.float32)

    @property
    def mask(self):
        return self._view("mask", np.uint8)


def tanh32(x: float) -> float:
    return float(_load().rtk_oracle_tanh32(float(np.float32(x))))


def tanh32_array(x) -> np.ndarray:
    xs = _f32(x).ravel()
    out = np.empty_like(xs)
    _load().rtk_oracle_tanh32_array(xs.ctypes.data, out.ctypes.data, xs.size)
    return out


def erf32(x: float) -> float:
    return float(_load().rtk_oracle_erf32(float(np.float32(x))))


def erf32_array(x) -> np.ndarray:
    xs = _f32(x).ravel()
    out = np.empty_like(xs)
    _load().rtk_oracle_erf32_array(xs.ctypes.data, out.ctypes.data, xs.size)
    return out


def likelihood_sent(a_now, a_before, g_before, w, mu) -> float:
    f = np.float32
    return float(_load().rtk_oracle_likelihood_sent(
        float(f(a_now)), float(f(a_before)), float(f(g_before)), float(f(w)), float(f(mu))))


def likelihood_sent_kind(a_now, a_before, g_before, w, mu, kind: int) -> float:
    f = np.float32
    return float(_load().rtk_oracle_likelihood_sent_kind(
        float(f(a_now)), float(f(a_before)), float(f(g_before)), float(f(w)), float(f(mu)), int(kind)))


def prior(a, sqrt_steps: int) -> float:
    return float(_load().rtk_oracle_prior(float(np.float32(a)), int(sqrt_steps)))


def prior_pow(a, y: float) -> float:
    return float(_load().rtk_oracle_prior_pow(float(np.float32(a)), float(np.float32(y))))


def prior_pow_array(x, y: float) -> np.ndarray:
    xs = _f32(x).ravel()
    out = np.empty_like(xs)
    _load().rtk_oracle_prior_pow_array(xs.ctypes.data, float(np.float32(y)), out.ctypes.data, xs.size)
    return out


def topk_mask(score, k: int) -> np.ndarray:
    s = _f32(score).ravel()
    mask = np.empty(s.size, dtype=np.uint8)
    _load().rtk_oracle_topk_mask(s.ctypes.data, s.size, int(k), mask.ctypes.data)
    return mask


def sgd_update(theta, g, eta: float) -> np.ndarray:
    """theta - eta * g in binary32 (returns a new array)."""
    th = _f32(theta).copy()
    gg = _f32(g)
    if th.shape != gg.shape or th.ndim != 1:
        raise ValueError("theta and g must be vectors of one length")
    _load().rtk_oracle_sgd_update(th.ctypes.data, gg.ctypes.data, float(np.float32(eta)), th.size)
    return th
