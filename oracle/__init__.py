"""ctypes loader for the DES-LOC CPU oracle.  TEST INFRASTRUCTURE, NOT PRODUCT CODE.

Only tests, the smoke check and the benchmark's cpu_baseline leg import this
package.  It never imports the HIP package and shares nothing with it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
SOURCE = os.path.join(_HERE, "desloc_oracle.cpp")
LIBRARY = os.path.join(_HERE, "libdesloc_oracle.so")

# Strict IEEE: no fast-math, no contraction, no x87 excess precision (SSE2 on x86-64).
CXXFLAGS = ["-std=c++17", "-O2", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
            "-Wall", "-Wextra", "-Werror"]

ADAM, ADOPT, SGDM = 0, 1, 2


def build(source: str = SOURCE, library: str = LIBRARY, extra_flags=()) -> str:
    """Compile the oracle with g++ (always recompiles)."""
    cmd = ["g++", *CXXFLAGS, *extra_flags, source, "-o", library]
    subprocess.run(cmd, check=True)
    return library


class _Cfg(ctypes.Structure):
    _fields_ = [
        ("variant", ctypes.c_int32),
        ("M", ctypes.c_int32),
        ("Kx", ctypes.c_uint64),
        ("Ku", ctypes.c_uint64),
        ("Kv", ctypes.c_uint64),
        ("lr", ctypes.c_double),
        ("beta1", ctypes.c_double),
        ("beta2", ctypes.c_double),
        ("eps", ctypes.c_double),
        ("rho", ctypes.c_double),
        ("adam_literal", ctypes.c_int32),
        ("adopt_avg_normaliser", ctypes.c_int32),
        ("adopt_init_g0sq", ctypes.c_int32),
        ("norm_clip", ctypes.c_int32),
        ("post_average", ctypes.c_int32),
        ("amsgrad", ctypes.c_int32),
    ]


@dataclass
class Config:
    variant: int = ADAM
    M: int = 1
    Kx: int = 1
    Ku: int = 1
    Kv: int = 1
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    rho: float = float("inf")
    adam_literal: bool = False
    adopt_avg_normaliser: bool = False
    adopt_init_g0sq: bool = False
    norm_clip: bool = False
    post_average: bool = False
    amsgrad: bool = False

    def as_f32_hypers(self) -> "Config":
        """The same config with every real hyper-parameter rounded to fp32, i.e. the
        values an fp32 caller actually holds."""
        f = lambda v: float(np.float32(v))
        return Config(self.variant, self.M, self.Kx, self.Ku, self.Kv, f(self.lr), f(self.beta1),
                      f(self.beta2), f(self.eps), f(self.rho), self.adam_literal,
                      self.adopt_avg_normaliser, self.adopt_init_g0sq, self.norm_clip,
                      self.post_average, self.amsgrad)

    def _c(self) -> _Cfg:
        return _Cfg(self.variant, self.M, self.Kx, self.Ku, self.Kv, self.lr, self.beta1,
                    self.beta2, self.eps, self.rho, int(self.adam_literal),
                    int(self.adopt_avg_normaliser), int(self.adopt_init_g0sq), int(self.norm_clip),
                    int(self.post_average), int(self.amsgrad))


class Oracle:
    """Thin handle on a built oracle library."""

    def __init__(self, library: str = LIBRARY):
        if not os.path.exists(library):
            build(library=library)
        self.lib = ctypes.CDLL(library)
        L = self.lib
        p = ctypes.c_void_p
        L.oracle_sync_mask.restype = ctypes.c_uint32
        L.oracle_sync_mask.argtypes = [ctypes.POINTER(_Cfg), ctypes.c_uint64]
        L.oracle_sync_count.restype = ctypes.c_uint64
        L.oracle_sync_count.argtypes = [ctypes.c_uint64, ctypes.c_uint64]
        L.oracle_widen_bf16.restype = ctypes.c_float
        L.oracle_widen_bf16.argtypes = [ctypes.c_uint16]
        for name in ("oracle_step_f32", "oracle_step_f64"):
            fn = getattr(L, name)
            fn.restype = None
            fn.argtypes = [ctypes.POINTER(_Cfg), ctypes.c_uint64, ctypes.c_uint64, p, p, p, p]
        for name in ("oracle_step_norm_f32", "oracle_step_norm_f64"):
            fn = getattr(L, name)
            fn.restype = None
            fn.argtypes = [ctypes.POINTER(_Cfg), ctypes.c_uint64, ctypes.c_uint64, p, p, p, p, p, p]
        for name in ("oracle_step_post_f32", "oracle_step_post_f64"):
            fn = getattr(L, name)
            fn.restype = None
            fn.argtypes = [ctypes.POINTER(_Cfg), ctypes.c_uint64, ctypes.c_uint64, p, p, p, p, p, p, p]
        L.oracle_state_change_f32.restype = None
        L.oracle_state_change_f32.argtypes = [ctypes.c_int32, ctypes.c_uint64, p, p, p, p]
        L.oracle_state_change_tensors_f32.restype = None
        L.oracle_state_change_tensors_f32.argtypes = [ctypes.c_int32, ctypes.c_uint64, p, ctypes.c_uint64,
                                                      p, p, p, p]
        for name in ("oracle_worker_mean_f32", "oracle_worker_mean_f64"):
            fn = getattr(L, name)
            fn.restype = None
            fn.argtypes = [ctypes.c_int32, ctypes.c_uint64, p, p]

    # -- schedule ---------------------------------------------------------
    def sync_mask(self, cfg: Config, t: int) -> int:
        c = cfg._c()
        return int(self.lib.oracle_sync_mask(ctypes.byref(c), t))

    def sync_count(self, T: int, K: int) -> int:
        return int(self.lib.oracle_sync_count(T, K))

    def widen_bf16(self, bits: np.ndarray) -> np.ndarray:
        bits = np.asarray(bits, dtype=np.uint16)
        out = np.empty(bits.shape, dtype=np.float32)
        flat_in, flat_out = bits.ravel(), out.ravel()
        for i in range(flat_in.size):
            flat_out[i] = self.lib.oracle_widen_bf16(int(flat_in[i]))
        return out

    # -- update -----------------------------------------------------------
    @staticmethod
    def _check(a, dtype, M, n, name):
        if a is None:
            return None
        if a.dtype != dtype or not a.flags["C_CONTIGUOUS"] or a.shape != (M, n):
            raise ValueError(f"{name}: need C-contiguous {dtype} array of shape ({M}, {n}), "
                             f"got {a.dtype} {a.shape}")
        return a.ctypes.data_as(ctypes.c_void_p)

    def step(self, cfg: Config, t: int, x, u, v, g, sumsq_rest=None, vmax=None):
        """One DES-LOC step in place on [M][n] arrays (all float32 or all float64).

        vmax: the AMSGrad state, required when cfg.amsgrad (post-average Adam only).

        Norm-clip mode: sumsq_rest (float64 [M], optional) adds the squared norm of gradient
        coordinates not passed here; returns the per-worker gradient norms."""
        dtype = x.dtype
        if dtype not in (np.float32, np.float64):
            raise ValueError("x must be float32 or float64")
        M, n = x.shape
        if M != cfg.M:
            raise ValueError("x.shape[0] != cfg.M")
        if cfg.variant != SGDM and v is None:
            raise ValueError("v required for Adam/ADOPT")
        px = self._check(x, dtype, M, n, "x")
        pu = self._check(u, dtype, M, n, "u")
        pv = self._check(v, dtype, M, n, "v")
        pg = self._check(g, dtype, M, n, "g")
        c = cfg._c()
        if cfg.post_average:
            if cfg.variant == ADOPT:
                raise ValueError("post_average is defined for Adam and SGDM only")
            if cfg.amsgrad and (vmax is None or cfg.variant != ADAM):
                raise ValueError("amsgrad needs vmax and the Adam variant")
            rest = None
            if sumsq_rest is not None:
                rest = np.ascontiguousarray(sumsq_rest, dtype=np.float64)
            norms = np.zeros(M, dtype=dtype)
            fn = self.lib.oracle_step_post_f32 if dtype == np.float32 else self.lib.oracle_step_post_f64
            fn(ctypes.byref(c), t, n, px, pu, pv, self._check(vmax, dtype, M, n, "vmax"), pg,
               rest.ctypes.data_as(ctypes.c_void_p) if rest is not None else None,
               norms.ctypes.data_as(ctypes.c_void_p))
            return norms if cfg.norm_clip else None
        if cfg.amsgrad:
            raise ValueError("amsgrad is only defined together with post_average")
        if cfg.norm_clip:
            rest = None
            if sumsq_rest is not None:
                rest = np.ascontiguousarray(sumsq_rest, dtype=np.float64)
                assert rest.shape == (M,)
            norms = np.zeros(M, dtype=dtype)
            fn = self.lib.oracle_step_norm_f32 if dtype == np.float32 else self.lib.oracle_step_norm_f64
            fn(ctypes.byref(c), t, n, px, pu, pv, pg,
               rest.ctypes.data_as(ctypes.c_void_p) if rest is not None else None,
               norms.ctypes.data_as(ctypes.c_void_p))
            return norms
        if sumsq_rest is not None:
            raise ValueError("sumsq_rest only applies to norm-clip mode")
        fn = self.lib.oracle_step_f32 if dtype == np.float32 else self.lib.oracle_step_f64
        fn(ctypes.byref(c), t, n, px, pu, pv, pg)
        return None

    def state_change(self, s, ref):
        """(||s^m - ref^m||_2, ||ref^m||_2) per worker for float32 [M][n] arrays."""
        M, n = s.shape
        change = np.empty(M, np.float32)
        base = np.empty(M, np.float32)
        self.lib.oracle_state_change_f32(M, n, self._check(s, np.float32, M, n, "s"),
                                         self._check(ref, np.float32, M, n, "ref"),
                                         change.ctypes.data_as(ctypes.c_void_p),
                                         base.ctypes.data_as(ctypes.c_void_p))
        return change, base

    def state_change_tensors(self, s, ref, numel):
        """Per tensor and worker: (||s^m - ref^m||_2, ||ref^m||_2) as float32 [n_tensors][M];
        tensor k is the coordinate range after the first sum(numel[:k]) coordinates."""
        M, n = s.shape
        numel = np.ascontiguousarray(numel, dtype=np.uint64)
        if int(numel.sum()) > n:
            raise ValueError("tensor sizes exceed the row length")
        change = np.empty((numel.size, M), np.float32)
        base = np.empty((numel.size, M), np.float32)
        self.lib.oracle_state_change_tensors_f32(M, numel.size, numel.ctypes.data_as(ctypes.c_void_p), n,
                                                 self._check(s, np.float32, M, n, "s"),
                                                 self._check(ref, np.float32, M, n, "ref"),
                                                 change.ctypes.data_as(ctypes.c_void_p),
                                                 base.ctypes.data_as(ctypes.c_void_p))
        return change, base

    def worker_mean(self, s) -> np.ndarray:
        M, n = s.shape
        out = np.empty(n, dtype=s.dtype)
        fn = (self.lib.oracle_worker_mean_f32 if s.dtype == np.float32
              else self.lib.oracle_worker_mean_f64)
        fn(M, n, self._check(s, s.dtype, M, n, "s"), out.ctypes.data_as(ctypes.c_void_p))
        return out
