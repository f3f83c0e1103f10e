"""ctypes binding of shadow_oracle.c and the per-iteration driver (TEST INFRASTRUCTURE ONLY).

The driver mirrors the loop the paper gives for shadow nodes (section 4.2.3,
second listing): receive every bucket of the iteration, then run the optimizer
step over all parameters.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence

import numpy as np

from .layout import Layout, build_layout

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "shadow_oracle.c")
_SO = os.path.join(_HERE, "liboracle.so")
CFLAGS = ["-O2", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, no GPU toolchain involved)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        tmp = _SO + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", *CFLAGS, "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _SO)
    return _SO


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        L = _lib
        pp = C.POINTER(C.c_void_p)
        L.oracle_set_threads.argtypes = [C.c_int]
        L.oracle_get_threads.restype = C.c_int
        L.oracle_widen_bf16.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p]
        for name in ("oracle_fold_f32", "oracle_fold_bf16", "oracle_fold_f32_f64", "oracle_fold_bf16_f64"):
            getattr(L, name).argtypes = [pp, C.c_uint32, C.c_uint64, C.c_int, C.c_void_p]
            getattr(L, name).restype = None
        L.oracle_sumsq_accumulate.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p]
        L.oracle_sumsq_accumulate_f64.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p]
        L.oracle_sumsq_accumulate_weighted.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p]
        L.oracle_sumsq_value.argtypes = [C.c_void_p]
        L.oracle_sumsq_value.restype = C.c_double
        L.oracle_clip_coef_f64.argtypes = [C.c_void_p, C.c_float]
        L.oracle_clip_coef_f64.restype = C.c_double
        L.oracle_clip_coef_f32.argtypes = [C.c_void_p, C.c_float]
        L.oracle_clip_coef_f32.restype = C.c_float
        L.oracle_step_scalars.argtypes = [C.c_float] * 4 + [C.c_uint64, C.c_void_p]
        L.oracle_adamw_f32.argtypes = ([C.c_void_p] * 4 + [C.c_uint64, C.c_int] + [C.c_float] * 5
                                       + [C.c_uint64, C.c_int, C.c_float])
        L.oracle_adamw_f64.argtypes = ([C.c_void_p] * 4 + [C.c_uint64, C.c_int] + [C.c_double] * 5
                                       + [C.c_uint64, C.c_int, C.c_double])
        L.oracle_adam_f32.argtypes = L.oracle_adamw_f32.argtypes
        L.oracle_adam_f64.argtypes = L.oracle_adamw_f64.argtypes
        L.oracle_sgd_f32.argtypes = [C.c_void_p] * 3 + [C.c_uint64, C.c_int] + [C.c_float] * 3 + [C.c_int, C.c_float]
        L.oracle_sgd_f64.argtypes = [C.c_void_p] * 3 + [C.c_uint64, C.c_int] + [C.c_double] * 3 + [C.c_int, C.c_double]
        for name in ("oracle_set_threads", "oracle_widen_bf16", "oracle_sumsq_accumulate",
                     "oracle_sumsq_accumulate_f64", "oracle_sumsq_accumulate_weighted",
                     "oracle_step_scalars", "oracle_adamw_f32", "oracle_adamw_f64", "oracle_adam_f32",
                     "oracle_adam_f64", "oracle_sgd_f32", "oracle_sgd_f64"):
            getattr(L, name).restype = None
    return _lib


def _bind_alternate(path: str):
    """Context manager: route every call to another build of the oracle's C file.

    Used only by the tests that plant a mistake in a copy of the C source and
    check that the pins notice.
    """
    import contextlib

    @contextlib.contextmanager
    def cm():
        global _lib
        saved = _lib
        _lib = None
        real_build = globals()["build"]
        globals()["build"] = lambda force=False: path
        try:
            lib()
            yield
        finally:
            globals()["build"] = real_build
            _lib = saved

    return cm()


def set_threads(n: int) -> None:
    lib().oracle_set_threads(int(n))


def get_threads() -> int:
    return int(lib().oracle_get_threads())


def _ptr(a: np.ndarray) -> C.c_void_p:
    return C.c_void_p(a.ctypes.data)


def _chk(a: np.ndarray, dtype) -> np.ndarray:
    if not (isinstance(a, np.ndarray) and a.dtype == dtype and a.flags["C_CONTIGUOUS"] and a.ndim == 1):
        raise TypeError(f"need contiguous 1-D {dtype}, got {getattr(a, 'dtype', type(a))}")
    return a


def widen_bf16(h: np.ndarray) -> np.ndarray:
    h = _chk(h, np.uint16)
    out = np.empty(h.shape, np.float32)
    lib().oracle_widen_bf16(_ptr(h), h.size, _ptr(out))
    return out


def fold(views: Sequence[np.ndarray], mean: bool = True, precision: str = "f32") -> np.ndarray:
    """Reduce W gradient views (all float32, or all uint16 bfloat16 patterns)."""
    W = len(views)
    n = views[0].size
    dt = views[0].dtype
    for g in views:
        _chk(g, dt)
        if g.size != n:
            raise ValueError("views differ in length")
    arr = (C.c_void_p * W)(*[g.ctypes.data for g in views])
    kind = {np.dtype(np.float32): "f32", np.dtype(np.uint16): "bf16"}[np.dtype(dt)]
    if precision == "f32":
        r = np.empty(n, np.float32)
        getattr(lib(), f"oracle_fold_{kind}")(arr, W, n, int(mean), _ptr(r))
    else:
        r = np.empty(n, np.float64)
        getattr(lib(), f"oracle_fold_{kind}_f64")(arr, W, n, int(mean), _ptr(r))
    return r


class SumSq:
    """Extended-precision running sum of squares of the reduced gradient."""

    def __init__(self) -> None:
        self._acc = C.c_longdouble(0.0)

    def add(self, r: np.ndarray, count: Optional[np.ndarray] = None) -> "SumSq":
        if count is not None:
            _chk(r, np.float32), _chk(count, np.uint64)
            lib().oracle_sumsq_accumulate_weighted(_ptr(r), _ptr(count), r.size, C.byref(self._acc))
        elif r.dtype == np.float32:
            lib().oracle_sumsq_accumulate(_ptr(_chk(r, np.float32)), r.size, C.byref(self._acc))
        else:
            lib().oracle_sumsq_accumulate_f64(_ptr(_chk(r, np.float64)), r.size, C.byref(self._acc))
        return self

    @property
    def value(self) -> float:
        return float(lib().oracle_sumsq_value(C.byref(self._acc)))

    def coef(self, max_norm: float, precision: str = "f32"):
        if precision == "f32":
            return np.float32(lib().oracle_clip_coef_f32(C.byref(self._acc), C.c_float(max_norm)))
        return float(lib().oracle_clip_coef_f64(C.byref(self._acc), C.c_float(max_norm)))


def clip_coef(rs: Sequence[np.ndarray], max_norm: float, precision: str = "f32"):
    s = SumSq()
    for r in rs:
        s.add(r)
    return s.coef(max_norm, precision)


@dataclass
class HParams:
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.01
    max_grad_norm: float = 0.0      # <= 0: clipping off
    mean: bool = True               # average (True) or sum (False) over workers
    optimizer: str = "adamw"        # "adamw" | "adam" (L2 penalty in the gradient) | "sgd" (momentum = beta1)

    def f32(self, name: str) -> float:
        """The hyper-parameter as the float the method receives, widened."""
        return float(np.float32(getattr(self, name)))


def step_scalars(hp: HParams, t: int) -> np.ndarray:
    out = np.empty(5, np.float32)
    lib().oracle_step_scalars(hp.lr, hp.beta1, hp.beta2, hp.weight_decay, int(t), _ptr(out))
    return out


def adamw_f32(p, m, v, r, wd_flag: bool, hp: HParams, t: int, c=None) -> None:
    """In place on float32 arrays; c is the clip coefficient or None (clipping off)."""
    n = p.size
    for a in (p, m, v, r):
        _chk(a, np.float32)
        assert a.size == n
    lib().oracle_adamw_f32(_ptr(p), _ptr(m), _ptr(v), _ptr(r), n, int(bool(wd_flag)),
                           hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay, int(t),
                           int(c is not None), C.c_float(0.0 if c is None else float(c)))


def adam_f32(p, m, v, r, wd_flag: bool, hp: HParams, t: int, c=None) -> None:
    n = p.size
    for a in (p, m, v, r):
        _chk(a, np.float32)
        assert a.size == n
    lib().oracle_adam_f32(_ptr(p), _ptr(m), _ptr(v), _ptr(r), n, int(bool(wd_flag)),
                          hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay, int(t),
                          int(c is not None), C.c_float(0.0 if c is None else float(c)))


def adam_f64(p, m, v, r, wd_flag: bool, hp: HParams, t: int, c=None) -> None:
    n = p.size
    for a in (p, m, v, r):
        _chk(a, np.float64)
        assert a.size == n
    lib().oracle_adam_f64(_ptr(p), _ptr(m), _ptr(v), _ptr(r), n, int(bool(wd_flag)),
                          hp.f32("lr"), hp.f32("beta1"), hp.f32("beta2"), hp.f32("eps"),
                          hp.f32("weight_decay"), int(t), int(c is not None),
                          C.c_double(0.0 if c is None else float(c)))


def sgd_f32(p, b, r, wd_flag: bool, hp: HParams, c=None) -> None:
    """Momentum SGD; the momentum coefficient is hp.beta1, the buffer b lives where Adam keeps m."""
    n = p.size
    for a in (p, b, r):
        _chk(a, np.float32)
        assert a.size == n
    lib().oracle_sgd_f32(_ptr(p), _ptr(b), _ptr(r), n, int(bool(wd_flag)), hp.lr, hp.beta1, hp.weight_decay,
                         int(c is not None), C.c_float(0.0 if c is None else float(c)))


def sgd_f64(p, b, r, wd_flag: bool, hp: HParams, c=None) -> None:
    n = p.size
    for a in (p, b, r):
        _chk(a, np.float64)
        assert a.size == n
    lib().oracle_sgd_f64(_ptr(p), _ptr(b), _ptr(r), n, int(bool(wd_flag)), hp.f32("lr"), hp.f32("beta1"),
                         hp.f32("weight_decay"), int(c is not None), C.c_double(0.0 if c is None else float(c)))


def adamw_f64(p, m, v, r, wd_flag: bool, hp: HParams, t: int, c=None) -> None:
    n = p.size
    for a in (p, m, v, r):
        _chk(a, np.float64)
        assert a.size == n
    lib().oracle_adamw_f64(_ptr(p), _ptr(m), _ptr(v), _ptr(r), n, int(bool(wd_flag)),
                           hp.f32("lr"), hp.f32("beta1"), hp.f32("beta2"), hp.f32("eps"),
                           hp.f32("weight_decay"), int(t), int(c is not None),
                           C.c_double(0.0 if c is None else float(c)))


class OracleShadow:
    """The shadow replica: per-bucket param/m/v arrays and the per-iteration update.

    precision "f32": canonical float evaluation; "f64": textbook formulas in double.
    """

    def __init__(self, layout: Layout, hp: HParams, params: Sequence[np.ndarray],
                 precision: str = "f32", start_step: int = 0,
                 m: Optional[Sequence[np.ndarray]] = None, v: Optional[Sequence[np.ndarray]] = None):
        """params (and m, v if given): one array per bucket; an entry may be None for a
        bucket whose state is not kept (then only update_bucket on the others is usable)."""
        self.layout, self.hp, self.precision = layout, hp, precision
        self.dt = np.float32 if precision == "f32" else np.float64
        self.p = [None if x is None else np.array(x, dtype=self.dt).copy() for x in params]
        zeros = [None if x is None else np.zeros(x.size, self.dt) for x in self.p]
        self.m = zeros if m is None else [None if x is None else np.array(x, dtype=self.dt).copy() for x in m]
        self.v = [None if x is None else z.copy() for x, z in zip(self.p, zeros)] if v is None else \
                 [None if x is None else np.array(x, dtype=self.dt).copy() for x in v]
        for b, arr in zip(layout.buckets, self.p):
            assert arr is None or arr.size == b.numel
        self.t = int(start_step)
        self.last_coef = None
        self.last_sumsq = None

    def update_bucket(self, b: int, r: np.ndarray, t: int, c) -> None:
        """Optimizer step on bucket b's tensors, each through its offset view."""
        f32 = self.precision == "f32"
        for s in self.layout.buckets[b].segments:
            sl = slice(s.offset, s.offset + s.numel)
            if self.hp.optimizer == "sgd":
                (sgd_f32 if f32 else sgd_f64)(self.p[b][sl], self.m[b][sl], r[sl], s.weight_decay, self.hp, c)
            else:
                fn = {"adamw": (adamw_f32, adamw_f64), "adam": (adam_f32, adam_f64)}[self.hp.optimizer][0 if f32 else 1]
                fn(self.p[b][sl], self.m[b][sl], self.v[b][sl], r[sl], s.weight_decay, self.hp, t, c)

    def step(self, grads: Dict[int, Sequence[np.ndarray]]) -> None:
        """One iteration: every bucket's W views must be present exactly once."""
        B = len(self.layout.buckets)
        if sorted(grads.keys()) != list(range(B)):
            raise ValueError("an iteration needs every bucket exactly once")
        t = self.t + 1
        r = [fold(grads[b], self.hp.mean, self.precision) for b in range(B)]
        c = None
        if self.hp.max_grad_norm > 0:
            s = SumSq()
            for b in range(B):
                s.add(r[b])
            self.last_sumsq = s.value
            c = s.coef(self.hp.max_grad_norm, self.precision)
            self.last_coef = c
        for b in range(B):
            self.update_bucket(b, r[b], t, c)
        self.t = t
