"""CPU oracle for DaSGD (Local SGD with delayed averaging, Eq. 2 of the paper).

TEST INFRASTRUCTURE ONLY: the GPU library never imports or calls this package; it exists so
that the tests, the smoke check and the benchmark's CPU-baseline leg have an independent,
plain implementation to compare against.  The arithmetic lives in dasgd_oracle.c; this file
is a ctypes wrapper plus a run loop that feeds it gradients.

Readings of the paper taken here (the text is silent or ambiguous on each):
  * momentum / weight decay (Section 4.1 gives only the constants): heavy-ball with coupled
    L2 decay, v <- momentum v + (g + wd x), x <- x - lr v, v_0 = 0;
  * momentum buffers are local state: never averaged, scaled or reset by a merge;
  * averages launch after local steps k with (k+1) mod tau == 0 and are merged exactly d
    steps later (appendix form of the trigger), first in first out, for any d >= 0;
  * the average is of the values after the local update and before any merge of that step;
  * the mean is a pairwise (tree-order) sum times 1/W;
  * averages still pending when the run ends are dropped.
"""
from __future__ import annotations

import ctypes
from typing import Callable, Optional

import numpy as np

from . import build as _build

_c_i64 = ctypes.c_int64
_LIBS = {}


def load(path: Optional[str] = None) -> ctypes.CDLL:
    """Load (building if needed) the oracle library and declare its signatures."""
    path = path or _build.build()
    if path in _LIBS:
        return _LIBS[path]
    lib = ctypes.CDLL(path)
    for suf, real in (("f32", ctypes.c_float), ("f64", ctypes.c_double)):
        rp = ctypes.POINTER(real)
        f = getattr(lib, f"dasgd_oracle_create_{suf}")
        f.restype = ctypes.c_void_p
        f.argtypes = [ctypes.c_int, _c_i64, ctypes.c_int, ctypes.c_int,
                      ctypes.c_double, ctypes.c_double, ctypes.c_double, ctypes.c_double, rp]
        getattr(lib, f"dasgd_oracle_destroy_{suf}").argtypes = [ctypes.c_void_p]
        getattr(lib, f"dasgd_oracle_destroy_{suf}").restype = None
        for nm in ("x", "v"):
            f = getattr(lib, f"dasgd_oracle_{nm}_{suf}")
            f.restype = rp
            f.argtypes = [ctypes.c_void_p]
        f = getattr(lib, f"dasgd_oracle_k_{suf}"); f.restype = _c_i64; f.argtypes = [ctypes.c_void_p]
        f = getattr(lib, f"dasgd_oracle_pending_{suf}"); f.restype = ctypes.c_int; f.argtypes = [ctypes.c_void_p]
        for nm in ("set_lr", "set_xi"):
            f = getattr(lib, f"dasgd_oracle_{nm}_{suf}")
            f.restype = None
            f.argtypes = [ctypes.c_void_p, ctypes.c_double]
        f = getattr(lib, f"dasgd_oracle_step_{suf}"); f.restype = ctypes.c_int; f.argtypes = [ctypes.c_void_p, rp]
        f = getattr(lib, f"dasgd_oracle_local_update_{suf}")
        f.restype = None
        f.argtypes = [ctypes.c_int, _c_i64, real, real, real, rp, rp, rp]
        f = getattr(lib, f"dasgd_oracle_mean_{suf}")
        f.restype = None
        f.argtypes = [ctypes.c_int, _c_i64, rp, rp]
        f = getattr(lib, f"dasgd_oracle_merge_{suf}")
        f.restype = None
        f.argtypes = [ctypes.c_int, _c_i64, real, rp, rp]
    lib.dasgd_oracle_set_threads.restype = ctypes.c_int
    lib.dasgd_oracle_set_threads.argtypes = [ctypes.c_int]
    _LIBS[path] = lib
    return lib


def set_threads(n: int, lib: Optional[ctypes.CDLL] = None) -> int:
    """Set the OpenMP thread count of the oracle loops; returns the count in effect."""
    return (lib or load()).dasgd_oracle_set_threads(int(n))


def f32(value: float) -> float:
    """Round a Python float to fp32 (the GPU library takes its constants as C floats; both
    oracle precisions start from the same rounded constants)."""
    return float(np.float32(value))


class Oracle:
    """One DaSGD run over W replicas of P parameters, held on the host.

    dtype "f64" is the reference; "f32" does the same operations in single precision.
    `x` and `v` are numpy views of shape [W, P] into the oracle's own memory.
    """

    def __init__(self, W: int, P: int, d: int, tau: int, lr: float, momentum: float, wd: float,
                 w0: np.ndarray, xi: float = 0.25, dtype: str = "f64",
                 lib: Optional[ctypes.CDLL] = None):
        assert dtype in ("f32", "f64")
        self.lib = lib or load()
        self.suf = dtype
        self.np_dtype = np.float32 if dtype == "f32" else np.float64
        self.c_real = ctypes.c_float if dtype == "f32" else ctypes.c_double
        self.W, self.P, self.d, self.tau = int(W), int(P), int(d), int(tau)
        w0 = np.ascontiguousarray(np.asarray(w0).reshape(-1), dtype=self.np_dtype)
        assert w0.size == self.P
        create = getattr(self.lib, f"dasgd_oracle_create_{dtype}")
        self._h = create(self.W, self.P, self.d, self.tau, f32(lr), f32(momentum), f32(wd), f32(xi),
                         w0.ctypes.data_as(ctypes.POINTER(self.c_real)))
        if not self._h:
            raise ValueError("dasgd_oracle_create rejected the arguments")
        self.x = self._view("x")
        self.v = self._view("v")

    def _fn(self, name: str):
        return getattr(self.lib, f"dasgd_oracle_{name}_{self.suf}")

    def _view(self, name: str) -> np.ndarray:
        ptr = self._fn(name)(self._h)
        return np.ctypeslib.as_array(ptr, shape=(self.W, self.P))

    @property
    def k(self) -> int:
        return int(self._fn("k")(self._h))

    @property
    def n_pending(self) -> int:
        return int(self._fn("pending")(self._h))

    def set_lr(self, lr: float) -> None:
        self._fn("set_lr")(self._h, f32(lr))

    def set_xi(self, xi: float) -> None:
        self._fn("set_xi")(self._h, f32(xi))

    def step(self, g: np.ndarray) -> int:
        """Run iteration k with gradients g [W, P]; returns 1 if an average was launched,
        2 if a merge was applied, 3 if both."""
        g = np.ascontiguousarray(g, dtype=self.np_dtype)
        assert g.shape == (self.W, self.P), (g.shape, (self.W, self.P))
        rc = self._fn("step")(self._h, g.ctypes.data_as(ctypes.POINTER(self.c_real)))
        if rc < 0:
            raise RuntimeError("oracle step failed")
        return rc

    def run(self, steps: int, grad_fn: Callable[[int, np.ndarray], np.ndarray],
            observer: Optional[Callable[[int, "Oracle", int], None]] = None) -> np.ndarray:
        """Run `steps` iterations; grad_fn(k, x) returns the [W, P] gradients at the current x.
        observer(k, oracle, what) is called after every step.  Returns x."""
        for _ in range(steps):
            k = self.k
            what = self.step(grad_fn(k, self.x))
            if observer is not None:
                observer(k, self, what)
        return self.x

    def close(self) -> None:
        if getattr(self, "_h", None):
            self.x = self.v = None
            self._fn("destroy")(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def local_update(x: np.ndarray, v: np.ndarray, g: np.ndarray, lr: float, momentum: float, wd: float,
                 lib: Optional[ctypes.CDLL] = None) -> None:
    """In-place local update of x, v ([W, P], fp32 or fp64 by x.dtype)."""
    lib = lib or load()
    suf, real = _suffix(x)
    assert x.dtype == v.dtype == g.dtype and x.shape == v.shape == g.shape and x.ndim == 2
    for a in (x, v, g):
        assert a.flags.c_contiguous
    rp = ctypes.POINTER(real)
    getattr(lib, f"dasgd_oracle_local_update_{suf}")(
        x.shape[0], x.shape[1], f32(lr), f32(momentum), f32(wd),
        x.ctypes.data_as(rp), v.ctypes.data_as(rp), g.ctypes.data_as(rp))


def mean(y: np.ndarray, lib: Optional[ctypes.CDLL] = None) -> np.ndarray:
    """Cross-replica mean of y [W, P] -> [P]."""
    lib = lib or load()
    suf, real = _suffix(y)
    assert y.ndim == 2 and y.flags.c_contiguous
    A = np.empty(y.shape[1], dtype=y.dtype)
    rp = ctypes.POINTER(real)
    getattr(lib, f"dasgd_oracle_mean_{suf}")(y.shape[0], y.shape[1], y.ctypes.data_as(rp), A.ctypes.data_as(rp))
    return A


def merge(x: np.ndarray, A: np.ndarray, xi: float, lib: Optional[ctypes.CDLL] = None) -> None:
    """In-place merge x <- xi x + (1 - xi) A for x [W, P], A [P]."""
    lib = lib or load()
    suf, real = _suffix(x)
    assert x.ndim == 2 and x.flags.c_contiguous and A.flags.c_contiguous and A.dtype == x.dtype
    assert A.shape == (x.shape[1],)
    rp = ctypes.POINTER(real)
    getattr(lib, f"dasgd_oracle_merge_{suf}")(x.shape[0], x.shape[1], f32(xi), x.ctypes.data_as(rp), A.ctypes.data_as(rp))


def _suffix(a: np.ndarray):
    if a.dtype == np.float32:
        return "f32", ctypes.c_float
    if a.dtype == np.float64:
        return "f64", ctypes.c_double
    raise TypeError(a.dtype)
