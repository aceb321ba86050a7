"""ctypes front end of oracle/def_oracle.c with the interface of DefOracle.

TEST INFRASTRUCTURE ONLY.  The C file holds the arithmetic; this wrapper holds
the state arrays, draws the block start (oracle/philox.py) and calls it.
float32 only.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

from .def_oracle import block_length
from .philox import block_start

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "def_oracle.c")
_LIB = os.path.join(_HERE, "libdef_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile def_oracle.c with gcc (no contraction, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
                               "-Wall", "-Wextra", "-o", _LIB, _SRC])
    return _LIB


def load(path: str):
    """A CDLL of a build of def_oracle.c with the argument types set."""
    L = ctypes.CDLL(path)
    _declare(L)
    return L


def lib():
    global _lib
    if _lib is None:
        _lib = load(build())
    return _lib


def _declare(L) -> None:
    f32p = ctypes.POINTER(ctypes.c_float)
    i64p = ctypes.POINTER(ctypes.c_int64)
    L.def_oracle_step_f32.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int32,
                                      ctypes.c_int64, ctypes.c_int64,
                                      ctypes.c_float, ctypes.c_float, ctypes.c_float,
                                      f32p, f32p, f32p, f32p, ctypes.c_int64, i64p, f32p]
    L.def_oracle_step_f32.restype = None
    L.def_oracle_y_f32.argtypes = [ctypes.c_int64, ctypes.c_int32, f32p, f32p, f32p]
    L.def_oracle_y_f32.restype = None
    L.def_oracle_detach_f32.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_float, f32p, f32p, f32p]
    L.def_oracle_detach_f32.restype = None
    L.def_oracle_threads.restype = ctypes.c_int
    L.def_oracle_set_threads.argtypes = [ctypes.c_int]


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


class DefOracleC:
    def __init__(self, x0, W: int, R: int, lr: float, momentum: float = 0.0,
                 weight_decay: float = 0.0, seed: int = 0, d: Optional[int] = None,
                 index=None, threads: Optional[int] = None, library=None):
        self.dtype = np.dtype(np.float32)
        self.x = np.ascontiguousarray(x0, dtype=np.float32).copy()
        n = self.x.shape[0]
        self.d = int(n if d is None else d)
        self.index = None if index is None else np.ascontiguousarray(index, dtype=np.int64).copy()
        if self.index is not None and self.index.shape != (n,):
            raise ValueError("index must have one entry per column of x0")
        self.W, self.R = int(W), int(R)
        self.B = block_length(self.d, self.R)
        self.lr, self.mu, self.wd = np.float32(lr), np.float32(momentum), np.float32(weight_decay)
        self.seed, self.t = int(seed), 0
        self.e = np.zeros((self.W, n), dtype=np.float32)
        self.m = np.zeros((self.W, n), dtype=np.float32)
        self.last_start = None
        self.last_cbar_dense = np.zeros(n, dtype=np.float32)
        self._lib = library if library is not None else lib()   # (a mutated build, in the pin tests)
        if threads is not None:
            self._lib.def_oracle_set_threads(int(threads))

    @property
    def threads(self) -> int:
        return int(self._lib.def_oracle_threads())

    def set_threads(self, threads: int) -> None:
        """OpenMP threads the C routines use from now on (process-wide)."""
        self._lib.def_oracle_set_threads(int(threads))

    def set_lr(self, lr: float) -> None:
        self.lr = np.float32(lr)

    def set_seed(self, seed: int) -> None:
        self.seed = int(seed)

    def set_step(self, t: int) -> None:
        self.t = int(t)

    def step(self, g, start: Optional[int] = None) -> int:
        g = np.asarray(g)
        if g.dtype != np.float32 or g.ndim != 2 or g.shape[0] != self.W or g.shape[1] < self.x.shape[0] \
                or g.strides[1] != 4:
            raise ValueError("g must be float32 [W][>=n] with unit column stride")
        s = block_start(self.seed, self.t, self.d) if start is None else int(start)
        if not 0 <= s < self.d:
            raise ValueError("start out of range")
        n = self.x.shape[0]
        idx = None if self.index is None else self.index.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))
        self._lib.def_oracle_step_f32(n, self.d, self.W, self.B, s, self.lr, self.mu, self.wd,
                                      _p(self.x), _p(self.e), _p(self.m), _p(g),
                                      g.strides[0] // 4, idx, _p(self.last_cbar_dense))
        self.last_start = s
        self.t += 1
        return s

    def y(self) -> np.ndarray:
        out = np.empty_like(self.x)
        self._lib.def_oracle_y_f32(self.x.shape[0], self.W, _p(self.x), _p(self.e), _p(out))
        return out

    def detached_points(self, lam: float) -> np.ndarray:
        out = np.empty_like(self.e)
        self._lib.def_oracle_detach_f32(self.x.shape[0], self.W, np.float32(lam), _p(self.x), _p(self.e),
                                        _p(out))
        return out

    def compact_block(self) -> np.ndarray:
        if self.index is not None:
            raise ValueError("compact_block needs the full index range")
        j = (np.int64(self.last_start) + np.arange(self.B, dtype=np.int64)) % np.int64(self.d)
        return self.last_cbar_dense[j]

    def get_state(self) -> dict:
        return dict(x=self.x.copy(), e=self.e.copy(), m=self.m.copy(), t=self.t, seed=self.seed,
                    lr=float(self.lr))

    def set_state(self, st: dict) -> None:
        self.x = np.ascontiguousarray(st["x"], dtype=np.float32).copy()
        self.e = np.ascontiguousarray(st["e"], dtype=np.float32).copy()
        self.m = np.ascontiguousarray(st["m"], dtype=np.float32).copy()
        self.t, self.seed, self.lr = int(st["t"]), int(st["seed"]), np.float32(st["lr"])
