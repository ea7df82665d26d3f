"""ctypes loader for the multi-threaded CPU baseline (TEST INFRASTRUCTURE, not the product).

``Workers`` drives the state of an existing ``Oracle`` with W threads (per_workers.c); results and
state are bit-identical to the sequential oracle's, which the CPU tests check.  Only tests and the
bench's CPU leg may import this.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

from .per_oracle import Oracle, _ptr

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "per_workers.c")
_DEP = os.path.join(_HERE, "per_oracle.c")
_LIB = os.path.join(_HERE, "libper_workers.so")


def build(force: bool = False) -> str:
    """Compile with gcc and OpenMP (no fast-math, no FMA contraction)."""
    newest = max(os.path.getmtime(_SRC), os.path.getmtime(_DEP))
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        subprocess.check_call([
            "gcc", "-std=c99", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra",
            "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = C.CDLL(build())
        vp, u32, f32, i = C.c_void_p, C.c_uint32, C.c_float, C.c_int
        lib.workers_max_threads.restype = i
        lib.workers_sample.restype = i
        lib.workers_sample.argtypes = [vp, u32, f32, vp, vp, vp, vp, i]
        lib.workers_gather.argtypes = [vp, u32, vp, vp, i]
        lib.workers_update.restype = i
        lib.workers_update.argtypes = [vp, u32, vp, vp, i]
        lib.workers_release.argtypes = [vp]
        _lib = lib
    return _lib


def default_threads() -> int:
    """Worker count: the cores this process may run on (OpenMP's own limit if lower)."""
    n = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    return max(1, min(n, _load().workers_max_threads()))


class Workers:
    """Same calls as ``Oracle.sample / gather / update`` on the oracle's state, on ``threads`` workers."""

    def __init__(self, oracle: Oracle, threads: int = 0):
        self.lib = _load()
        self.o = oracle
        self.threads = threads or default_threads()

    def __del__(self):
        if getattr(self, "o", None) is not None and getattr(self.o, "_h", None):
            self.lib.workers_release(self.o._h)

    def sample(self, u: np.ndarray, beta: float = 0.4, want_weights: bool = True):
        u = np.ascontiguousarray(u, dtype=np.float32)
        B = u.size
        idx = np.empty(B, dtype=np.uint32)
        w = np.empty(B, dtype=np.float32) if want_weights else None
        v = np.empty(B, dtype=np.float32)
        self.lib.workers_sample(self.o._h, B, beta, _ptr(u), _ptr(idx), _ptr(w), _ptr(v), self.threads)
        return idx, w, v

    def gather(self, idx: np.ndarray):
        idx = np.ascontiguousarray(idx, dtype=np.uint32)
        outs = [np.empty((idx.size, b), dtype=np.uint8) for b in self.o.field_bytes]
        arr = (C.c_void_p * max(1, len(outs)))(*[o.ctypes.data for o in outs])
        self.lib.workers_gather(self.o._h, idx.size, _ptr(idx), arr, self.threads)
        return outs

    def update(self, idx: np.ndarray, prio: np.ndarray) -> None:
        idx = np.ascontiguousarray(idx, dtype=np.uint32)
        prio = np.ascontiguousarray(prio, dtype=np.float32)
        if self.lib.workers_update(self.o._h, idx.size, _ptr(idx), _ptr(prio), self.threads) != 0:
            raise MemoryError("workers_update: work arrays")
