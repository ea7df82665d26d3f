"""ctypes loader for the CPU oracle (TEST INFRASTRUCTURE, not the product).

Only tests, ``__graft_entry__.smoke()`` and the bench's ``cpu_baseline`` leg may
import this.  It never touches the HIP library.  ``MultiOracle`` runs T
independent oracles side by side, mirroring the [T][...] array layout of the
batched multi-tree calls.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "per_oracle.c")
_LIB = os.path.join(_HERE, "libper_oracle.so")

FLAG_BAD_INDEX, FLAG_BAD_PRIORITY, FLAG_ZERO_TOTAL = 1, 2, 4


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call([
            "gcc", "-std=c99", "-O2", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra",
            "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    lib = C.CDLL(build())
    vp, u32, u64, f32 = C.c_void_p, C.c_uint32, C.c_uint64, C.c_float
    lib.oracle_create.restype = vp
    lib.oracle_create.argtypes = [u32, u64, u32, C.POINTER(u32), f32, C.c_int]
    lib.oracle_destroy.argtypes = [vp]
    lib.oracle_update.argtypes = [vp, u32, vp, vp]
    lib.oracle_update_delta.argtypes = [vp, u32, vp, vp]
    lib.oracle_update_td.argtypes = [vp, u32, vp, vp, C.c_double, C.c_double]
    lib.oracle_insert.restype = C.c_int
    lib.oracle_insert.argtypes = [vp, u32, vp, vp, vp]
    lib.oracle_insert_protected.restype = C.c_int
    lib.oracle_insert_protected.argtypes = [vp, u32, vp, vp, vp, u32, vp]
    lib.oracle_set_weight_norm.restype = C.c_int
    lib.oracle_set_weight_norm.argtypes = [vp, C.c_int]
    lib.oracle_sample.restype = C.c_int
    lib.oracle_sample.argtypes = [vp, u32, f32, vp, vp, vp, vp]
    lib.oracle_gather.argtypes = [vp, u32, vp, vp]
    lib.oracle_philox4x32_10.argtypes = [vp, vp, vp]
    lib.oracle_uniforms.argtypes = [u64, u64, u32, u32, vp]
    lib.oracle_get_priority.argtypes = [vp, u32, vp, vp]
    lib.oracle_level_count.restype = u64
    lib.oracle_level_count.argtypes = [vp, u32]
    lib.oracle_read_level.restype = C.c_int
    lib.oracle_read_level.argtypes = [vp, u32, vp, C.POINTER(u64)]
    lib.oracle_read_binary_depth.restype = C.c_int
    lib.oracle_read_binary_depth.argtypes = [vp, u32, vp, u64]
    for name, rt in [("oracle_total", f32), ("oracle_max_priority", f32), ("oracle_size", u64),
                     ("oracle_cursor", u64), ("oracle_height", u32), ("oracle_binary_height", u32),
                     ("oracle_status", u32)]:
        getattr(lib, name).restype = rt
        getattr(lib, name).argtypes = [vp]
    lib.oracle_clear_status.argtypes = [vp]
    _lib = lib
    return lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def philox4x32_10(ctr, key) -> np.ndarray:
    """One block of the counter-based generator (4 counter words, 2 key words -> 4 output words)."""
    c = np.ascontiguousarray(ctr, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.empty(4, dtype=np.uint32)
    _load().oracle_philox4x32_10(_ptr(c), _ptr(k), _ptr(out))
    return out


def uniforms(seed: int, call: int, tree: int, B: int) -> np.ndarray:
    """The uniforms of sampling call number `call` of tree `tree` under `seed`."""
    u = np.empty(B, dtype=np.float32)
    _load().oracle_uniforms(int(seed), int(call), int(tree), int(B), _ptr(u))
    return u


class Oracle:
    """One prioritized replay buffer on the CPU."""

    def __init__(self, K: int, N: int, field_bytes: Sequence[int] = (), init_max: float = 1.0,
                 with_payload: bool = True):
        self._lib = _load()
        self.K, self.N = int(K), int(N)
        self.field_bytes = tuple(int(b) for b in field_bytes)
        fb = (C.c_uint32 * max(1, len(self.field_bytes)))(*self.field_bytes)
        self._h = self._lib.oracle_create(self.K, self.N, len(self.field_bytes), fb,
                                          float(init_max), 1 if with_payload else 0)
        if not self._h:
            raise ValueError("oracle_create failed (bad fanout / capacity / field count, or out of memory)")
        self.with_payload = with_payload
        self.H = self._lib.oracle_height(self._h)
        self.HB = self._lib.oracle_binary_height(self._h)

    def __del__(self):
        if getattr(self, "_h", None):
            self._lib.oracle_destroy(self._h)
            self._h = None

    # -- operations -----------------------------------------------------------------
    def insert(self, n: int, rows: Optional[Sequence[np.ndarray]] = None,
               prio: Optional[np.ndarray] = None, protect: Optional[np.ndarray] = None) -> np.ndarray:
        """protect: indices whose slots must not be overwritten (their rows are deferred, slot 0xFFFFFFFF)."""
        out = np.empty(n, dtype=np.uint32)
        src = None
        keep = []
        if rows is not None:
            assert len(rows) == len(self.field_bytes)
            arr = (C.c_void_p * len(rows))()
            for f, r in enumerate(rows):
                r = np.ascontiguousarray(r).view(np.uint8).reshape(n, self.field_bytes[f])
                keep.append(r)
                arr[f] = r.ctypes.data
            src = C.cast(arr, C.c_void_p)
        p = None if prio is None else np.ascontiguousarray(prio, dtype=np.float32)
        if p is not None:
            assert p.shape == (n,)
        if protect is not None:
            pr = np.ascontiguousarray(protect, dtype=np.uint32).ravel()
            rc = self._lib.oracle_insert_protected(self._h, n, src, _ptr(p), _ptr(out), pr.size, _ptr(pr))
        else:
            rc = self._lib.oracle_insert(self._h, n, src, _ptr(p), _ptr(out))
        if rc != 0:
            raise ValueError(f"oracle_insert rc={rc}")
        return out

    def sample(self, u: np.ndarray, beta: float = 0.4, want_weights: bool = True):
        u = np.ascontiguousarray(u, dtype=np.float32)
        B = u.shape[0]
        idx = np.empty(B, dtype=np.uint32)
        w = np.empty(B, dtype=np.float32) if want_weights else None
        v = np.empty(B, dtype=np.float32)
        self._lib.oracle_sample(self._h, B, float(beta), _ptr(u), _ptr(idx), _ptr(w), _ptr(v))
        return idx, w, v

    def gather(self, idx: np.ndarray):
        idx = np.ascontiguousarray(idx, dtype=np.uint32)
        B = idx.shape[0]
        outs = [np.empty((B, b), dtype=np.uint8) for b in self.field_bytes]
        arr = (C.c_void_p * max(1, len(outs)))(*[o.ctypes.data for o in outs])
        self._lib.oracle_gather(self._h, B, _ptr(idx), C.cast(arr, C.c_void_p))
        return outs

    def update(self, idx: np.ndarray, prio: np.ndarray) -> None:
        idx = np.ascontiguousarray(idx, dtype=np.uint32)
        prio = np.ascontiguousarray(prio, dtype=np.float32)
        assert idx.shape == prio.shape and idx.ndim == 1
        self._lib.oracle_update(self._h, idx.shape[0], _ptr(idx), _ptr(prio))

    def update_td(self, idx: np.ndarray, td: np.ndarray, eps: float, alpha: float) -> None:
        idx = np.ascontiguousarray(idx, dtype=np.uint32)
        td = np.ascontiguousarray(td, dtype=np.float32)
        assert idx.shape == td.shape and idx.ndim == 1
        self._lib.oracle_update_td(self._h, idx.shape[0], _ptr(idx), _ptr(td), float(eps), float(alpha))

    def update_delta(self, idx: np.ndarray, delta: np.ndarray) -> None:
        idx = np.ascontiguousarray(idx, dtype=np.uint32)
        delta = np.ascontiguousarray(delta, dtype=np.float32)
        assert idx.shape == delta.shape and idx.ndim == 1
        self._lib.oracle_update_delta(self._h, idx.shape[0], _ptr(idx), _ptr(delta))

    def get_priority(self, idx: np.ndarray) -> np.ndarray:
        idx = np.ascontiguousarray(idx, dtype=np.uint32)
        out = np.empty(idx.shape[0], dtype=np.float32)
        self._lib.oracle_get_priority(self._h, idx.shape[0], _ptr(idx), _ptr(out))
        return out

    # -- inspection -----------------------------------------------------------------
    def level_count(self, height: int) -> int:
        return int(self._lib.oracle_level_count(self._h, height))

    def read_level(self, height: int) -> np.ndarray:
        out = np.empty(self.level_count(height), dtype=np.float32)
        cnt = C.c_uint64(0)
        if self._lib.oracle_read_level(self._h, height, _ptr(out), C.byref(cnt)) != 0:
            raise ValueError("bad height")
        return out

    def read_binary_depth(self, depth: int) -> np.ndarray:
        out = np.empty(1 << depth, dtype=np.float32)
        if self._lib.oracle_read_binary_depth(self._h, depth, _ptr(out), out.shape[0]) != 0:
            raise ValueError("bad depth")
        return out

    @property
    def total(self) -> float:
        return float(self._lib.oracle_total(self._h))

    @property
    def max_priority(self) -> float:
        return float(self._lib.oracle_max_priority(self._h))

    @property
    def size(self) -> int:
        return int(self._lib.oracle_size(self._h))

    @property
    def cursor(self) -> int:
        return int(self._lib.oracle_cursor(self._h))

    def set_weight_norm(self, mode: str) -> None:
        """'batch': weights relative to the largest weight of the sampled batch; 'buffer': of all stored rows."""
        if self._lib.oracle_set_weight_norm(self._h, {"batch": 0, "buffer": 1}[mode]) != 0:
            raise ValueError(mode)

    @property
    def status(self) -> int:
        return int(self._lib.oracle_status(self._h))

    def clear_status(self) -> None:
        self._lib.oracle_clear_status(self._h)


class MultiOracle:
    """T independent oracles; arrays carry a leading T dimension."""

    def __init__(self, T: int, K: int, N: int, field_bytes=(), init_max: float = 1.0,
                 with_payload: bool = True):
        self.trees = [Oracle(K, N, field_bytes, init_max, with_payload) for _ in range(T)]
        self.T, self.K, self.N = T, K, N
        self.field_bytes = tuple(field_bytes)
        self.H = self.trees[0].H

    def insert(self, n, rows=None, prio=None, protect=None):
        return np.stack([
            o.insert(n, None if rows is None else [r[t] for r in rows],
                     None if prio is None else prio[t],
                     None if protect is None else protect[t]) for t, o in enumerate(self.trees)])

    def sample(self, u, beta=0.4, want_weights=True):
        res = [o.sample(u[t], beta, want_weights) for t, o in enumerate(self.trees)]
        idx = np.stack([r[0] for r in res])
        w = np.stack([r[1] for r in res]) if want_weights else None
        v = np.stack([r[2] for r in res])
        return idx, w, v

    def gather(self, idx):
        res = [o.gather(idx[t]) for t, o in enumerate(self.trees)]
        return [np.stack([r[f] for r in res]) for f in range(len(self.field_bytes))]

    def update(self, idx, prio):
        for t, o in enumerate(self.trees):
            o.update(idx[t], prio[t])

    def update_td(self, idx, td, eps, alpha):
        for t, o in enumerate(self.trees):
            o.update_td(idx[t], td[t], eps, alpha)

    def update_delta(self, idx, delta):
        for t, o in enumerate(self.trees):
            o.update_delta(idx[t], delta[t])

    def get_priority(self, idx):
        return np.stack([o.get_priority(idx[t]) for t, o in enumerate(self.trees)])

    def read_level(self, tree, height):
        return self.trees[tree].read_level(height)

    @property
    def total(self):
        return np.array([o.total for o in self.trees], dtype=np.float32)

    def set_weight_norm(self, mode):
        for o in self.trees:
            o.set_weight_norm(mode)

    @property
    def status(self):
        s = 0
        for o in self.trees:
            s |= o.status
        return s
