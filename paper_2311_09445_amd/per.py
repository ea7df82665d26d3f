"""Thin ctypes binding of ``libper_hip.so`` (the C-ABI declared in ``include/per.h``).

Argument marshalling only: every step runs in the library's HIP kernels.  PyTorch
supplies device memory (the arena and the I/O arrays are torch tensors) and the
stream.  There is no CPU fallback: if the library has not been built, loading
fails with an error that says how to build it.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libper_hip.so")
MAX_FIELDS = 8

OK, EINVAL, ENOMEM, EEMPTY, ERANGE, EHIP = 0, -1, -2, -3, -4, -5
FLAG_BAD_INDEX, FLAG_BAD_PRIORITY, FLAG_ZERO_TOTAL = 1, 2, 4

EXPORTS = [
    "per_arena_bytes", "per_create", "per_destroy", "per_insert", "per_insert_protected", "per_sample", "per_sample_gather",
    "per_sample_gather_update", "per_step", "per_insert_step", "per_gather",
    "per_update", "per_update_td", "per_update_delta", "per_rebuild", "per_set_rng", "per_rng_calls", "per_run_steps",
    "per_run_steps_fits", "per_run_requests", "per_set_weight_norm", "per_min_priority", "per_min_priority_static", "per_note_replay", "per_get_priority", "per_read_level", "per_total", "per_max_priority",
    "per_status", "per_clear_status", "per_height", "per_size", "per_cursor", "per_set_ring", "per_set_tuning",
    "per_profile", "per_profile_read", "per_strerror",
]


class PerConfig(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32),
        ("fanout", C.c_uint32),
        ("capacity", C.c_uint64),
        ("n_trees", C.c_uint32),
        ("n_fields", C.c_uint32),
        ("field_bytes", C.c_uint32 * MAX_FIELDS),
        ("init_max_priority", C.c_float),
    ]


class PerStreamIO(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32),
        ("d_ins_rows", C.c_void_p),
        ("d_ins_prio", C.c_void_p),
        ("d_u", C.c_void_p),
        ("d_beta", C.c_void_p),
        ("d_out_idx", C.c_void_p),
        ("d_out_weight", C.c_void_p),
        ("d_out_prio", C.c_void_p),
        ("d_rows_out", C.c_void_p),
        ("d_upd_idx", C.c_void_p),
        ("d_upd_prio", C.c_void_p),
    ]


OP_INSERT, OP_SAMPLE, OP_UPDATE = 1, 2, 3


class PerRequest(C.Structure):
    _fields_ = [
        ("op", C.c_uint32),
        ("n", C.c_uint32),
        ("beta", C.c_float),
        ("n_protect", C.c_uint32),
        ("prio", C.c_void_p),
        ("u", C.c_void_p),
        ("idx", C.c_void_p),
        ("out_weight", C.c_void_p),
        ("out_prio", C.c_void_p),
        ("protect", C.c_void_p),
        ("field", C.c_void_p * MAX_FIELDS),
    ]


class PerError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {code} ({_lib().per_strerror(code).decode()})")


_LIB = None


def _lib():
    global _LIB
    if _LIB is not None:
        return _LIB
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2311_09445_amd.build` "
            "(hipcc, gfx950). There is no CPU fallback.")
    lib = C.CDLL(LIB_PATH)
    vp, u32, u64, i64, f32 = C.c_void_p, C.c_uint32, C.c_uint64, C.c_int64, C.c_float
    cfgp = C.POINTER(PerConfig)
    sig = {
        "per_arena_bytes": (C.c_int, [cfgp, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]),
        "per_create": (C.c_int, [cfgp, vp, C.c_size_t, vp, C.POINTER(vp)]),
        "per_destroy": (C.c_int, [vp]),
        "per_insert": (C.c_int, [vp, u32, vp, vp, vp, vp]),
        "per_insert_protected": (C.c_int, [vp, u32, vp, vp, vp, u32, vp, vp]),
        "per_sample": (C.c_int, [vp, u32, f32, vp, vp, vp, vp, vp]),
        "per_sample_gather": (C.c_int, [vp, u32, f32, vp, vp, vp, vp, vp, vp]),
        "per_sample_gather_update": (C.c_int, [vp, u32, f32, vp, vp, vp, vp, vp, u32, vp, vp, vp]),
        "per_step": (C.c_int, [vp, u32, f32, vp, vp, vp, vp, vp, vp, vp, vp]),
        "per_insert_step": (C.c_int, [vp, u32, vp, vp, vp, u32, f32, vp, vp, vp, vp, vp, vp, vp, vp]),
        "per_gather": (C.c_int, [vp, u32, vp, vp, vp]),
        "per_update": (C.c_int, [vp, u32, vp, vp, vp]),
        "per_update_delta": (C.c_int, [vp, u32, vp, vp, vp]),
        "per_rebuild": (C.c_int, [vp, vp]),
        "per_set_rng": (C.c_int, [vp, C.c_uint64, C.c_uint64]),
        "per_rng_calls": (C.c_uint64, [vp]),
        "per_run_steps": (C.c_int, [vp, u32, u32, u32, C.POINTER(PerStreamIO), vp]),
        "per_run_steps_fits": (C.c_int, [vp]),
        "per_run_requests": (C.c_int, [vp, u32, vp, vp, vp]),
        "per_set_weight_norm": (C.c_int, [vp, C.c_int]),
        "per_note_replay": (C.c_int, [vp]),
        "per_min_priority": (C.c_int, [vp, vp, vp]),
        "per_min_priority_static": (C.c_int, [vp, vp, vp]),
        "per_update_td": (C.c_int, [vp, u32, vp, vp, C.c_double, C.c_double, vp]),
        "per_get_priority": (C.c_int, [vp, u32, vp, vp, vp]),
        "per_read_level": (C.c_int, [vp, u32, u32, vp, C.POINTER(u64), vp]),
        "per_total": (C.c_int, [vp, vp, vp]),
        "per_max_priority": (C.c_int, [vp, vp, vp]),
        "per_status": (C.c_int, [vp, vp, C.POINTER(u32)]),
        "per_clear_status": (C.c_int, [vp, vp]),
        "per_height": (u32, [vp]),
        "per_size": (u64, [vp]),
        "per_cursor": (u64, [vp]),
        "per_set_ring": (C.c_int, [vp, u64, u64]),
        "per_set_tuning": (C.c_int, [vp, C.c_char_p, i64]),
        "per_profile": (C.c_int, [vp, C.c_int]),
        "per_profile_read": (C.c_int, [vp, u32, C.POINTER(C.c_char_p), C.POINTER(C.c_double),
                                       C.POINTER(u64), C.POINTER(u32)]),
        "per_strerror": (C.c_char_p, [C.c_int]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _LIB = lib
    return lib


def make_config(fanout: int, capacity: int, n_trees: int = 1, field_bytes: Sequence[int] = (),
                init_max_priority: float = 1.0) -> PerConfig:
    cfg = PerConfig()
    cfg.struct_size = C.sizeof(PerConfig)
    cfg.fanout = fanout
    cfg.capacity = capacity
    cfg.n_trees = n_trees
    cfg.n_fields = len(field_bytes)
    for i, b in enumerate(field_bytes[:MAX_FIELDS]):
        cfg.field_bytes[i] = b
    cfg.init_max_priority = init_max_priority
    return cfg


def arena_bytes(cfg: PerConfig):
    nbytes, align = C.c_size_t(0), C.c_size_t(0)
    rc = _lib().per_arena_bytes(C.byref(cfg), C.byref(nbytes), C.byref(align))
    if rc != OK:
        raise PerError(rc, "per_arena_bytes")
    return nbytes.value, align.value


def _dptr(t, dtype=None):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected dtype {dtype}, got {t.dtype}")
    return C.c_void_p(t.data_ptr())


class PrioritizedReplay:
    """T prioritized replay buffers of capacity N with fanout K on the current device.

    Mirrors the paper's library interface ``PER(size=..., fanout=...)`` (Listing 2).
    All array arguments are contiguous device tensors shaped [T, ...] (a leading
    dimension of size T may be omitted when T == 1).
    """

    def __init__(self, fanout: int, capacity: int, n_trees: int = 1, field_bytes: Sequence[int] = (),
                 init_max_priority: float = 1.0, device="cuda"):
        import torch
        self._torch = torch
        self.lib = _lib()
        self.K, self.N, self.T = int(fanout), int(capacity), int(n_trees)
        self.field_bytes = tuple(int(b) for b in field_bytes)
        if len(self.field_bytes) > MAX_FIELDS:
            raise PerError(EINVAL, "per_create")
        self.cfg = make_config(self.K, self.N, self.T, self.field_bytes, init_max_priority)
        nbytes, _ = arena_bytes(self.cfg)
        self.device = torch.device(device)
        self.arena = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        h = C.c_void_p()
        rc = self.lib.per_create(C.byref(self.cfg), C.c_void_p(self.arena.data_ptr()), nbytes,
                                 self._stream(), C.byref(h))
        if rc != OK:
            raise PerError(rc, "per_create")
        self._h = h
        self.H = self.lib.per_height(self._h)

    def __del__(self):
        h = getattr(self, "_h", None)
        if h:
            self.lib.per_destroy(h)
            self._h = None

    def _stream(self):
        return C.c_void_p(self._torch.cuda.current_stream(self.device).cuda_stream)

    def _check(self, rc, what):
        if rc != OK:
            raise PerError(rc, what)

    def _ptr_array(self, tensors, n_rows):
        if tensors is None:
            return None, None
        if len(tensors) != len(self.field_bytes):
            raise ValueError("one tensor (or None) per payload field is required")
        arr = (C.c_void_p * max(1, len(tensors)))()
        for f, t in enumerate(tensors):
            if t is None:
                arr[f] = None
                continue
            if t.numel() * t.element_size() != self.T * n_rows * self.field_bytes[f]:
                raise ValueError(f"field {f}: expected {self.T}x{n_rows}x{self.field_bytes[f]} bytes")
            arr[f] = _dptr(t).value
        return arr, C.cast(arr, C.c_void_p)

    # ---------------------------------------------------------------- operations
    def insert(self, n: int, rows=None, prio=None, out_idx=None, protect=None):
        """``protect`` ([T, m] indices): rows whose ring slot is among them are deferred (per_insert_protected)."""
        torch = self._torch
        _keep, src = self._ptr_array(rows, n)
        if prio is not None and prio.numel() != self.T * n:
            raise ValueError("prio must hold T*n values")
        if out_idx is not None and out_idx.numel() != self.T * n:
            raise ValueError("out_idx must hold T*n values")
        if protect is not None:
            rc = self.lib.per_insert_protected(self._h, n, src, _dptr(prio, torch.float32), _dptr(out_idx, torch.int32),
                                               protect.numel() // self.T, _dptr(protect, torch.int32), self._stream())
        else:
            rc = self.lib.per_insert(self._h, n, src, _dptr(prio, torch.float32), _dptr(out_idx, torch.int32),
                                     self._stream())
        self._check(rc, "per_insert")

    def sample(self, u, beta: float = 0.4, want_weights: bool = True, want_prio: bool = True,
               out_idx=None, out_weight=None, out_prio=None, rows_out=None, update=None, B=None):
        """Returns (idx int32 [T,B] holding uint32 bit patterns, weights or None, prio or None).

        ``u=None`` with ``B`` given: the call draws its own uniforms (after ``set_rng``).

        With ``rows_out`` (one [T,B,bytes] uint8 tensor or None per field) the sampled rows are
        gathered by the same call (per_sample_gather).  With ``update=(idx, prio)`` that priority
        update is applied after the sampling, still in the same call (per_sample_gather_update)."""
        torch = self._torch
        if u is None:
            if B is None:
                raise ValueError("without uniforms the batch size B must be given")
        else:
            B = u.numel() // self.T
            if u.numel() != B * self.T:
                raise ValueError("u must hold T*B values")
        shape = (self.T, B)
        if out_idx is None:
            out_idx = torch.empty(shape, dtype=torch.int32, device=self.device)
        if want_weights and out_weight is None:
            out_weight = torch.empty(shape, dtype=torch.float32, device=self.device)
        if want_prio and out_prio is None:
            out_prio = torch.empty(shape, dtype=torch.float32, device=self.device)
        args = (self._h, B, float(beta), _dptr(u, torch.float32), _dptr(out_idx, torch.int32),
                _dptr(out_weight, torch.float32) if want_weights else None,
                _dptr(out_prio, torch.float32) if want_prio else None)
        dst = None
        if rows_out is not None:
            _keep, dst = self._ptr_array(rows_out, B)
        if update is not None:
            uidx, uprio = update
            if uprio.numel() != uidx.numel():
                raise ValueError("update idx and prio must have the same number of elements")
            rc = self.lib.per_sample_gather_update(*args, dst, uidx.numel() // self.T, _dptr(uidx, torch.int32),
                                                   _dptr(uprio, torch.float32), self._stream())
        elif rows_out is None:
            rc = self.lib.per_sample(*args, self._stream())
        else:
            rc = self.lib.per_sample_gather(*args, dst, self._stream())
        self._check(rc, "per_sample")
        return out_idx, (out_weight if want_weights else None), (out_prio if want_prio else None)

    def step(self, u, beta, upd_prio, upd_pos=None, want_weights: bool = True, want_prio: bool = True,
             out_idx=None, out_weight=None, out_prio=None, rows_out=None, B=None, insert=None):
        """per_step: sample, gather and update the batch just drawn; element j of ``upd_prio`` goes to the leaf
        drawn by sample ``upd_pos[j]`` (``None``: sample j).  Returns (idx, weights or None, prio or None).

        ``insert=(n, rows, prio, out_idx)`` (as for ``insert``; the last three may be None): per_insert_step, the
        insertion of n rows per tree followed by the step, as one call."""
        torch = self._torch
        if u is None:
            if B is None:
                raise ValueError("without uniforms the batch size B must be given")
        else:
            B = u.numel() // self.T
        shape = (self.T, B)
        if upd_prio.numel() != self.T * B or (upd_pos is not None and upd_pos.numel() != self.T * B):
            raise ValueError("upd_prio and upd_pos must hold T*B values")
        if out_idx is None:
            out_idx = torch.empty(shape, dtype=torch.int32, device=self.device)
        if want_weights and out_weight is None:
            out_weight = torch.empty(shape, dtype=torch.float32, device=self.device)
        if want_prio and out_prio is None:
            out_prio = torch.empty(shape, dtype=torch.float32, device=self.device)
        dst = None
        if rows_out is not None:
            _keep, dst = self._ptr_array(rows_out, B)
        if insert is not None:
            n, ins_rows, ins_prio, ins_out = insert
            _keep_src, src = self._ptr_array(ins_rows, n)
            if ins_prio is not None and ins_prio.numel() != self.T * n:
                raise ValueError("the insertion's prio must hold T*n values")
            if ins_out is not None and ins_out.numel() != self.T * n:
                raise ValueError("the insertion's out_idx must hold T*n values")
            rc = self.lib.per_insert_step(self._h, n, src, _dptr(ins_prio, torch.float32), _dptr(ins_out, torch.int32),
                                          B, float(beta), _dptr(u, torch.float32), _dptr(out_idx, torch.int32),
                                          _dptr(out_weight, torch.float32) if want_weights else None,
                                          _dptr(out_prio, torch.float32) if want_prio else None, dst,
                                          _dptr(upd_prio, torch.float32), _dptr(upd_pos, torch.int32), self._stream())
            self._check(rc, "per_insert_step")
            return out_idx, (out_weight if want_weights else None), (out_prio if want_prio else None)
        rc = self.lib.per_step(self._h, B, float(beta), _dptr(u, torch.float32), _dptr(out_idx, torch.int32),
                               _dptr(out_weight, torch.float32) if want_weights else None,
                               _dptr(out_prio, torch.float32) if want_prio else None, dst,
                               _dptr(upd_prio, torch.float32), _dptr(upd_pos, torch.int32), self._stream())
        self._check(rc, "per_step")
        return out_idx, (out_weight if want_weights else None), (out_prio if want_prio else None)

    def run_steps_fits(self) -> bool:
        return bool(self.lib.per_run_steps_fits(self._h))

    def run_steps(self, u, beta, out_idx, out_weight=None, out_prio=None, rows_out=None, upd_prio=None, upd_idx=None,
                  n_insert: int = 0, ins_rows=None, ins_prio=None):
        """A list of steps (insert -> sample -> gather -> update) in one launch on an LDS copy of the tree.
        ``u``: [steps, T, B]; ``beta``: [steps] device tensor; the other arrays as in per.h (leading step
        dimension).  ``upd_prio`` without ``upd_idx`` updates, in every step, the batch just sampled."""
        torch = self._torch
        steps, B = int(u.shape[0]), int(u.shape[-1])
        if u.numel() != steps * self.T * B or beta.numel() != steps:
            raise ValueError("u must be [steps, T, B] and beta [steps]")
        for name, x in (("out_idx", out_idx), ("out_weight", out_weight), ("out_prio", out_prio),
                        ("upd_prio", upd_prio), ("upd_idx", upd_idx)):
            if x is not None and x.numel() != u.numel():
                raise ValueError(f"{name} must hold steps*T*B values")
        if ins_prio is not None and ins_prio.numel() != steps * self.T * n_insert:
            raise ValueError("ins_prio must hold steps*T*n_insert values")
        io = PerStreamIO()
        io.struct_size = C.sizeof(PerStreamIO)
        keep = []

        def table(tensors, rows_per_tree):
            if tensors is None:
                return None
            if len(tensors) != len(self.field_bytes):
                raise ValueError("one tensor (or None) per payload field is required")
            arr = (C.c_void_p * max(1, len(tensors)))()
            for f, t in enumerate(tensors):
                if t is None:
                    arr[f] = None
                    continue
                if t.numel() * t.element_size() != steps * self.T * rows_per_tree * self.field_bytes[f]:
                    raise ValueError(f"field {f}: expected steps*T*rows*{self.field_bytes[f]} bytes")
                arr[f] = _dptr(t).value
            keep.append(arr)
            return C.cast(arr, C.c_void_p)

        def ptr(x, dtype):
            p = _dptr(x, dtype)
            return None if p is None else p.value

        io.d_ins_rows = table(ins_rows, n_insert)
        io.d_ins_prio = ptr(ins_prio, torch.float32)
        io.d_u = ptr(u, torch.float32)
        io.d_beta = ptr(beta, torch.float32)
        io.d_out_idx = ptr(out_idx, torch.int32)
        io.d_out_weight = ptr(out_weight, torch.float32)
        io.d_out_prio = ptr(out_prio, torch.float32)
        io.d_rows_out = table(rows_out, B)
        io.d_upd_idx = ptr(upd_idx, torch.int32)
        io.d_upd_prio = ptr(upd_prio, torch.float32)
        rc = self.lib.per_run_steps(self._h, steps, int(n_insert), B, C.byref(io), self._stream())
        self._check(rc, "per_run_steps")

    def prepare_requests(self, requests):
        """Encodes a list of requests for run_requests: a host array of per_request and its device copy.
        ``requests``: a list of dicts, each with ``op`` (OP_INSERT / OP_SAMPLE / OP_UPDATE) and device tensors
        under the names of per.h's per_request (``prio``, ``u``, ``idx``, ``out_weight``, ``out_prio``,
        ``protect``, ``beta``, ``rows``: one tensor or None per payload field).  The batch of a request is
        taken from ``u`` (SAMPLE), ``prio`` (UPDATE), or ``n`` (INSERT)."""
        torch = self._torch
        arr = (PerRequest * max(1, len(requests)))()
        for r, q in enumerate(requests):
            op = int(q["op"])
            if op == OP_SAMPLE:
                n = q["u"].numel() // self.T
            elif op == OP_UPDATE:
                n = q["prio"].numel() // self.T
            else:
                n = int(q["n"])
            a = arr[r]
            a.op, a.n, a.beta = op, n, float(q.get("beta", 0.0))
            for name, dtype in (("prio", torch.float32), ("u", torch.float32), ("idx", torch.int32),
                                ("out_weight", torch.float32), ("out_prio", torch.float32), ("protect", torch.int32)):
                x = q.get(name)
                if x is not None and name != "protect" and x.numel() != self.T * n:
                    raise ValueError(f"request {r}: {name} must hold T*n values")
                ptr = _dptr(x, dtype)
                setattr(a, name, None if ptr is None else ptr.value)
            if q.get("protect") is not None:
                a.n_protect = q["protect"].numel() // self.T
            rows = q.get("rows")
            if rows is not None:
                if len(rows) != len(self.field_bytes):
                    raise ValueError("one tensor (or None) per payload field is required")
                for f, x in enumerate(rows):
                    if x is None:
                        continue
                    if x.numel() * x.element_size() != self.T * n * self.field_bytes[f]:
                        raise ValueError(f"request {r}, field {f}: expected T*n*{self.field_bytes[f]} bytes")
                    a.field[f] = _dptr(x).value
        nbytes = C.sizeof(PerRequest) * len(requests)
        host = torch.frombuffer(bytearray(bytes(arr)[:max(nbytes, 1)]), dtype=torch.uint8)
        return len(requests), arr, host.to(self.device)

    def run_requests(self, requests):
        """A queue of op-coded requests in one launch on an LDS copy of the tree.  ``requests``: what
        prepare_requests returned, or a list of request dicts (encoded here).  Returns the encoded queue,
        which must stay alive until the stream's work is done."""
        prepared = requests if isinstance(requests, tuple) else self.prepare_requests(requests)
        n, arr, d_queue = prepared
        rc = self.lib.per_run_requests(self._h, n, C.cast(arr, C.c_void_p), C.c_void_p(d_queue.data_ptr()), self._stream())
        self._check(rc, "per_run_requests")
        return prepared

    def note_replay(self):
        """Call after replaying a captured graph of calls on this buffer, before the next call outside it."""
        self._check(self.lib.per_note_replay(self._h), "per_note_replay")

    def set_weight_norm(self, mode: str):
        """'batch' (default): importance weights relative to the largest weight of the sampled batch;
        'buffer': relative to the largest weight any stored row could get."""
        self._check(self.lib.per_set_weight_norm(self._h, {"batch": 0, "buffer": 1}[mode]), "per_set_weight_norm")

    def min_priority(self):
        """Smallest positive leaf of every tree (+inf where there is none)."""
        out = self._torch.empty(self.T, dtype=self._torch.float32, device=self.device)
        self._check(self.lib.per_min_priority(self._h, _dptr(out), self._stream()), "per_min_priority")
        return out

    def min_priority_static(self, out=None):
        """per_min_priority with the reduction's scratch in the library's static device array (no allocation when
        ``out`` is given)."""
        if out is None:
            out = self._torch.empty(self.T, dtype=self._torch.float32, device=self.device)
        self._check(self.lib.per_min_priority_static(self._h, _dptr(out), self._stream()), "per_min_priority_static")
        return out

    def set_rng(self, seed: int, next_call: int = 0):
        """Sampling calls without uniforms draw them from a counter-based generator keyed by ``seed``."""
        self._check(self.lib.per_set_rng(self._h, int(seed), int(next_call)), "per_set_rng")

    def rng_calls(self) -> int:
        return int(self.lib.per_rng_calls(self._h))

    def gather(self, idx, out=None):
        torch = self._torch
        B = idx.numel() // self.T
        if out is None:
            out = [torch.empty((self.T, B, b), dtype=torch.uint8, device=self.device) for b in self.field_bytes]
        _keep, dst = self._ptr_array(out, B)
        rc = self.lib.per_gather(self._h, B, _dptr(idx, torch.int32), dst, self._stream())
        self._check(rc, "per_gather")
        return out

    def update(self, idx, prio):
        torch = self._torch
        B = idx.numel() // self.T
        if prio.numel() != idx.numel():
            raise ValueError("idx and prio must have the same number of elements")
        rc = self.lib.per_update(self._h, B, _dptr(idx, torch.int32), _dptr(prio, torch.float32), self._stream())
        self._check(rc, "per_update")

    def update_td(self, idx, td, eps: float = 1e-6, alpha: float = 0.6):
        """per_update with the priorities computed on the device from temporal-difference errors."""
        torch = self._torch
        B = idx.numel() // self.T
        if td.numel() != idx.numel():
            raise ValueError("idx and td must have the same number of elements")
        rc = self.lib.per_update_td(self._h, B, _dptr(idx, torch.int32), _dptr(td, torch.float32), float(eps),
                                    float(alpha), self._stream())
        self._check(rc, "per_update_td")

    def update_delta(self, idx, delta):
        """The paper's form of the update: add delta[j] to leaf idx[j] and to all its ancestors."""
        torch = self._torch
        B = idx.numel() // self.T
        if delta.numel() != idx.numel():
            raise ValueError("idx and delta must have the same number of elements")
        rc = self.lib.per_update_delta(self._h, B, _dptr(idx, torch.int32), _dptr(delta, torch.float32), self._stream())
        self._check(rc, "per_update_delta")

    def rebuild(self):
        """Recomputes every node above the leaves from its children (full bottom-up rebuild)."""
        self._check(self.lib.per_rebuild(self._h, self._stream()), "per_rebuild")

    def get_priority(self, idx, out=None):
        torch = self._torch
        n = idx.numel() // self.T
        if out is None:
            out = torch.empty((self.T, n), dtype=torch.float32, device=self.device)
        rc = self.lib.per_get_priority(self._h, n, _dptr(idx, torch.int32), _dptr(out, torch.float32),
                                       self._stream())
        self._check(rc, "per_get_priority")
        return out

    # ---------------------------------------------------------------- inspection
    def level_count(self, height: int) -> int:
        cnt = C.c_uint64(0)
        self._check(self.lib.per_read_level(self._h, 0, height, None, C.byref(cnt), self._stream()),
                    "per_read_level")
        return cnt.value

    def read_level(self, tree: int, height: int):
        torch = self._torch
        out = torch.empty(self.level_count(height), dtype=torch.float32, device=self.device)
        cnt = C.c_uint64(0)
        self._check(self.lib.per_read_level(self._h, tree, height, _dptr(out), C.byref(cnt), self._stream()),
                    "per_read_level")
        return out

    def total(self):
        out = self._torch.empty(self.T, dtype=self._torch.float32, device=self.device)
        self._check(self.lib.per_total(self._h, _dptr(out), self._stream()), "per_total")
        return out

    def max_priority(self):
        out = self._torch.empty(self.T, dtype=self._torch.float32, device=self.device)
        self._check(self.lib.per_max_priority(self._h, _dptr(out), self._stream()), "per_max_priority")
        return out

    def status(self) -> int:
        flags = C.c_uint32(0)
        self._check(self.lib.per_status(self._h, self._stream(), C.byref(flags)), "per_status")
        return flags.value

    def clear_status(self):
        self._check(self.lib.per_clear_status(self._h, self._stream()), "per_clear_status")

    @property
    def size(self) -> int:
        return int(self.lib.per_size(self._h))

    @property
    def cursor(self) -> int:
        return int(self.lib.per_cursor(self._h))

    def set_ring(self, cursor: int, size: int):
        """Host mirrors of a restored arena (checkpoint / resume)."""
        self._check(self.lib.per_set_ring(self._h, int(cursor), int(size)), "per_set_ring")

    def set_tuning(self, name: str, value: int):
        self._check(self.lib.per_set_tuning(self._h, name.encode(), int(value)), "per_set_tuning")

    def profile(self, enable: bool):
        self._check(self.lib.per_profile(self._h, 1 if enable else 0), "per_profile")

    def profile_read(self):
        """{kernel name: (total ms, launches)} since profiling was last enabled."""
        cap = 32
        names = (C.c_char_p * cap)()
        ms = (C.c_double * cap)()
        cnt = (C.c_uint64 * cap)()
        n = C.c_uint32(0)
        self._check(self.lib.per_profile_read(self._h, cap, names, ms, cnt, C.byref(n)), "per_profile_read")
        return {names[i].decode(): (ms[i], cnt[i]) for i in range(min(n.value, cap))}
