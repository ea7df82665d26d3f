"""CPU-only checks of the boundary: the library loads, exports what include/per.h declares,
and the host-side argument checks and arena layout behave (no kernel is launched here)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2311_09445_amd import per, workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "per.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(per_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = per._lib()
    names = declared_functions()
    assert {"per_create", "per_insert", "per_sample", "per_update", "per_gather"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(per.EXPORTS) == names


def test_config_struct_matches_header():
    assert C.sizeof(per.PerConfig) == 4 + 4 + 8 + 4 + 4 + 4 * 8 + 4 + 4   # with tail padding to 8


@pytest.mark.parametrize("name", list(wl.WORKLOADS))
def test_arena_size_covers_tree_and_payload(name):
    w = wl.WORKLOADS[name]
    nbytes, align = per.arena_bytes(per.make_config(w.K, w.N, w.T, w.field_bytes))
    assert align == 256 and nbytes % 256 == 0
    tree = 0
    n = w.N
    while True:
        tree += n * 4
        if n == 1:
            break
        n = -(-n // w.K)
    need = w.T * (tree + w.N * 8 + w.N * w.row_bytes)      # levels + last-writer stamps + rows
    # rows are stored with every field aligned to its access width and 16 bytes (or a multiple) apart
    padded_row = -(-(w.row_bytes + 7 * len(w.field_bytes)) // 16) * 16
    most = w.T * (tree + w.N * 8 + w.N * padded_row)
    assert need <= nbytes <= most * 1.02 + (1 << 20)


def test_bad_configurations_are_rejected_on_the_host():
    lib = per._lib()
    nbytes = C.c_size_t(0)
    good = dict(fanout=16, capacity=1000, n_trees=1, field_bytes=(4,), init_max_priority=1.0)
    for bad in [dict(fanout=0), dict(fanout=3), dict(fanout=128), dict(capacity=0), dict(capacity=(1 << 31) + 1),
                dict(n_trees=0), dict(n_trees=70000), dict(field_bytes=(0,)), dict(init_max_priority=0.0),
                dict(init_max_priority=float("inf")), dict(init_max_priority=float("nan"))]:
        cfg = per.make_config(**{**good, **bad})
        assert lib.per_arena_bytes(C.byref(cfg), C.byref(nbytes), None) == per.EINVAL, bad
    cfg = per.make_config(**good)
    cfg.struct_size = 12
    assert lib.per_arena_bytes(C.byref(cfg), C.byref(nbytes), None) == per.EINVAL
    cfg = per.make_config(**good)
    cfg.n_fields = 9
    assert lib.per_arena_bytes(C.byref(cfg), C.byref(nbytes), None) == per.EINVAL
    # per_create: null and misaligned arenas, arena too small -- all refused before any HIP call
    cfg = per.make_config(**good)
    h = C.c_void_p()
    assert lib.per_create(C.byref(cfg), None, 1 << 30, None, C.byref(h)) == per.EINVAL
    assert lib.per_create(C.byref(cfg), C.c_void_p(0x1001), 1 << 30, None, C.byref(h)) == per.EINVAL
    assert lib.per_create(C.byref(cfg), C.c_void_p(0x1000), 16, None, C.byref(h)) == per.ENOMEM
    # null handles
    assert lib.per_destroy(None) == per.EINVAL
    assert lib.per_sample(None, 1, 0.4, None, None, None, None, None) == per.EINVAL
    assert lib.per_update(None, 1, None, None, None) == per.EINVAL
    assert lib.per_insert(None, 1, None, None, None, None) == per.EINVAL
    assert lib.per_gather(None, 1, None, None, None) == per.EINVAL
    assert lib.per_update_td(None, 1, None, None, 1e-6, 0.6, None) == per.EINVAL
    assert lib.per_update_delta(None, 1, None, None, None) == per.EINVAL
    assert lib.per_run_requests(None, 1, None, None, None) == per.EINVAL
    assert lib.per_run_steps(None, 1, 0, 1, None, None) == per.EINVAL
    assert lib.per_set_weight_norm(None, 0) == per.EINVAL
    assert lib.per_min_priority(None, None, None) == per.EINVAL
    assert lib.per_note_replay(None) == per.EINVAL
    assert lib.per_set_rng(None, 1, 0) == per.EINVAL
    assert lib.per_set_ring(None, 0, 0) == per.EINVAL
    assert lib.per_set_tuning(None, b"lazy_top", 1) == per.EINVAL
    assert lib.per_run_steps_fits(None) == 0
    assert lib.per_size(None) == 0
    assert lib.per_strerror(per.ENOMEM) == b"arena too small"


def test_binding_fails_loudly_without_the_library(monkeypatch):
    monkeypatch.setattr(per, "_LIB", None)
    monkeypatch.setattr(per, "LIB_PATH", "/nonexistent/libper_hip.so")
    with pytest.raises(ImportError, match="no CPU fallback"):
        per._lib()


def test_workload_generator_is_seeded_and_exact():
    w = wl.WORKLOADS["c4_stress"]
    a = wl.step_inputs(w, 3, 0, B=1024)
    b = wl.step_inputs(w, 3, 0, B=1024)
    assert all(np.array_equal(a[k], b[k]) for k in a if k != "beta")
    assert a["u"].dtype == np.float32 and a["u"].min() >= 0 and a["u"].max() < 1
    assert np.all(a["u"] * 2 ** 24 == np.floor(a["u"] * 2 ** 24))
    assert len(a["dup_dst"][0]) == 102 and len(np.unique(a["dup_dst"][0])) == 102
    v = wl.initial_priorities(w, 0, n=100000)
    assert 0.005 < (v == 0).mean() < 0.015 and v[v > 0].min() >= 1.0
    w2 = wl.WORKLOADS["c2_dqn"]
    assert w2.beta(0) == 0.4 and abs(w2.beta(w2.steps - 1) - 1.0) < 1e-12
    r1 = wl.row_bytes(2, [5, 6], 1, 24)
    assert r1.shape == (2, 24) and not np.array_equal(r1[0], r1[1])
    assert np.array_equal(wl.row_bytes(2, [6], 1, 24)[0], r1[1])
    assert np.array_equal(wl.row_bytes(2, [6], 1, 21)[0], r1[1][:21])


def test_row_hash_matches_between_numpy_and_torch():
    import torch
    c = np.array([0, 1, 7, 2 ** 24 + 3, 2 ** 31 + 9], dtype=np.int64)
    for f, b in enumerate((68, 24, 4, 1, 128)):
        a = wl.row_bytes(3, c, f, b)
        t = wl.row_bytes_torch(3, torch.from_numpy(c), f, b).numpy()
        assert np.array_equal(a, t)


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in (r.stdout + r.stderr)
