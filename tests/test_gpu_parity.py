"""Parity of the HIP path (through the C-ABI) with the CPU oracle, element by element."""
import os

import gc
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():   # collected everywhere, run only where a GPU is present
    pytest.skip("needs a GPU", allow_module_level=True)

from scipy import stats  # noqa: E402

from paper_2311_09445_amd import workloads as wl  # noqa: E402
from paper_2311_09445_amd.per import (EEMPTY, EINVAL, ERANGE, FLAG_BAD_INDEX, FLAG_BAD_PRIORITY,  # noqa: E402
                                      FLAG_ZERO_TOTAL, PerError, PrioritizedReplay)
from oracle.per_oracle import MultiOracle  # noqa: E402
from tests.harness import Mirror, dev, idx_to_dev, idx_to_host  # noqa: E402

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
FIELDS = (16, 4, 4, 16, 1)


def log(msg):
    print(msg, flush=True)


@pytest.fixture(autouse=True, params=["group", "leaf", "owner"])
def claim_form(request, monkeypatch):
    """Every test runs three times: update batches claim their leaves through the group entries (the default),
    leaf by leaf, or (third run) steps that update the batch they sample run as the one-kernel step wherever the
    tree fits it, not only where it pays off."""
    if request.param != "group":
        created = PrioritizedReplay.__init__
        name, value = ("group_claim", 0) if request.param == "leaf" else ("step_kernel", 2)

        def create_then_set(self, *a, **kw):
            created(self, *a, **kw)
            self.set_tuning(name, value)

        monkeypatch.setattr(PrioritizedReplay, "__init__", create_then_set)
    return request.param


# ------------------------------------------------------------------ small, every fanout
@pytest.mark.parametrize("K", [2, 4, 8, 16, 32, 64])
@pytest.mark.parametrize("N,T", [(1, 1), (5, 2), (1000, 1), (4097, 3), (70000, 1)])
def test_random_operation_mix(K, N, T):
    """Several tiles and a ragged tail: inserts (explicit and max priority, with wrap), samples with
    batch sizes that are not powers of two, gathers, updates with duplicates and invalid elements."""
    log(f"mix K={K} N={N} T={T}")
    rng = np.random.default_rng(K * 1000003 + N * 7 + T)
    m = Mirror(K, N, T, FIELDS)
    first = max(1, (2 * N) // 3)
    m.insert(first, prio=wl._draw_priorities("lognormal_0_1", rng, (T, first)))
    m.compare_tree()
    for it in range(4):
        B = int(rng.choice([1, 3, 64, 257, 1500]))
        u = wl.uniform01(rng, (T, B))
        gi, ci = m.sample(u, beta=float(rng.choice([0.0, 0.4, 1.0])), fused_rows=(it % 2 == 0))
        m.gather(gi, ci)
        upd_idx = ci.copy()
        upd_prio = wl._draw_updates("absnormal1_eps_pow0.6", rng, (T, B))
        if B > 4:   # duplicates, an out-of-range index and invalid values
            upd_idx[:, B // 2:] = upd_idx[:, : B - B // 2]
            upd_idx[:, 0] = m.N + 5
            upd_prio[:, 1] = np.nan
            upd_prio[:, 2] = -1.0
            upd_prio[:, 3] = np.inf
        m.update(upd_idx, upd_prio)
        m.compare_tree()
        n_ins = int(rng.integers(1, max(2, N // 2)))
        m.insert(n_ins, prio=None if it % 2 == 0 else wl._draw_priorities("exponential_1", rng, (T, n_ins)))
        m.compare_tree()
    m.compare_status()


def test_golden_worked_example_on_gpu():
    g = {}
    with open(os.path.join(GOLDEN, "eq1_worked_example.txt")) as f:
        for line in f:
            if not line.startswith("#") and line.strip():
                k, *v = line.split()
                g[k] = [float(x) for x in v]
    for K in (2, 4, 8):
        p = PrioritizedReplay(K, 8)
        p.insert(8, None, dev(np.array([g["leaves"]], np.float32)))
        idx, w, v = p.sample(dev(np.array([g["u"]], np.float32)), beta=g["beta"][0])
        assert idx_to_host(idx)[0].tolist() == [int(x) for x in g["idx"]]
        assert v.cpu().numpy()[0].tolist() == g["prio"]
        np.testing.assert_allclose(w.cpu().numpy()[0], g["weight"], rtol=1e-6)
        h = 1
        while f"k{K}_h{h}" in g:
            assert p.read_level(0, h).cpu().numpy().tolist() == g[f"k{K}_h{h}"]
            h += 1


# ------------------------------------------------------------------ last writer
@pytest.mark.parametrize("K", [2, 16, 32])
def test_last_writer_adversarial(K):
    log(f"last writer K={K}")
    rng = np.random.default_rng(K)
    N, T = 5000, 2
    m = Mirror(K, N, T, ())
    m.insert(N, prio=np.ones((T, N), np.float32), with_rows=False)
    B = 3000                                            # spans many workgroups
    cases = [
        np.full((T, B), 77, np.uint32),                 # every element hits one leaf
        np.tile(np.array([3, 4000], np.uint32), (T, B // 2)),      # two leaves alternating
        np.repeat(np.arange(B // 250, dtype=np.uint32), 250)[None].repeat(T, 0),  # runs straddling blocks
        rng.integers(0, 64, (T, B)).astype(np.uint32),  # heavy random duplication
        rng.integers(0, N, (T, B)).astype(np.uint32),
    ]
    for idx in cases:
        m.update(idx, rng.random((T, B)).astype(np.float32))
        m.compare_tree()
    m.compare_status()


def test_group_stamp_counter_turns_over():
    """The stamps of the group entries come from a counter in device memory; the tree pass of the batch that
    takes it past 2^25 clears all entries and starts it over.  Entries of earlier batches must never count."""
    rng = np.random.default_rng(11)
    N, T, B = 20000, 2, 3000
    for K in (4, 32, 64):
        m = Mirror(K, N, T, ())
        m.insert(N, prio=rng.random((T, N)).astype(np.float32), with_rows=False)
        m.update(rng.integers(0, N, (T, B)).astype(np.uint32), rng.random((T, B)).astype(np.float32))
        torch.cuda.synchronize()
        m.gpu.set_tuning("group_stamp_next", (1 << 25) - 2 * B - 5)
        torch.cuda.synchronize()
        for it in range(5):        # the second call ends beyond the turning point
            idx = rng.integers(0, 200 if it % 2 else N, (T, B)).astype(np.uint32)
            m.update(idx, rng.random((T, B)).astype(np.float32))
            m.compare_tree()
        m.compare_status()


def test_update_batch_too_long_for_the_group_entries(claim_form):
    """A batch of 2^26 + 3 elements cannot use the group entries (at most 2^25 elements): it claims leaf by
    leaf, between batches that use the entries."""
    if claim_form != "group":
        pytest.skip("the same path as the other form")
    rng = np.random.default_rng(26)
    K, N, T = 16, 1 << 16, 1
    B = (1 << 26) + 3
    m = Mirror(K, N, T, ())
    m.insert(N, prio=rng.random((T, N)).astype(np.float32), with_rows=False)
    m.update(rng.integers(0, N, (T, 5000)).astype(np.uint32), rng.random((T, 5000)).astype(np.float32))   # leaves entries behind
    idx = rng.integers(0, N, (T, B), dtype=np.uint32)
    prio = rng.random((T, B), dtype=np.float32)      # all below the initial running maximum of 1, which so stays put
    log("long batch: device")
    m.gpu.update(idx_to_dev(idx), dev(prio))
    # expected leaves: the last writer of every index (the oracle's loop over 2^26 elements takes too long here)
    last = np.full(N, -1, dtype=np.int64)
    last[idx[0]] = np.arange(B)                 # later assignments win
    leaves = m.cpu.read_level(0, 0).copy()
    hit = last >= 0
    leaves[hit] = prio[0, last[hit]]
    log("long batch: oracle")
    m.cpu.update(np.nonzero(hit)[0].astype(np.uint32)[None], leaves[hit][None])     # one element per written leaf
    del idx, prio
    m.compare_tree()
    for it in range(2):
        m.update(rng.integers(0, 300, (T, 4000)).astype(np.uint32), rng.random((T, 4000)).astype(np.float32))
        m.compare_tree()
    m.compare_status()


@pytest.mark.parametrize("K", [2, 16, 32, 64])
def test_claim_forms_alternate_on_one_buffer(K):
    """Batches that claim leaf by leaf and batches that claim through group entries follow one another on
    the same few groups: what one form leaves behind must not count for the other."""
    log(f"alternating claim forms K={K}")
    rng = np.random.default_rng(K + 100)
    N, T, B = 3000, 2, 700
    m = Mirror(K, N, T, ())
    m.insert(N, prio=np.ones((T, N), np.float32), with_rows=False)
    for it in range(12):
        m.gpu.set_tuning("group_claim", 1 if it % 3 else 0)
        hi = [N, 70, 33, 130][it % 4]
        idx = rng.integers(0, hi, (T, B)).astype(np.uint32)
        if it % 5 == 4:
            idx[:, ::2] = idx[:, 0:1]          # half the batch on one leaf
        m.update(idx, rng.random((T, B)).astype(np.float32))
        m.compare_tree()
    m.compare_status()


def test_resume_in_a_fresh_buffer():
    """A byte copy of the arena plus (cursor, size) is the whole state: copied into a buffer created
    afterwards (whose stamp counter starts over) the next updates must still find the last writers."""
    rng = np.random.default_rng(21)
    K, N, T, B = 16, 6000, 2, 900
    m = Mirror(K, N, T, FIELDS)
    m.insert(5000, prio=rng.random((T, 5000)).astype(np.float32))
    for it in range(3):
        m.update(rng.integers(0, 300, (T, B)).astype(np.uint32), rng.random((T, B)).astype(np.float32))
    saved, cursor, size = m.gpu.arena.clone(), m.gpu.cursor, m.gpu.size
    fresh = PrioritizedReplay(K, N, T, FIELDS)
    fresh.arena.copy_(saved)
    fresh.set_ring(cursor, size)
    m.gpu = fresh
    for it in range(3):
        m.update(rng.integers(0, 300, (T, B)).astype(np.uint32), rng.random((T, B)).astype(np.float32))
        m.compare_tree()
    gi, ci = m.sample(wl.uniform01(rng, (T, 257)), beta=0.5, fused_rows=True)
    m.insert(2000)
    m.compare_tree()
    m.compare_status()


def test_determinism_same_state_same_bits():
    rng = np.random.default_rng(0)
    N, B = 100000, 4096
    leaves = wl._draw_priorities("pareto_1.5", rng, (1, N))
    u = wl.uniform01(rng, (1, B))
    idx = rng.integers(0, N, (1, B)).astype(np.uint32)
    pr = rng.random((1, B)).astype(np.float32)
    outs = []
    for rep in range(2):
        p = PrioritizedReplay(16, N)
        p.insert(N, None, dev(leaves))
        p.update(idx_to_dev(idx), dev(pr))
        i, w, v = p.sample(dev(u), 0.4)
        outs.append([i.cpu().numpy().tobytes(), w.cpu().numpy().tobytes(), v.cpu().numpy().tobytes()] +
                    [p.read_level(0, h).cpu().numpy().tobytes() for h in range(p.H + 1)])
    assert outs[0] == outs[1]


# ------------------------------------------------------------------ edge cases
def test_denormals_and_negative_zero_on_gpu():
    tiny = np.float32(1e-42)
    leaves = np.array([[0.0, -0.0, tiny, 0.0, tiny, -0.0, tiny, tiny]], np.float32)
    for K in (2, 4, 8):
        m = Mirror(K, 8, 1, ())
        m.insert(8, prio=leaves, with_rows=False)
        m.compare_tree()
        gi, ci = m.sample(np.array([[0.0, 0.5, 0.5, 0.99]], np.float32))
        assert ci[0].tolist() == [2, 4, 6, 7]
        m.compare_status()


def test_zero_total_empty_and_error_codes():
    p = PrioritizedReplay(4, 100, 2, (8,))
    u = dev(np.zeros((2, 16), np.float32))
    with pytest.raises(PerError) as e:
        p.sample(u)
    assert e.value.code == EEMPTY
    p.insert(10, None, dev(np.zeros((2, 10), np.float32)))     # rows present, all priorities zero
    idx, w, v = p.sample(u)
    assert np.all(idx_to_host(idx) == 0xFFFFFFFF) and np.all(w.cpu().numpy() == 0) and np.all(v.cpu().numpy() == 0)
    assert p.status() == FLAG_ZERO_TOTAL
    rows = p.gather(idx)                                        # sentinel indices gather zeros
    assert np.all(rows[0].cpu().numpy() == 0) and p.status() == FLAG_ZERO_TOTAL | FLAG_BAD_INDEX
    p.clear_status()
    fused = [torch.full((2, 16, 8), 7, dtype=torch.uint8, device="cuda")]
    idx, w, v = p.sample(u, rows_out=fused)                     # same through the fused call
    assert np.all(idx_to_host(idx) == 0xFFFFFFFF) and np.all(fused[0].cpu().numpy() == 0)
    assert p.status() == FLAG_ZERO_TOTAL | FLAG_BAD_INDEX
    p.clear_status()
    assert p.status() == 0
    with pytest.raises(PerError) as e:
        p.insert(101)
    assert e.value.code == ERANGE
    with pytest.raises(PerError) as e:
        p.sample(u, beta=-1.0)
    assert e.value.code == EINVAL
    # empty batches are valid and change nothing
    p.update(torch.empty((2, 0), dtype=torch.int32, device="cuda"), torch.empty((2, 0), device="cuda"))
    p.insert(0)
    assert p.size == 10 and p.cursor == 10
    for bad in [dict(fanout=3), dict(fanout=128), dict(capacity=0), dict(n_trees=0), dict(init_max_priority=0.0)]:
        kw = dict(fanout=4, capacity=10)
        kw.update(bad)
        with pytest.raises(PerError):
            PrioritizedReplay(**kw)


def test_priority_retrieval_and_flags():
    m = Mirror(16, 300, 2, ())
    rng = np.random.default_rng(1)
    m.insert(200, prio=rng.random((2, 200)).astype(np.float32), with_rows=False)
    idx = rng.integers(0, 300, (2, 64)).astype(np.uint32)
    idx[:, 5] = 300
    got = m.gpu.get_priority(idx_to_dev(idx)).cpu().numpy()
    want = m.cpu.get_priority(idx)
    assert got.tobytes() == want.tobytes()
    m.compare_status()
    assert m.gpu.status() == FLAG_BAD_INDEX


@pytest.mark.parametrize("K", [16, 32])
def test_results_do_not_depend_on_tuning(K):
    rng = np.random.default_rng(3)
    N, B = 1 << 16, 5000
    leaves = wl._draw_priorities("pareto_1.5", rng, (1, N))
    u = wl.uniform01(rng, (1, B))
    ref = None
    for lds, blk, lazy in [(0, 64, 1), (4096, 256, 0), (64 * 1024, 256, 1), (96 * 1024, 1024, 0), (160 * 1024, 512, 1)]:
        p = PrioritizedReplay(K, N)
        p.set_tuning("lds_budget_bytes", lds)
        p.set_tuning("lazy_top", lazy)
        for name in ("sample_block", "update_block", "gather_block", "tree_block"):
            p.set_tuning(name, blk)
        p.insert(N, None, dev(leaves))
        i, w, v = p.sample(dev(u), 0.5)
        p.update(i, dev(np.full((1, B), 0.25, np.float32)))
        i2, w2, v2 = p.sample(dev(u), 0.5)          # reads the tree the update left behind
        p.update(i2, dev(np.full((1, B), 0.75, np.float32)))
        out = [x.cpu().numpy().tobytes() for x in (i, v, w, i2, v2, w2)] + \
              [p.read_level(0, h).cpu().numpy().tobytes() for h in range(p.H + 1)]
        if ref is None:
            ref = out
        assert out == ref, (lds, blk)


@pytest.mark.parametrize("K,N", [(2, (1 << 20) + 77), (8, 3 << 20), (16, 1 << 16), (64, 300001), (4, 70001)])
def test_update_sample_chain(K, N):
    """Update -> sample -> update -> insert chains, on trees large enough that the update finishes the
    top heights itself (K = 2, 8) and on one where it leaves them to the next reader (K = 16)."""
    log(f"chain K={K} N={N}")
    rng = np.random.default_rng(N + K)
    m = Mirror(K, N, 1, ())
    m.insert(N, prio=wl._draw_priorities("exponential_1", rng, (1, N)), with_rows=False)
    for it in range(3):
        B = 2000
        idx = rng.integers(0, N, (1, B)).astype(np.uint32)
        m.update(idx, rng.random((1, B)).astype(np.float32))
        gi, ci = m.sample(wl.uniform01(rng, (1, 777)), 0.4)
        m.update(ci, rng.random((1, 777)).astype(np.float32))
        if it == 1:
            m.compare_tree()
        m.update(idx, rng.random((1, B)).astype(np.float32))     # two updates in a row
        m.sample_gather_update(wl.uniform01(rng, (1, 500)), 0.7, True, rng.random((1, 500)).astype(np.float32),
                               alias=(it % 2 == 0))                # fused step right after an update
        m.insert(100)                                             # insert right after an update
        m.compare_tree()
    m.compare_status()


@pytest.mark.parametrize("K,N,B,fb", [(32, 1 << 17, 3000, (128,)), (16, 50000, 700, (68, 24, 4, 68, 1)), (2, 5000, 64, ())])
def test_fused_step_wherever_the_update_batch_lies(K, N, B, fb):
    """per_sample_gather_update places the claim phase of its update by where the update batch lies: the
    sampled batch itself, memory apart from the sampling outputs (also with another batch size), or a
    part of the output index array.  All three, and the three-kernel form forced by the tuning knob,
    against the oracle."""
    log(f"fused step placements K={K} N={N} B={B}")
    rng = np.random.default_rng(K * N + B)
    m = Mirror(K, N, 1, fb)
    m.insert(N, prio=wl._draw_priorities("pareto_1.5", rng, (1, N)))
    for knob in (1, 0):
        m.gpu.set_tuning("claim_in_sample", knob)
        for want_w in (True, False):
            pr = lambda n: rng.random((1, n)).astype(np.float32)
            m.sample_gather_update(wl.uniform01(rng, (1, B)), 0.5, want_w, pr(B), alias=True)
            m.compare_tree()
            m.sample_gather_update(wl.uniform01(rng, (1, B)), 0.5, want_w, pr(B), alias=False)
            m.compare_tree()
            m.sample_gather_update(wl.uniform01(rng, (1, B)), 0.5, want_w, pr(B), tail=B // 3)
            m.compare_tree()
            # an update batch of another size than the sampled one, in memory of its own
            idx = rng.integers(0, N, (1, 2 * B + 5)).astype(np.uint32)
            ci, cw, cv = m.cpu.sample(u := wl.uniform01(rng, (1, B)), 0.5, want_w)
            up = pr(2 * B + 5)
            gi, gw, gv = m.gpu.sample(dev(u), 0.5, want_weights=want_w, want_prio=True,
                                      update=(idx_to_dev(idx), dev(up)))
            assert np.array_equal(idx_to_host(gi), ci)
            m.cpu.update(idx, up)
            m.compare_tree()
    m.compare_status()


def test_sampling_frequency_on_gpu():
    rng = np.random.default_rng(12345)
    N, B, steps = 256, 64, 2000
    td = wl.td_to_priority(rng.standard_normal(N), 1e-6, 0.6)
    p = PrioritizedReplay(16, N)
    p.insert(N, None, dev(td[None]))
    u = dev(wl.uniform01(rng, (steps, B)))
    counts = np.zeros(N)
    for s in range(steps):
        idx, _, _ = p.sample(u[s:s + 1], want_weights=False, want_prio=False)
        np.add.at(counts, idx_to_host(idx)[0], 1)
    expect = B * steps * td.astype(np.float64) / td.astype(np.float64).sum()
    assert float(((counts - expect) ** 2 / expect).sum()) < stats.chi2.ppf(0.9999, N - 1)


# ------------------------------------------------------------------ whole workloads
@pytest.mark.parametrize("name,steps,tree_every", [
    ("c1_binary_small", 100, 1),
    ("c2_dqn", 300, 25),
    ("c3_ddpg", 60, 10),
])
def test_workload_parity(name, steps, tree_every):
    w = wl.WORKLOADS[name]
    log(f"workload {name}: {steps} steps")
    m = Mirror(w.K, w.N, w.T, w.field_bytes)
    m.insert(w.N, prio=wl.initial_priorities(w, 0), chunk=1 << 18)
    m.compare_tree()
    for s in range(steps):
        m.step(w, s, check_tree=(s % tree_every == 0 or s == steps - 1))
    m.compare_status()


def test_workload_c5_many_trees():
    w = wl.WORKLOADS["c5_multi"]
    log("workload c5_multi")
    m = Mirror(w.K, w.N, w.T, w.field_bytes, oracle_payload=False)
    m.insert(w.N, prio=wl.initial_priorities(w, 0), chunk=1 << 16)
    m.compare_tree(heights=range(1, m.gpu.H + 1))
    for s in range(12):
        m.step(w, s, check_tree=False)
        if s % 4 == 3:
            m.compare_tree(heights=range(1, m.gpu.H + 1))
    m.compare_tree()
    m.compare_status()


def test_workload_c4_full_size():
    """N = 2^24, B = 65536 in the launch configuration the bench times.  The oracle runs the full
    descent and update; gathered rows are checked against the row hash of the slot they came from."""
    w = wl.WORKLOADS["c4_stress"]
    log("workload c4_stress (full size)")
    m = Mirror(w.K, w.N, w.T, w.field_bytes, oracle_payload=False)
    v0 = wl.initial_priorities(w, 0)
    m.insert(w.N, prio=v0, chunk=1 << 20)
    log("  filled")
    m.compare_tree()
    for s in range(4):
        inp = wl.step_inputs(w, s, 0)
        if s % 2 == 0:     # the call sequence the bench times: whole step fused
            leaves = m.cpu.read_level(0, 0)
            gi, ci = m.sample_gather_update(inp["u"], inp["beta"], True, inp["upd_prio"], dup=inp)
            assert np.all(leaves[ci[0]] > 0), "a zero-priority row was sampled"
        else:
            gi, ci = m.sample(inp["u"], inp["beta"], True, fused_rows=True)
            assert np.all(m.cpu.read_level(0, 0)[ci[0]] > 0), "a zero-priority row was sampled"
            m.gather(gi, ci)
            m.update(wl.apply_dup_map(ci, inp), inp["upd_prio"])
        m.compare_tree(heights=range(1, m.gpu.H + 1))
        log(f"  step {s} ok")
    m.compare_tree()
    m.compare_status()


@pytest.mark.parametrize("name,steps", [("c2_dqn", 10000), ("c3_ddpg", 2000), ("c4_stress", 600), ("c5_multi", 1000)])
def test_workloads_at_full_length(name, steps, claim_form):
    """The workloads over their whole length (the stress workload past the point where the stamp counter of the claim
    group entries turns over, every 512 of its steps): indices, sampled values, weights and rows compared with the
    oracle at every step, every stored node every 50th step and at the end; the first mismatch stops the run.
    The steps rotate through the call forms (separate calls, sample + gather, the fused step with a separate
    update array, per_step).  One run per workload (the default claim form)."""
    if claim_form != "group":
        pytest.skip("one run per workload")
    import time
    w = wl.WORKLOADS[name]
    t0 = time.time()
    log(f"workload {name}: all {steps} steps")
    big = w.N * w.T >= 1 << 24
    m = Mirror(w.K, w.N, w.T, w.field_bytes, oracle_payload=not big)
    m.insert(w.N, prio=wl.initial_priorities(w, 0), chunk=1 << (20 if w.T == 1 else 16))
    m.compare_tree()
    for s in range(steps):
        m.step(w, s, check_tree=False)
        if s % 50 == 49 or s == steps - 1:
            m.compare_tree()
            log(f"  {name}: step {s + 1} of {steps}, tree equal, {time.time() - t0:.0f} s")
    m.compare_status()


# ---------------------------------------------------------------------------------------------
# Priority update in the paper's form (per_update_delta, Section V-A).  Changes meet in no fixed order,
# so: bit-exact against the oracle where every fp32 sum is exact (dyadic values: any order gives the same
# bits, which checks every index, level and sign), and within a rounding bound of the fp64 sums elsewhere.
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("K,N,T,B", [(2, 5000, 1, 700), (4, 70001, 2, 3000), (16, 1 << 18, 3, 4096),
                                     (32, 1 << 20, 1, 65536), (64, 300001, 1, 9000)])
def test_delta_update_is_exact_on_dyadic_values(K, N, T, B):
    log(f"delta update, dyadic K={K} N={N} T={T} B={B}")
    rng = np.random.default_rng(K + N + B)
    scale = np.float32(2.0 ** -5)
    top = max(4, min(1 << 10, (1 << 22) // N))         # all partial sums (also with duplicates) stay exact
    m = Mirror(K, N, T, ())
    m.insert(N, prio=(rng.integers(top // 2, top, (T, N)) * scale).astype(np.float32), with_rows=False)
    for it in range(3):
        idx = rng.integers(0, N, (T, B)).astype(np.uint32)          # duplicates add up
        delta = (rng.integers(-(top // 4) // 8, top // 4, (T, B)) * scale).astype(np.float32)
        if it == 1:                                                  # a few elements that must be skipped
            idx[:, ::97] = N + 5
            delta[:, 5::101] = np.float32("inf")
        if it == 2:                                                  # right after an update that left the top stale
            ui = rng.integers(0, N, (T, 100)).astype(np.uint32)
            m.update(ui, (rng.integers(1, top, (T, 100)) * scale).astype(np.float32))
        m.gpu.update_delta(idx_to_dev(idx), dev(delta))
        m.cpu.update_delta(idx, delta)
        m.compare_tree()
    assert m.gpu.status() == m.cpu.status == (FLAG_BAD_INDEX | FLAG_BAD_PRIORITY)


def test_retrieval_then_delta_update_equals_the_set_form_on_dyadic_values():
    """The paper realises a priority update as retrieval followed by the delta update."""
    K, N, B = 16, 1 << 16, 5000
    rng = np.random.default_rng(5)
    scale = np.float32(2.0 ** -4)
    m = Mirror(K, N, 1, ())
    m.insert(N, prio=(rng.integers(1, 64, (1, N)) * scale).astype(np.float32), with_rows=False)
    idx = rng.choice(N, size=(1, B), replace=False).astype(np.uint32)
    new = (rng.integers(0, 64, (1, B)) * scale).astype(np.float32)
    di = idx_to_dev(idx)
    old = m.gpu.get_priority(di)
    m.gpu.update_delta(di, dev(new) - old)
    m.cpu.update(idx, new)                       # the oracle's set form
    m.compare_tree(heights=range(m.gpu.H + 1))


@pytest.mark.parametrize("K,N,B", [(32, 1 << 20, 65536), (8, 100000, 4000)])
def test_delta_update_stays_within_the_rounding_bound(K, N, B):
    log(f"delta update, floats K={K} N={N} B={B}")
    rng = np.random.default_rng(N + B)
    leaves = rng.exponential(1.0, (1, N)).astype(np.float32)
    p = PrioritizedReplay(K, N)
    p.insert(N, None, dev(leaves))
    truth = leaves[0].astype(np.float64)
    steps = 5
    for _ in range(steps):
        idx = rng.integers(0, N, (1, B)).astype(np.uint32)
        delta = (rng.standard_normal((1, B)) * 0.1).astype(np.float32)
        p.update_delta(idx_to_dev(idx), dev(delta))
        np.add.at(truth, idx[0], delta[0].astype(np.float64))
    HB = p.H * (K.bit_length() - 1)
    for h in range(p.H + 1):
        got = p.read_level(0, h).cpu().numpy().astype(np.float64)
        n, span = got.size, K ** h
        pad = np.zeros(n * span)
        pad[:N] = truth
        mag = np.zeros(n * span)
        mag[:N] = np.abs(leaves[0].astype(np.float64)) + 0.1 * 4 * steps
        # every addition rounds by at most half an ulp of a partial result bounded by the magnitudes below the node
        adds = HB + steps * B
        bound = 2.0 ** -23 * np.minimum(adds, span * 64 + 64) * mag.reshape(n, span).sum(axis=1)
        assert np.all(np.abs(got - pad.reshape(n, span).sum(axis=1)) <= bound), h
    assert p.status() == 0
    # sampling still works on the drifted tree
    i, w, v = p.sample(dev(wl.uniform01(rng, (1, 1000))), 0.4)
    assert int(idx_to_host(i).max()) < N


@pytest.mark.parametrize("K,N,T,fb", [(2, 1000, 1, (5,)), (16, 5000, 3, (68, 24, 4, 68, 1)), (32, 40000, 1, (128,)),
                                      (64, 4097, 2, ())])
@pytest.mark.parametrize("one_kernel", [1, 0])
def test_small_inserts_in_one_kernel_or_several(K, N, T, fb, one_kernel):
    """Few rows per insert take a single-kernel path (rows, leaves and ancestors by one workgroup per tree);
    it must behave like the general path: ring wrap-around, explicit and default priorities, invalid
    priorities, and heights that the preceding update left to its next reader."""
    log(f"small inserts K={K} N={N} T={T} one_kernel={one_kernel}")
    rng = np.random.default_rng(K + N + T)
    m = Mirror(K, N, T, fb)
    m.gpu.set_tuning("insert_small", one_kernel)
    m.insert(N - 7, prio=wl._draw_priorities("exponential_1", rng, (T, N - 7)), chunk=3000)   # ring almost full
    for it, n in enumerate([1, 5, 16, 3, 200, 64, 1000, 7]):
        if it % 2 == 0:
            m.insert(n)                                   # running maximum; the ring wraps during these steps
        else:
            pr = rng.random((T, n)).astype(np.float32) * 3
            if it == 3:
                pr[:, 1] = np.float32("nan")
            m.insert(n, prio=pr)
        m.compare_tree()
        idx = rng.integers(0, N, (T, 300)).astype(np.uint32)
        m.update(idx, rng.random((T, 300)).astype(np.float32) * 5)     # leaves the top heights stale on larger trees
    gi, ci = m.sample(wl.uniform01(rng, (T, 256)), 0.4)
    m.gather(gi, ci)
    m.compare_tree()
    m.compare_status()


@pytest.mark.parametrize("K,N,T,B", [(16, 1 << 16, 2, 5000), (32, 1 << 20, 1, 65536)])
def test_update_from_td_errors(K, N, T, B):
    """per_update_td: the priority (|td| + eps)^alpha is computed on the device in fp64.  Two power routines
    may differ in the last bit, so the leaves are compared within one fp32 rounding and the tree above
    them bit for bit against the oracle's set form fed with the device's own leaf values."""
    log(f"update from TD errors K={K} N={N} T={T} B={B}")
    rng = np.random.default_rng(B + K)
    m = Mirror(K, N, T, ())
    m.insert(N, prio=wl._draw_priorities("exponential_1", rng, (T, N)), with_rows=False)
    idx = rng.integers(0, N, (T, B)).astype(np.uint32)          # duplicates: last writer wins
    td = (rng.standard_normal((T, B)) * 2).astype(np.float32)
    td[:, 3::500] = np.float32("nan")
    m.gpu.update_td(idx_to_dev(idx), dev(td), 1e-6, 0.6)
    m.cpu.update_td(idx, td, 1e-6, 0.6)
    for t in range(T):
        g = m.gpu.read_level(t, 0).cpu().numpy()
        c = m.cpu.read_level(t, 0)
        np.testing.assert_allclose(g, c, rtol=2.0 ** -23, atol=0)
        ref = MultiOracle(1, K, N, ())         # the set form on the device's own leaves must give the device's tree
        ref.insert(N, None, g[None])
        for h in range(m.gpu.H + 1):
            assert m.gpu.read_level(t, h).cpu().numpy().tobytes() == ref.read_level(0, h).tobytes(), (t, h)
    assert m.gpu.status() == m.cpu.status == FLAG_BAD_PRIORITY
    assert np.allclose(m.gpu.max_priority().cpu().numpy(), [o.max_priority for o in m.cpu.trees], rtol=2.0 ** -23)


@pytest.mark.parametrize("K,N,T,B", [(16, 1 << 16, 3, 1000), (32, 1 << 20, 1, 65536), (2, 4096, 1, 64)])
def test_sampling_with_uniforms_drawn_on_the_device(K, N, T, B):
    """Sampling calls without a uniform array draw from the counter-based generator; the oracle side has its
    own implementation of the same published generator, so indices, values and rows must match bit for bit."""
    from oracle.per_oracle import uniforms
    log(f"device uniforms K={K} N={N} T={T} B={B}")
    rng = np.random.default_rng(K * B)
    fb = (12,)
    m = Mirror(K, N, T, fb)
    m.insert(N, prio=wl._draw_priorities("lognormal_0_1", rng, (T, N)))
    seed = 0xC0FFEE1234567890
    with pytest.raises(Exception):
        m.gpu.sample(None, 0.4, B=B)                       # no generator set up yet
    m.gpu.set_rng(seed, next_call=(1 << 32) - 1)           # the call counter crosses a word boundary below
    for step in range(3):
        call = m.gpu.rng_calls()
        u = np.stack([uniforms(seed, call, t, B) for t in range(T)])
        rows = [torch.empty((T, B, b), dtype=torch.uint8, device="cuda") for b in fb]
        upd = rng.random((T, B)).astype(np.float32)
        out_idx = torch.empty((T, B), dtype=torch.int32, device="cuda")
        gi, gw, gv = m.gpu.sample(None, 0.5, B=B, out_idx=out_idx, rows_out=rows,
                                  update=(out_idx, dev(upd)) if step < 2 else None)
        ci, cw, cv = m.cpu.sample(u, 0.5, True)
        assert np.array_equal(idx_to_host(gi), ci) and gv.cpu().numpy().tobytes() == cv.tobytes()
        np.testing.assert_allclose(gw.cpu().numpy(), cw, rtol=1e-6, atol=0)
        m.gather(gi, ci, got=rows)
        if step < 2:
            m.cpu.update(ci, upd)
        assert m.gpu.rng_calls() == call + 1
    m.compare_tree()


# ---------------------------------------------------------------------------------------------
# per_run_steps: a list of steps in one launch on an LDS copy of the tree.  Same results as the calls.
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("K,N,T,B,n_ins,fb,explicit", [
    (2, 4096, 1, 64, 4, (16, 4, 4, 16, 1), False), (16, 30000, 2, 512, 16, (12,), True),
    (32, 32768, 1, 1024, 0, (128,), False), (4, 1000, 3, 100, 7, (), True), (64, 20000, 1, 33, 1, (5,), False),
    # trees whose leaves stay in memory (heights 1 .. H in LDS): the paper's 100K entries and beyond
    (16, 100000, 2, 512, 16, (12,), True), (8, 200001, 1, 300, 4, (4, 1), False), (32, 1 << 20, 1, 1024, 8, (), True),
    (64, 1500000, 1, 700, 3, (8,), False)])
@pytest.mark.parametrize("own_batch", [True, False])
def test_run_steps_equals_the_separate_calls(K, N, T, B, n_ins, fb, explicit, own_batch):
    log(f"run_steps K={K} N={N} T={T} B={B} n_ins={n_ins} own_batch={own_batch}")
    rng = np.random.default_rng(K * N + B + n_ins)
    m = Mirror(K, N, T, fb)
    assert m.gpu.run_steps_fits()
    m.insert(N - 10, prio=wl._draw_priorities("exponential_1", rng, (T, N - 10)), chunk=max(5000, N // 8))   # the ring wraps below
    steps = 6
    u = wl.uniform01(rng, (steps, T, B))
    beta = np.linspace(0.4, 1.0, steps).astype(np.float32)
    upd_prio = (rng.random((steps, T, B)) * 4).astype(np.float32)
    upd_prio[2, :, ::7] = np.float32("nan")
    upd_prio[3, :, 1::9] = -1.0
    upd_idx = rng.integers(0, N, (steps, T, B)).astype(np.uint32)
    upd_idx[:, :, 1::2] = upd_idx[:, :, 0::2][:, :, :upd_idx[:, :, 1::2].shape[2]]   # every other element repeats its neighbour
    upd_idx[4, :, 0] = N + 3                                                        # out of range
    counters = m.counter + np.arange(steps * n_ins).reshape(steps, n_ins) if n_ins else None
    ins_rows = [np.stack([np.stack([wl.row_bytes(t, counters[s], f, b) for t in range(T)]) for s in range(steps)])
                for f, b in enumerate(fb)] if n_ins and fb else None
    ins_prio = (rng.random((steps, T, n_ins)) * 6).astype(np.float32) if explicit and n_ins else None
    if ins_prio is not None:
        ins_prio[1, :, 0] = np.float32("inf")
    out_idx = torch.empty((steps, T, B), dtype=torch.int32, device="cuda")
    out_w = torch.empty((steps, T, B), dtype=torch.float32, device="cuda")
    out_v = torch.empty((steps, T, B), dtype=torch.float32, device="cuda")
    rows_out = [torch.empty((steps, T, B, b), dtype=torch.uint8, device="cuda") for b in fb] if fb else None
    m.gpu.run_steps(dev(u), dev(beta), out_idx, out_w, out_v, rows_out, upd_prio=dev(upd_prio),
                    upd_idx=None if own_batch else idx_to_dev(upd_idx), n_insert=n_ins,
                    ins_rows=[dev(r) for r in ins_rows] if ins_rows else None,
                    ins_prio=None if ins_prio is None else dev(ins_prio))
    gi = idx_to_host(out_idx)
    gw, gv = out_w.cpu().numpy(), out_v.cpu().numpy()
    grows = [r.cpu().numpy() for r in rows_out] if fb else []
    for s in range(steps):
        if n_ins:
            m.cpu.insert(n_ins, [r[s] for r in ins_rows] if ins_rows else None, None if ins_prio is None else ins_prio[s])
        ci, cw, cv = m.cpu.sample(u[s], float(beta[s]), True)
        assert np.array_equal(gi[s], ci), f"step {s}: sampled indices"
        assert gv[s].tobytes() == cv.tobytes(), f"step {s}: sampled values"
        np.testing.assert_allclose(gw[s], cw, rtol=1e-6, atol=0)
        for f, want in enumerate(m.cpu.gather(ci)):
            assert np.array_equal(grows[f][s], want), f"step {s}: rows of field {f}"
        m.cpu.update(ci if own_batch else upd_idx[s], upd_prio[s])
    m.counter += steps * n_ins
    m.compare_tree()
    m.compare_status()
    assert m.gpu.cursor == m.cpu.trees[0].cursor and m.gpu.size == m.cpu.trees[0].size
    if not fb:   # the separate calls carry on from the state the step kernel left
        m.update(rng.integers(0, N, (T, 50)).astype(np.uint32), rng.random((T, 50)).astype(np.float32))
        m.sample(wl.uniform01(rng, (T, B)), 0.4)
        m.compare_tree()


def test_run_steps_limits_and_empty_tree():
    p = PrioritizedReplay(16, 1 << 20)
    assert not p.run_steps_fits()
    z = torch.zeros((1, 1, 8), device="cuda")
    with pytest.raises(PerError) as e:
        p.run_steps(z, torch.zeros(1, device="cuda"), torch.zeros((1, 1, 8), dtype=torch.int32, device="cuda"))
    assert e.value.code == ERANGE
    q = PrioritizedReplay(4, 256)
    q.insert(256, None, torch.zeros((1, 256), device="cuda"))          # nothing can be sampled
    oi = torch.zeros((2, 1, 8), dtype=torch.int32, device="cuda")
    ow = torch.ones((2, 1, 8), device="cuda")
    q.run_steps(torch.zeros((2, 1, 8), device="cuda"), torch.zeros(2, device="cuda"), oi, ow)
    assert np.all(idx_to_host(oi) == 0xFFFFFFFF) and float(ow.abs().max()) == 0.0
    assert q.status() == FLAG_ZERO_TOTAL


# ---------------------------------------------------------------------------------------------
# a captured fused step can be replayed: nothing of a sampling + update call lives in host counters
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("K,N,B", [(16, 50000, 4096), (32, 300000, 20000), (2, 4096, 64)])
def test_captured_step_replays(K, N, B):
    """One per_sample_gather_update call (uniforms given, weights, rows, update of the batch sampled before) is
    captured into a HIP graph and replayed with fresh inputs in the same buffers; eager calls run between
    the replays.  Every replay must give what the oracle gives for that step."""
    log(f"graph replay K={K} N={N} B={B}")
    rng = np.random.default_rng(K + B)
    T, fb = 1, (32,)
    m = Mirror(K, N, T, fb)
    m.insert(N, prio=wl._draw_priorities("lognormal_0_1", rng, (T, N)), chunk=100000)
    u_buf = torch.empty((T, B), dtype=torch.float32, device="cuda")
    upd_idx = torch.empty((T, B), dtype=torch.int32, device="cuda")
    upd_prio = torch.empty((T, B), dtype=torch.float32, device="cuda")
    oi = torch.empty((T, B), dtype=torch.int32, device="cuda")
    ow = torch.empty((T, B), dtype=torch.float32, device="cuda")
    ov = torch.empty((T, B), dtype=torch.float32, device="cuda")
    rows = [torch.empty((T, B, b), dtype=torch.uint8, device="cuda") for b in fb]

    def call():
        m.gpu.sample(u_buf, 0.5, out_idx=oi, out_weight=ow, out_prio=ov, rows_out=rows, update=(upd_idx, upd_prio))

    def feed():
        u = wl.uniform01(rng, (T, B))
        idx = rng.integers(0, N, (T, B)).astype(np.uint32)
        idx[:, 1::2] = idx[:, 0::2][:, :idx[:, 1::2].shape[1]]
        pr = wl._draw_updates("absnormal1_eps_pow0.6", rng, (T, B))
        u_buf.copy_(dev(u)); upd_idx.copy_(idx_to_dev(idx)); upd_prio.copy_(dev(pr))
        return u, idx, pr

    def check(u, idx, pr, tree=True):
        ci, cw, cv = m.cpu.sample(u, 0.5, True)
        assert np.array_equal(idx_to_host(oi), ci), "sampled indices"
        assert ov.cpu().numpy().tobytes() == cv.tobytes(), "sampled values"
        np.testing.assert_allclose(ow.cpu().numpy(), cw, rtol=1e-6, atol=0)
        for f, want in enumerate(m.cpu.gather(ci)):
            assert np.array_equal(rows[f].cpu().numpy(), want)
        m.cpu.update(idx, pr)
        if tree:
            m.compare_tree()

    args = feed()
    call()                                   # eager: leaves the buffer in the state every step starts from
    check(*args)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    args = feed()
    with torch.cuda.graph(graph):
        call()                               # recorded, not run
    for it in range(4):
        if it:
            args = feed()
        graph.replay()
        m.gpu.note_replay()
        torch.cuda.synchronize()
        check(*args)
        if it == 1:                          # the program's own eager work between replays
            m.update(rng.integers(0, N, (T, 100)).astype(np.uint32), rng.random((T, 100)).astype(np.float32))
            m.compare_tree()
    # the tight loop: captured right after a step, replayed back to back, the library not called in between
    # (only the outputs are read, through torch)
    args = feed()
    call()
    check(*args, tree=False)
    loop = torch.cuda.CUDAGraph()
    args = feed()
    with torch.cuda.graph(loop):
        call()
    for it in range(4):
        if it:
            args = feed()
        loop.replay()
        torch.cuda.synchronize()
        check(*args, tree=False)
    m.gpu.note_replay()
    m.compare_tree()
    m.compare_status()


@pytest.mark.parametrize("K,N,T,B,fb", [(32, 1 << 20, 1, 30000, (128,)), (16, 1 << 18, 3, 1024, (68, 24, 4, 68, 1)),
                                        (2, 5000, 1, 64, ()), (4, 70001, 2, 3000, (12,)), (64, 300001, 1, 5000, (8,)),
                                        (8, 1 << 21, 1, 9000, ())])
@pytest.mark.parametrize("one_kernel", [2, 3, 4, 0])
def test_step_call_updates_the_batch_it_draws(K, N, T, B, fb, one_kernel):
    """per_step: the update targets the leaves drawn by this very call, directly or through a position map
    (the duplicate map of the stress workload; maps with many elements on one sample; invalid positions).
    Run with sampling and update as one kernel where the tree takes it (the call ending inside that kernel, or,
    one_kernel = 3 and 4, in a second one: 3 with the owners' tables in the arena, 4 with the tables in the
    library's static array, which a buffer with one tree gets when it is free) and as separate kernels."""
    log(f"per_step K={K} N={N} T={T} B={B} one_kernel={one_kernel}")
    rng = np.random.default_rng(K * 31 + B)
    m = Mirror(K, N, T, fb)
    m.gpu.set_tuning("step_kernel", min(one_kernel, 2))
    m.gpu.set_tuning("step_tail", 0 if one_kernel >= 3 else 1)
    m.gpu.set_tuning("static_tables", 0)
    if one_kernel == 4:
        gc.collect()
        if T == 1 and K >= 8:                      # (trees that the one-kernel form takes)
            m.gpu.set_tuning("static_tables", 1)   # (free: every other buffer of this process has been destroyed or has given it back)
        else:
            with pytest.raises(Exception):
                m.gpu.set_tuning("static_tables", 1)
    prio = wl._draw_priorities("pareto_1.5", rng, (T, N))
    prio[rng.random((T, N)) < 0.01] = 0.0
    m.insert(N, prio=prio, chunk=1 << 18)
    for it in range(8):
        u = wl.uniform01(rng, (T, B))
        pr = wl._draw_updates("absnormal1_eps_pow0.6", rng, (T, B))
        if it % 4 == 0:
            pos = None
        elif it % 4 == 1:                      # a tenth of the elements redirected to another sample's leaf
            pos = np.tile(np.arange(B, dtype=np.uint32), (T, 1))
            for t in range(T):
                dst = rng.choice(B, size=B // 10, replace=False)
                pos[t, dst] = rng.integers(0, B, B // 10)
        elif it % 4 == 2:                      # everything onto a handful of samples; some elements invalid
            pos = rng.integers(0, 7, (T, B)).astype(np.uint32)
            pos[:, ::5] = B + 3
            pr[:, 1::7] = np.float32(-1.0)
        else:                                   # a random permutation
            pos = np.stack([rng.permutation(B) for _ in range(T)]).astype(np.uint32)
        m.step_call(u, 0.4 + 0.05 * it, it % 2 == 0, pr, pos)
        m.compare_tree()
        if it % 4 == 2:
            assert m.gpu.status() & (FLAG_BAD_INDEX | FLAG_BAD_PRIORITY) == (FLAG_BAD_INDEX | FLAG_BAD_PRIORITY)
    m.compare_status()


def test_static_tables_change_hands():
    """Two buffers with one tree each, stepped in turn: the library's static table array belongs to one of them at
    a time; it is taken, refused while the other holds it, given back and taken over, and every step of both
    buffers matches the oracle whichever of them holds it."""
    log("static tables change hands")
    gc.collect()
    rng = np.random.default_rng(77)
    K, N, B = 16, 1 << 18, 40000
    a = Mirror(K, N, 1, (8,))
    b = Mirror(K, N, 1, (8,))
    for m in (a, b):
        m.gpu.set_tuning("step_kernel", 2)
        m.insert(N, prio=wl._draw_priorities("pareto_1.5", rng, (1, N)), chunk=1 << 18)

    def steps(m, n=2):
        for _ in range(n):
            m.step_call(wl.uniform01(rng, (1, B)), 0.5, True, wl._draw_updates("absnormal1_eps_pow0.6", rng, (1, B)))
        m.compare_tree()

    a.gpu.set_tuning("static_tables", 1)            # a holds it (it did already if nobody else did when it was created)
    with pytest.raises(Exception):
        b.gpu.set_tuning("static_tables", 1)        # refused: held
    steps(a); steps(b); steps(a)
    a.gpu.set_tuning("static_tables", 0)            # given back: a goes on with the tables in its arena
    b.gpu.set_tuning("static_tables", 1)
    steps(b); steps(a); steps(b)
    del b, m                                        # destroyed while holding it (m: the loop variable above)
    gc.collect()
    a.gpu.set_tuning("static_tables", 1)
    steps(a)
    a.compare_status()


def kernel_launches(m):
    """{kernel name: launches} since profiling was switched on."""
    return {k: int(v[1]) for k, v in m.gpu.profile_read().items() if v[1]}


# shapes whose sampling kernel can carry an insertion (lazily rebuilt top within reach of its LDS copy), and two that cannot
RIDE_SHAPES = [(16, 1 << 20, 1, 32, (4, 4, 1, 8, 8), True), (16, 1 << 20, 1, 4096, (68, 24, 4, 68, 1), True),
               (16, 1 << 18, 4, 1024, (68, 24, 4, 68, 1), True), (32, 1 << 20, 1, 30000, (128,), True),
               (4, 50001, 2, 700, (12,), True), (8, 300001, 1, 2500, (), True), (64, 1 << 19, 1, 3000, (8,), True),
               (2, 5000, 1, 64, (3,), False), (4, 1 << 18, 1, 512, (), False)]


@pytest.mark.parametrize("K,N,T,B,fb,rides", RIDE_SHAPES)
def test_insert_carried_by_the_step(K, N, T, B, fb, rides):
    """per_insert_step = per_insert, then per_step: few rows and many, at the running maximum and at given priorities
    (above the running maximum, zero, invalid), slots that wrap around the ring's end, slots that are drawn and updated
    by the same step, with and without a position map, on a ring that is still filling.  Where the shape and the
    insertion's size allow it the sampling kernel carries the insertion (no insert kernel is launched); elsewhere the
    same call makes two."""
    log(f"per_insert_step K={K} N={N} T={T} B={B} rides={rides}")
    rng = np.random.default_rng(K * 7 + B)
    m = Mirror(K, N, T, fb)
    m.gpu.set_tuning("step_kernel", 0)
    filled = N - N // 8                                    # the ring fills up and wraps during the test
    prio = wl._draw_priorities("pareto_1.5", rng, (T, filled))
    prio[rng.random((T, filled)) < 0.01] = 0.0
    m.insert(filled, prio=prio, chunk=1 << 18)
    m.gpu.profile(True)
    sizes = [1, 4, K, K + 1, 3 * K * K + 5, 700, 16, 2]
    for it, n in enumerate(sizes):
        if it == 4:                                        # next to the ring's end: this insertion or the next wraps
            gap = N - (m.gpu.cursor % N)
            m.insert(max(gap - n // 2 - 1, 1), prio=wl._draw_priorities("pareto_1.5", rng, (T, max(gap - n // 2 - 1, 1))),
                     chunk=1 << 18)
        n = min(n, N)
        u = wl.uniform01(rng, (T, B))
        pr = wl._draw_updates("absnormal1_eps_pow0.6", rng, (T, B))
        ins = None
        if it % 3 == 1:                                    # given priorities: far above the rest (so the new slots are drawn), one invalid, one zero
            ins = (wl._draw_priorities("pareto_1.5", rng, (T, n)) * np.float32(1e4 if it == 1 else 1.0)).astype(np.float32)
            if n > 2:
                ins[:, 1] = np.float32(np.nan)
                ins[:, 2] = 0.0
        pos = None
        if it % 2 == 1:
            pos = np.stack([rng.permutation(B) for _ in range(T)]).astype(np.uint32)
            pos[:, ::9] = pos[:, 0:1]
        before = kernel_launches(m)
        m.insert_step_call(n, ins, u, 0.4 + 0.05 * it, it % 2 == 0, pr, pos)
        after = kernel_launches(m)
        own = {k: v - before.get(k, 0) for k, v in after.items() if v != before.get(k, 0)}
        log(f"  n={n}: launches {own}")
        carried = not any(k.startswith("k_insert") or k in ("k_rows_scatter", "k_resum_dense", "k_resum_tail") for k in own)
        if not rides:
            assert not carried, own
        elif n <= 4:                                       # (runs of child groups no longer than the sampling workgroup)
            assert carried, own
        m.compare_tree()
    m.gpu.profile(False)
    m.compare_status()


@pytest.mark.parametrize("K,N,T,B", [(32, 1 << 20, 1, 8192), (16, 1 << 18, 2, 2048), (8, 1 << 18, 1, 4096), (64, 1 << 19, 1, 3000)])
def test_step_call_when_the_mass_sits_in_few_places(K, N, T, B):
    """The samples of one subtree are one workgroup's work in the one-kernel step.  Here nearly all mass sits in one
    leaf (a run of several thousand equal samples), then in one subtree spread over many leaves, then at the two
    ends of the tree, then nowhere but one leaf; runs far longer than a workgroup go through the chunked path."""
    log(f"per_step, concentrated mass K={K} N={N} T={T} B={B}")
    rng = np.random.default_rng(K + B)
    m = Mirror(K, N, T, ())
    m.gpu.set_tuning("step_kernel", 2)
    base = (rng.random((T, N)).astype(np.float32) * 0.5 + 0.25).astype(np.float32)
    m.insert(N, prio=base, chunk=1 << 18, with_rows=False)
    hot = N // 3 + 5
    span = np.arange(hot, hot + 3000, dtype=np.uint32)
    stages = [
        (np.array([hot], dtype=np.uint32), np.float32(3e6)),                       # one leaf holds most of the mass
        (span, np.float32(2e3)),                                                  # one stretch of leaves does
        (np.array([0, 1, N - 2, N - 1], dtype=np.uint32), np.float32(5e6)),       # the two ends of the tree
    ]
    for idx, value in stages:
        ii = np.tile(idx, (T, 1))
        m.update(ii, np.full(ii.shape, value, dtype=np.float32))
        for rep in range(2):
            u = wl.uniform01(rng, (T, B))
            pr = wl._draw_updates("absnormal1_eps_pow0.6", rng, (T, B))
            pos = None
            if rep == 1:
                pos = np.stack([rng.permutation(B) for _ in range(T)]).astype(np.uint32)
                nn = min(pos[:, ::9].shape[1], pos[:, 1::9].shape[1])
                pos[:, 0:9 * nn:9] = pos[:, 1::9][:, :nn]
            m.step_call(u, 0.5, True, pr, pos)
            m.compare_tree()
    # everything to zero but one leaf
    every = np.tile(np.arange(N, dtype=np.uint32), (T, 1))
    zeros = np.zeros((T, N), dtype=np.float32)
    zeros[:, N // 2] = 0.75
    m.update(every, zeros)
    u = wl.uniform01(rng, (T, B))
    m.step_call(u, 0.5, True, wl._draw_updates("absnormal1_eps_pow0.6", rng, (T, B)), None)
    m.compare_tree()
    # and an empty total: nothing sampled, every element invalid
    m.update(np.full((T, 1), N // 2, dtype=np.uint32), np.zeros((T, 1), dtype=np.float32))
    for pos in (None, np.tile(np.arange(B, dtype=np.uint32)[::-1].copy(), (T, 1))):
        m.step_call(u, 0.5, True, wl._draw_updates("absnormal1_eps_pow0.6", rng, (T, B)), pos)
        assert m.gpu.status() & FLAG_ZERO_TOTAL
        m.compare_tree()
    m.insert(3, prio=np.full((T, 3), 0.5, dtype=np.float32), with_rows=False)
    m.step_call(u, 0.5, True, wl._draw_updates("absnormal1_eps_pow0.6", rng, (T, B)), None)
    m.compare_tree()
    m.compare_status()


@pytest.mark.parametrize("K,N,B", [(16, 1 << 20, 4096), (32, 300000, 20000)])
def test_step_captured_on_a_fresh_top_replays(K, N, B):
    """The capture happens right after an insert, when the topmost heights in memory are current and the host
    knows it.  From the second replay on they are stale (the replayed update leaves them to the next
    reader), so the captured sampling kernel must rebuild them whatever the host believed at capture time.
    Also: a sampling call captured alone, and per_total captured alone, replayed after eager updates."""
    log(f"graph captured on a fresh top K={K} N={N} B={B}")
    rng = np.random.default_rng(K * 7 + B)
    T = 1
    m = Mirror(K, N, T, ())
    m.insert(N, prio=wl._draw_priorities("exponential_1", rng, (T, N)), chunk=1 << 18, with_rows=False)
    u_buf = torch.empty((T, B), dtype=torch.float32, device="cuda")
    upd_prio = torch.empty((T, B), dtype=torch.float32, device="cuda")
    oi = torch.empty((T, B), dtype=torch.int32, device="cuda")
    ov = torch.empty((T, B), dtype=torch.float32, device="cuda")
    tot = torch.empty(T, dtype=torch.float32, device="cuda")
    m.insert(3, prio=np.full((T, 3), 2.0, dtype=np.float32), with_rows=False)   # leaves the top fresh
    torch.cuda.synchronize()
    step = torch.cuda.CUDAGraph()
    with torch.cuda.graph(step):       # sample, then update the batch just sampled
        m.gpu.sample(u_buf, 0.4, want_weights=False, out_idx=oi, out_prio=ov, update=(oi, upd_prio))
    only_sample = torch.cuda.CUDAGraph()
    with torch.cuda.graph(only_sample):
        m.gpu.sample(u_buf, 0.4, want_weights=False, out_idx=oi, out_prio=ov)
    only_total = torch.cuda.CUDAGraph()
    with torch.cuda.graph(only_total):
        m.gpu.lib.per_total(m.gpu._h, tot.data_ptr(), m.gpu._stream())
    for it in range(4):
        u = wl.uniform01(rng, (T, B))
        pr = wl._draw_updates("absnormal1_eps_pow0.6", rng, (T, B))
        u_buf.copy_(dev(u)); upd_prio.copy_(dev(pr))
        step.replay()
        torch.cuda.synchronize()
        ci, _, cv = m.cpu.sample(u, 0.4, False)
        assert np.array_equal(idx_to_host(oi), ci), f"replay {it}: sampled indices"
        assert ov.cpu().numpy().tobytes() == cv.tobytes()
        m.cpu.update(ci, pr)
        only_total.replay()            # the root must be rebuilt by the captured call itself
        torch.cuda.synchronize()
        assert tot.cpu().numpy().tobytes() == m.cpu.total.tobytes(), f"replay {it}: captured per_total"
        only_sample.replay()
        torch.cuda.synchronize()
        ci2, _, _ = m.cpu.sample(u, 0.4, False)
        assert np.array_equal(idx_to_host(oi), ci2), f"replay {it}: captured plain sampling"
    m.gpu.note_replay()
    m.compare_tree()
    m.compare_status()


@pytest.mark.parametrize("K,N", [(16, 1 << 20), (32, 1 << 22)])
def test_update_to_all_zero_on_a_tree_whose_top_is_rebuilt_lazily(K, N):
    """A tree large enough for the update to leave its topmost heights to the next reader: every stored row is
    updated to priority 0, then a plain sampling call finds the total 0.  That call has told the host that the
    top is current again, so it must have stored the rebuilt heights: total, a second sampling call and a small
    insert afterwards all agree with the oracle."""
    log(f"all-zero update, lazy top K={K} N={N}")
    rng = np.random.default_rng(K)
    T, n = 1, 64
    m = Mirror(K, N, T, ())
    m.insert(n, prio=(rng.random((T, n)).astype(np.float32) + 0.5), with_rows=False)
    idx = np.arange(n, dtype=np.uint32)[None, :]
    m.update(idx, np.zeros((T, n), dtype=np.float32))
    u = wl.uniform01(rng, (T, 256))
    m.sample(u, 0.4)                                   # total 0: indices 0xFFFFFFFF, flag ZERO_TOTAL
    assert m.gpu.status() & FLAG_ZERO_TOTAL
    assert m.gpu.total().cpu().numpy().tobytes() == m.cpu.total.tobytes(), "root after the all-zero update"
    m.sample(u, 0.4)
    m.compare_tree()
    m.insert(5, prio=np.full((T, 5), 0.25, dtype=np.float32), with_rows=False)
    m.compare_tree()
    m.sample(u, 0.4)
    m.compare_status()


def test_small_insert_that_would_overflow_the_default_lds_takes_the_general_path():
    """K = 2 near N = 2^19 with a few thousand rows: the single-workgroup insert would need more than 64 KB of
    staged child groups once an update has left the top stale; the insert must still succeed and match."""
    log("small insert, K=2, many staged groups")
    rng = np.random.default_rng(5)
    K, N, T, n = 2, (1 << 19) - 3, 1, 4000
    m = Mirror(K, N, T, ())
    m.insert(N, prio=wl._draw_priorities("uniform_1e-3_1", rng, (T, N)), chunk=1 << 17, with_rows=False)
    m.update(rng.integers(0, N, (T, 3000)).astype(np.uint32), rng.random((T, 3000)).astype(np.float32))
    m.insert(n, prio=rng.random((T, n)).astype(np.float32), with_rows=False)
    m.compare_tree()
    assert m.gpu.cursor == m.cpu.trees[0].cursor and m.gpu.size == m.cpu.trees[0].size
    m.compare_status()


@pytest.mark.parametrize("K,N,T,B", [(32, 1 << 18, 1, 30000), (16, 70001, 2, 5000), (2, 5000, 1, 300)])
def test_rebuild_restores_the_invariant_after_the_delta_form(K, N, T, B):
    """per_update_delta on arbitrary floats leaves the upper levels equal to the sums of their children only up
    to rounding; per_rebuild must make every level bit-equal to the oracle's set-form tree of the same leaves."""
    log(f"rebuild after delta K={K} N={N} T={T}")
    rng = np.random.default_rng(K + N)
    m = Mirror(K, N, T, ())
    m.insert(N, prio=wl._draw_priorities("lognormal_0_1", rng, (T, N)), chunk=1 << 17, with_rows=False)
    idx = rng.integers(0, N, (T, B)).astype(np.uint32)
    delta = (rng.random((T, B)).astype(np.float32) * 0.37).astype(np.float32)
    m.gpu.update_delta(idx_to_dev(idx), dev(delta))
    leaves = np.stack([m.gpu.read_level(t, 0).cpu().numpy() for t in range(T)])
    m.gpu.rebuild()
    # the oracle's set form fed with the device's leaves (every leaf set once: the invariant tree of those leaves)
    ref = MultiOracle(T, K, N, ())
    ref.insert(N, None, np.ascontiguousarray(leaves))
    for t in range(T):
        for h in range(m.gpu.H + 1):
            assert m.gpu.read_level(t, h).cpu().numpy().tobytes() == ref.read_level(t, h).tobytes(), (t, h)
    assert m.gpu.total().cpu().numpy().tobytes() == ref.total.tobytes()


# ---------------------------------------------------------------------------------------------
# importance weights relative to the whole buffer (companion minimum of the sum tree)
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("K", [2, 4, 8, 16, 32, 64])
@pytest.mark.parametrize("N,T", [(5, 2), (1000, 1), (4097, 3), (70000, 1)])
def test_buffer_wide_weights_through_an_operation_mix(K, N, T):
    """As the random operation mix, with the weights relative to the smallest positive leaf of the tree: the
    companion minimum has to follow large inserts (rebuilt), small inserts and updates (renewed in place),
    the delta-form update (rebuilt), zeros and duplicates; it is compared with its definition after every
    operation, and the weights with the oracle's."""
    log(f"buffer-wide weights K={K} N={N} T={T}")
    rng = np.random.default_rng(K * 7919 + N + T)
    m = Mirror(K, N, T, (8,))
    first = max(1, (2 * N) // 3)
    prio = wl._draw_priorities("lognormal_0_1", rng, (T, first))
    prio[:, ::5] = 0.0
    m.insert(first, prio=prio)
    m.set_weight_norm("buffer")
    m.compare_min_priority()
    for it in range(5):
        B = int(rng.choice([1, 3, 64, 257, 1500]))
        gi, ci = m.sample(wl.uniform01(rng, (T, B)), beta=float(rng.choice([0.4, 1.0])), fused_rows=(it % 2 == 0))
        upd_idx = ci.copy()
        if m.cpu.trees[0].size:
            upd_idx[:, ::2] = rng.integers(0, m.cpu.trees[0].size, upd_idx[:, ::2].shape)
        upd_prio = wl._draw_updates("absnormal1_eps_pow0.6", rng, (T, B))
        upd_prio[:, ::3] *= np.float32(1e-3)                       # new minima now and then
        if B > 4:
            upd_idx[:, B // 2:] = upd_idx[:, : B - B // 2]
            upd_prio[:, 1] = np.nan
            upd_prio[:, 2] = 0.0
        if it == 3:                                                # the current minimum goes away
            for t in range(T):
                leaves = m.cpu.read_level(t, 0)
                upd_idx[t, 0] = int(np.argmin(np.where(leaves > 0, leaves, np.inf)))
                upd_prio[t, 0] = 5.0
        m.update(upd_idx, upd_prio)
        m.compare_tree()
        m.compare_min_priority()
        n_ins = int(rng.integers(1, max(2, N // 2))) if it % 2 else int(rng.integers(1, 9))
        n_ins = min(n_ins, N)
        ins = wl._draw_priorities("exponential_1", rng, (T, n_ins)) * np.float32(1e-2 if it == 2 else 1.0)
        m.insert(n_ins, prio=None if it == 4 else ins)
        m.compare_min_priority()
        if it == 1:   # the delta form leaves the minimum to a rebuild (zeros: sums in any order stay bit-comparable)
            didx = rng.integers(0, m.cpu.trees[0].size, (T, 20)).astype(np.uint32)
            delta = np.zeros((T, 20), np.float32)
            m.gpu.update_delta(idx_to_dev(didx), dev(delta))
            m.cpu.update_delta(didx, delta)
            m.compare_min_priority()
    m.set_weight_norm("batch")                                     # and back: the largest weight is 1 again
    gi, ci = m.sample(wl.uniform01(rng, (T, 64)), beta=0.7)
    m.compare_status()


@pytest.mark.parametrize("K,N,B", [(16, 65536, 4096), (32, 200000, 8192), (2, 3000, 300)])
def test_buffer_wide_weights_in_the_fused_step_and_the_one_launch_forms(K, N, B):
    log(f"buffer-wide weights, fused K={K} N={N} B={B}")
    from paper_2311_09445_amd.per import OP_SAMPLE, OP_UPDATE
    rng = np.random.default_rng(K + N)
    T = 1
    m = Mirror(K, N, T, (16,))
    m.insert(N, prio=wl._draw_priorities("pareto_1.5", rng, (T, N)), chunk=50000)
    m.set_weight_norm("buffer")
    for it in range(4):                      # update batch = sampled batch (in place), apart, overlapping
        upd = wl._draw_updates("absnormal1_eps_pow0.6", rng, (T, B)) * np.float32(0.1 if it == 1 else 1.0)
        if it == 3:
            m.sample_gather_update(wl.uniform01(rng, (T, B)), 0.6, True, upd, tail=B // 3)
        else:
            m.sample_gather_update(wl.uniform01(rng, (T, B)), 0.6, True, upd, alias=(it % 2 == 0))
        m.compare_tree()
        m.compare_min_priority()
    if m.gpu.run_steps_fits():
        steps, Bs = 3, 64
        u = wl.uniform01(rng, (steps, T, Bs))
        beta = np.array([0.4, 0.7, 1.0], np.float32)
        upd = (rng.random((steps, T, Bs)) * np.float32(0.01)).astype(np.float32)
        oi = torch.empty((steps, T, Bs), dtype=torch.int32, device="cuda")
        ow = torch.empty((steps, T, Bs), dtype=torch.float32, device="cuda")
        m.gpu.run_steps(dev(u), dev(beta), oi, ow, upd_prio=dev(upd))
        for s_ in range(steps):
            ci, cw, cv = m.cpu.sample(u[s_], float(beta[s_]), True)
            assert np.array_equal(idx_to_host(oi)[s_], ci)
            np.testing.assert_allclose(ow.cpu().numpy()[s_], cw, rtol=1e-6, atol=0)
            m.cpu.update(ci, upd[s_])
        m.compare_min_priority()
        u2 = wl.uniform01(rng, (T, Bs))
        o2 = torch.empty((T, Bs), dtype=torch.int32, device="cuda")
        w2 = torch.empty((T, Bs), dtype=torch.float32, device="cuda")
        p2 = (rng.random((T, Bs)) * 2).astype(np.float32)
        keep = m.gpu.run_requests([{"op": OP_SAMPLE, "u": dev(u2), "beta": 0.5, "idx": o2, "out_weight": w2},
                                   {"op": OP_UPDATE, "prio": dev(p2)}])
        ci, cw, cv = m.cpu.sample(u2, 0.5, True)
        assert np.array_equal(idx_to_host(o2), ci)
        np.testing.assert_allclose(w2.cpu().numpy(), cw, rtol=1e-6, atol=0)
        m.cpu.update(ci, p2)
        del keep
        m.compare_tree()
        m.compare_min_priority()
    gi, ci = m.sample(wl.uniform01(rng, (T, 500)), beta=1.0)
    m.compare_status()


# ---------------------------------------------------------------------------------------------
# per_run_requests: a queue of op-coded requests in one launch.  Same results as the calls, in queue order.
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("K,N,T,fb,seed", [(2, 4096, 1, (16, 4, 4, 16, 1), 1), (16, 30000, 2, (12,), 2),
                                           (32, 32768, 1, (128,), 3), (4, 1000, 3, (), 4), (64, 20000, 1, (5, 68), 5),
                                           (16, 100000, 2, (12,), 6), (32, 700001, 1, (), 7)])   # (leaves in memory)
def test_run_requests_equals_the_separate_calls(K, N, T, fb, seed):
    """A random queue of insert (plain and collision-free), sample (+ weights, + rows) and update requests
    (given indices, or the batch sampled last).  The oracle gets every request as it is drawn, so later
    requests can refer to what earlier ones returned; the library gets the whole queue in one call."""
    from paper_2311_09445_amd.per import OP_INSERT, OP_SAMPLE, OP_UPDATE
    log(f"run_requests K={K} N={N} T={T} fb={fb}")
    rng = np.random.default_rng(seed)
    m = Mirror(K, N, T, fb)
    first = N - 300
    m.insert(first, prio=wl._draw_priorities("exponential_1", rng, (T, first)), chunk=max(5000, N // 8))   # the ring wraps below
    queue, checks = [], []
    sampled = None                  # indices of the latest sampling request (from the oracle)
    for r in range(40):
        kind = rng.choice(["insert", "protected", "sample", "update", "update_sampled"])
        if kind == "update_sampled" and sampled is None:
            kind = "sample"
        if kind in ("insert", "protected"):
            n = min(int(rng.choice([1, 7, 64, 333, 1024])), N)
            counters = m.counter + np.arange(n)
            m.counter += n
            rows = [np.stack([wl.row_bytes(t, counters, f, b) for t in range(T)]) for f, b in enumerate(fb)] \
                if fb and r % 5 else None
            prio = None
            if rng.random() < 0.5:
                prio = (rng.random((T, n)) * 5).astype(np.float32)
                if r % 3 == 0:
                    prio[:, 0] = np.float32("nan")
            protect = None
            if kind == "protected":   # the batch sampled last, or slots around the cursor
                protect = sampled if sampled is not None else \
                    ((m.cpu.trees[0].cursor + rng.integers(0, 2 * n, (T, 50))) % N).astype(np.uint32)
            out = torch.full((T, n), -7, dtype=torch.int32, device="cuda")
            queue.append({"op": OP_INSERT, "n": n, "prio": None if prio is None else dev(prio), "idx": out,
                          "rows": None if rows is None else [dev(x) for x in rows],
                          "protect": None if protect is None else idx_to_dev(protect)})
            checks.append(("slots", out, m.cpu.insert(n, rows, prio, protect=protect)))
        elif kind == "sample":
            B = int(rng.choice([1, 33, 256, 1000, 1024]))
            u = wl.uniform01(rng, (T, B))
            beta = float(rng.choice([0.0, 0.4, 1.0]))
            want_w = bool(r % 4)
            oi = torch.empty((T, B), dtype=torch.int32, device="cuda")
            ow = torch.empty((T, B), dtype=torch.float32, device="cuda") if want_w else None
            ov = torch.empty((T, B), dtype=torch.float32, device="cuda")
            rows_out = [torch.empty((T, B, b), dtype=torch.uint8, device="cuda") for b in fb] if fb and r % 3 else None
            queue.append({"op": OP_SAMPLE, "u": dev(u), "beta": beta, "idx": oi, "out_weight": ow, "out_prio": ov,
                          "rows": rows_out})
            ci, cw, cv = m.cpu.sample(u, beta, want_w)
            checks.append(("sample", oi, ow, ov, rows_out, ci, cw, cv, m.cpu.gather(ci) if rows_out else None))
            sampled = ci
        else:
            B = sampled.shape[1] if kind == "update_sampled" else int(rng.choice([1, 50, 700, 1024]))
            prio = (rng.random((T, B)) * 3).astype(np.float32)
            if r % 2:
                prio[:, ::11] = -1.0
            idx = None
            if kind == "update":
                idx = rng.integers(0, N, (T, B)).astype(np.uint32)
                idx[:, 1::2] = idx[:, 0::2][:, :idx[:, 1::2].shape[1]]     # every other element repeats its neighbour
                idx[:, 0] = N + 1                                          # out of range
            queue.append({"op": OP_UPDATE, "prio": dev(prio), "idx": None if idx is None else idx_to_dev(idx)})
            m.cpu.update(sampled if idx is None else idx, prio)
    keep = m.gpu.run_requests(queue)
    torch.cuda.synchronize()
    del keep
    for r, c in enumerate(checks):
        if c[0] == "slots":
            assert np.array_equal(idx_to_host(c[1]), c[2]), f"check {r}: slots reported by an insert request"
        else:
            _, oi, ow, ov, rows_out, ci, cw, cv, crow = c
            assert np.array_equal(idx_to_host(oi), ci), f"check {r}: sampled indices"
            assert ov.cpu().numpy().tobytes() == cv.tobytes(), f"check {r}: sampled values"
            if ow is not None:
                np.testing.assert_allclose(ow.cpu().numpy(), cw, rtol=1e-6, atol=0)
            if rows_out:
                for f, want in enumerate(crow):
                    assert np.array_equal(rows_out[f].cpu().numpy(), want), f"check {r}: rows of field {f}"
    m.compare_tree()
    m.compare_status()
    assert m.gpu.cursor == m.cpu.trees[0].cursor and m.gpu.size == m.cpu.trees[0].size
    # the separate calls carry on from the state the queue left
    m.update(rng.integers(0, N, (T, 50)).astype(np.uint32), rng.random((T, 50)).astype(np.float32))
    m.sample(wl.uniform01(rng, (T, 64)), 0.4)
    m.compare_tree()


def test_run_requests_argument_checks():
    from paper_2311_09445_amd.per import OP_SAMPLE, OP_UPDATE
    big = PrioritizedReplay(16, 1 << 20)
    z = torch.zeros((1, 8), device="cuda")
    zi = torch.zeros((1, 8), dtype=torch.int32, device="cuda")
    with pytest.raises(PerError) as e:
        big.run_requests([{"op": OP_SAMPLE, "u": z, "idx": zi}])
    assert e.value.code == ERANGE                                  # the tree does not fit
    p = PrioritizedReplay(4, 256)
    with pytest.raises(PerError) as e:
        p.run_requests([{"op": OP_SAMPLE, "u": z, "idx": zi}])
    assert e.value.code == EEMPTY
    p.insert(10, None, torch.ones((1, 10), device="cuda"))
    for bad in ([{"op": 9, "n": 1}], [{"op": OP_SAMPLE, "u": z, "idx": None}],
                [{"op": OP_UPDATE, "prio": z, "idx": None}],                       # no sampling request before it
                [{"op": OP_SAMPLE, "u": z, "idx": zi}, {"op": OP_UPDATE, "prio": torch.zeros((1, 4), device="cuda")}]):
        with pytest.raises(PerError) as e:
            p.run_requests(bad)
        assert e.value.code == EINVAL, bad
    with pytest.raises(PerError) as e:
        p.run_requests([{"op": OP_SAMPLE, "u": torch.zeros((1, 2000), device="cuda"),
                         "idx": torch.zeros((1, 2000), dtype=torch.int32, device="cuda")}])
    assert e.value.code == ERANGE
    assert p.size == 10 and p.cursor == 10                          # nothing was enqueued
    p.run_requests([])


@pytest.mark.parametrize("K,N,T,seed", [(16, 20000, 2, 1), (2, 3000, 1, 2), (32, 32768, 1, 3), (4, 25000, 3, 4)])
def test_interleaved_operations(K, N, T, seed):
    """Every entry point in random order on one buffer, the tree compared with the oracle after each call.  All
    values are small multiples of 2^-6, so every fp32 sum is exact and the delta-form update (which is
    order-dependent in general) stays bit-comparable too; what is tested here is the hand-over of state
    between the calls (stale top heights, stamps, dirty bits, ring position, LDS copy of the step kernel)."""
    from oracle.per_oracle import uniforms
    log(f"interleaved K={K} N={N} T={T} seed={seed}")
    rng = np.random.default_rng(seed)
    scale = np.float32(2.0 ** -6)
    top = max(8, (1 << 22) // N)

    def values(shape, lo=0):
        return (rng.integers(lo, top, shape) * scale).astype(np.float32)

    fb = (8, 3)
    m = Mirror(K, N, T, fb)
    m.insert(N - 50, prio=values((T, N - 50), 1), chunk=6000)
    m.gpu.set_rng(99)
    fits = m.gpu.run_steps_fits()
    ops = ["insert_small", "insert_large", "sample", "fused_own", "fused_other", "update", "delta", "rng", "retrieve"]
    if fits:
        ops.append("stream")
    for it in range(28):
        op = ops[int(rng.integers(0, len(ops)))]
        B = int(rng.choice([7, 64, 300, 1024]))
        if op == "insert_small":
            n = int(rng.integers(1, 40))
            m.insert(n, prio=None if it % 2 else values((T, n)))
        elif op == "insert_large":
            n = int(rng.integers(4097, 6000)) if N > 8000 else int(rng.integers(100, N // 2))
            m.insert(n, prio=values((T, n), 1))
        elif op == "sample":
            gi, ci = m.sample(wl.uniform01(rng, (T, B)), 0.5, fused_rows=bool(it % 2))
        elif op == "fused_own":
            m.sample_gather_update(wl.uniform01(rng, (T, B)), 0.5, True, values((T, B)), alias=True)
        elif op == "fused_other":
            gi, ci = m.sample(wl.uniform01(rng, (T, B)), 0.5)
            m.sample_gather_update(wl.uniform01(rng, (T, B)), 0.5, bool(it % 2), values((T, B)),
                                   dup={"dup_dst": np.stack([rng.integers(0, B, B // 4 + 1) for _ in range(T)]),
                                        "dup_src": np.stack([rng.integers(0, B, B // 4 + 1) for _ in range(T)])})
        elif op == "update":
            m.update(rng.integers(0, N, (T, B)).astype(np.uint32), values((T, B)))
        elif op == "delta":
            idx = np.stack([rng.choice(N, B, replace=False) for _ in range(T)]).astype(np.uint32)
            old = np.stack([o.get_priority(idx[t]) for t, o in enumerate(m.cpu.trees)])
            delta = values((T, B)) - old                      # exact: both are multiples of 2^-6
            m.gpu.update_delta(idx_to_dev(idx), dev(delta))
            m.cpu.update_delta(idx, delta)
        elif op == "rng":
            call = m.gpu.rng_calls()
            u = np.stack([uniforms(99, call, t, B) for t in range(T)])
            gi, _, gv = m.gpu.sample(None, 0.4, B=B, want_weights=False)
            ci, _, cv = m.cpu.sample(u, 0.4, False)
            assert np.array_equal(idx_to_host(gi), ci) and gv.cpu().numpy().tobytes() == cv.tobytes()
        elif op == "retrieve":
            idx = rng.integers(0, N, (T, B)).astype(np.uint32)
            got = m.gpu.get_priority(idx_to_dev(idx)).cpu().numpy()
            assert got.tobytes() == m.cpu.get_priority(idx).tobytes()
        elif op == "stream":
            steps, Bs = 3, min(B, 512)
            u = wl.uniform01(rng, (steps, T, Bs))
            up = values((steps, T, Bs))
            oi = torch.empty((steps, T, Bs), dtype=torch.int32, device="cuda")
            m.gpu.run_steps(dev(u), dev(np.full(steps, 0.4, np.float32)), oi, upd_prio=dev(up))
            for s in range(steps):
                ci, _, _ = m.cpu.sample(u[s], 0.4, False)
                assert np.array_equal(idx_to_host(oi[s]), ci), f"stream step {s}"
                m.cpu.update(ci, up[s])
        m.compare_tree()
    m.compare_status()


@pytest.mark.parametrize("K", [32, 2])
def test_largest_capacity(K):
    """N = 2^31 leaves per tree, the most the interface accepts (8 GiB of leaves, 16 GiB of stamps; with K = 2
    the deepest tree, 31 heights).  No oracle of that size: every leaf is 1 and later 1 + a multiple of 256,
    so every fp32 sum on the way to the root is exact and the results have closed forms (Eq. 1 on a
    uniform tree: sample i of B with u = 0.5 is leaf (i + 0.5) * N / B)."""
    N, B = 1 << 31, 4096
    log(f"largest capacity K={K}")
    p = PrioritizedReplay(K, N)
    chunk = 1 << 26
    ones = torch.ones((1, chunk), device="cuda")
    for _ in range(N // chunk):
        p.insert(chunk, None, ones)
    del ones
    assert p.size == N and p.cursor == 0
    assert float(p.total().cpu()[0]) == float(N)
    half = torch.full((1, B), 0.5, device="cuda")
    idx, w, v = p.sample(half, 0.4)
    want = (np.arange(B, dtype=np.int64) << 19) + (1 << 18)
    assert np.array_equal(idx_to_host(idx)[0].astype(np.int64), want)
    assert np.all(w.cpu().numpy() == 1.0) and np.all(v.cpu().numpy() == 1.0)
    # updates at both ends and in the middle; changes are multiples of 256, so the root stays exact
    ui = np.array([[0, 12345678, N - 1, (1 << 30) + 7, N - 1]], dtype=np.uint32)      # the last index twice: last writer
    uv = np.array([[257.0, 513.0, 99.0, 769.0, 1025.0]], dtype=np.float32)
    p.update(idx_to_dev(ui), dev(uv))
    assert float(p.total().cpu()[0]) == float(N) + 256 + 512 + 768 + 1024
    got = p.get_priority(idx_to_dev(ui)).cpu().numpy()[0]
    assert got.tolist() == [257.0, 513.0, 1025.0, 769.0, 1025.0]
    assert float(p.max_priority().cpu()[0]) == 1025.0
    changed = {0: 256, 12345678: 512, N - 1: 1024, (1 << 30) + 7: 768}               # leaf -> change of its value
    for h in (1, p.H - 1):                                                           # first and last node of two heights
        lvl = p.read_level(0, h).cpu().numpy()
        span = K ** h
        for node in (0, lvl.size - 1):
            extra = sum(d for leaf, d in changed.items() if leaf // span == node)
            assert float(lvl[node]) == float(span + extra), (h, node)
    # one whole step on the sampled batch itself with unchanged values: nothing may move
    out_idx = torch.empty((1, B), dtype=torch.int32, device="cuda")
    u = torch.rand((1, B), device="cuda")
    i2, w2, v2 = p.sample(u, 0.4, out_idx=out_idx)
    i3, w3, v3 = p.sample(u, 0.4, out_idx=out_idx, update=(out_idx, v2))
    assert torch.equal(i2.cpu(), i3.cpu()) and int(idx_to_host(i3).max()) < N
    assert float(p.total().cpu()[0]) == float(N) + 2560 and p.status() == 0


def test_large_batch():
    """A batch of 2^22 samples and updates on 2^24 leaves (64 times the headline batch): grids, job ranges and the
    stamp counter far from their usual sizes; element by element against the oracle."""
    K, N, B = 32, 1 << 24, 1 << 22
    log("large batch")
    rng = np.random.default_rng(77)
    m = Mirror(K, N, 1, ())
    m.insert(N, prio=wl._draw_priorities("pareto_1.5", rng, (1, N)), with_rows=False, chunk=1 << 22)
    gi, ci = m.sample(wl.uniform01(rng, (1, B)), 0.4)
    m.update(ci, rng.random((1, B)).astype(np.float32))
    m.compare_tree()
    m.sample_gather_update(wl.uniform01(rng, (1, B)), 0.7, True, rng.random((1, B)).astype(np.float32), alias=True)
    m.compare_tree()
    m.compare_status()


@pytest.mark.parametrize("K,N,T,fb", [(16, 5000, 2, (68, 24, 4, 68, 1)), (2, 300, 1, (5,)), (32, 40000, 1, ())])
def test_collision_free_insert(K, N, T, fb):
    """per_insert_protected: rows aimed at a slot of the protected batch are deferred (Section IV-B)."""
    log(f"protected insert K={K} N={N} T={T}")
    rng = np.random.default_rng(N + K)
    m = Mirror(K, N, T, fb)
    m.insert(N - 20, prio=wl._draw_priorities("exponential_1", rng, (T, N - 20)), chunk=3000)
    deferred_total = 0
    for it in range(6):
        gi, ci = m.sample(wl.uniform01(rng, (T, 200)), 0.4)            # the batch "in flight"
        n = int(rng.choice([3, 40, 250]))
        protect = ci.copy()
        if it % 2:                                                      # some that certainly collide, one out of range
            protect[:, :5] = (m.gpu.cursor + np.arange(5)) % N
            protect[:, 5] = N + 9
        counters = np.arange(m.counter, m.counter + n)
        rows_np = [np.stack([wl.row_bytes(t, counters, f, b) for t in range(T)]) for f, b in enumerate(fb)]
        prio = (rng.random((T, n)) * 3).astype(np.float32) if it % 3 == 0 else None
        out = torch.empty((T, n), dtype=torch.int32, device="cuda")
        m.gpu.insert(n, [dev(r) for r in rows_np] if fb else None, None if prio is None else dev(prio), out,
                     protect=idx_to_dev(protect))
        slots = m.cpu.insert(n, rows_np if fb else None, prio, protect)
        assert np.array_equal(idx_to_host(out), slots)
        deferred_total += int((slots == 0xFFFFFFFF).sum())
        m.counter += n
        m.compare_tree()
        if fb:                                                          # payload of the whole ring
            allidx = np.broadcast_to(np.arange(N, dtype=np.uint32), (T, N)).copy()
            want = m.cpu.gather(allidx)
            got = m.gpu.gather(idx_to_dev(allidx))
            for f in range(len(fb)):
                assert np.array_equal(got[f].cpu().numpy(), want[f]), f
        m.update(ci, rng.random((T, 200)).astype(np.float32))          # the batch comes back from the Learner
    assert deferred_total > 0
    m.compare_status()
    with pytest.raises(PerError) as e:                                  # the protected form is for small inserts
        big = PrioritizedReplay(16, 100000)
        big.insert(5000, None, None, None, protect=torch.zeros((1, 4), dtype=torch.int32, device="cuda"))
    assert e.value.code == ERANGE


@pytest.mark.parametrize("K,N", [(2, 3000), (16, 1 << 16)])
def test_fused_step_on_an_empty_total_that_the_update_fills(K, N):
    """Sampling finds a total of zero (weights 0, index 0xFFFFFFFF) while the update fused into the same call
    makes the tree non-zero: the weights job runs beside the tree pass and must not look at the new root."""
    log(f"fused step, zero total then filled K={K} N={N}")
    rng = np.random.default_rng(N)
    B = 3000                                                  # several sampling workgroups: weights finished by the job
    m = Mirror(K, N, 1, (4,))
    m.insert(N, prio=np.zeros((1, N), np.float32))
    upd_idx = rng.integers(0, N, (1, B)).astype(np.uint32)
    upd_prio = (rng.random((1, B)) + 0.5).astype(np.float32)
    u = wl.uniform01(rng, (1, B))
    rows = [torch.empty((1, B, 4), dtype=torch.uint8, device="cuda")]
    gi, gw, gv = m.gpu.sample(dev(u), 0.4, rows_out=rows, update=(idx_to_dev(upd_idx), dev(upd_prio)))
    ci, cw, cv = m.cpu.sample(u, 0.4, True)
    m.cpu.gather(ci)
    m.cpu.update(upd_idx, upd_prio)
    assert np.all(idx_to_host(gi) == 0xFFFFFFFF) and np.array_equal(idx_to_host(gi), ci)
    assert float(gw.abs().max()) == 0.0 and np.all(cw == 0.0)
    m.compare_tree()
    m.compare_status()
    m.step(wl.WORKLOADS["c3_ddpg"], 2, B=700)                 # and the next step samples the filled tree
    m.compare_tree()


# a seeded sweep of shapes beyond the hand-picked ones above
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("sweep_seed", [11, 12, 13])
def test_seeded_sweep_of_shapes(sweep_seed):
    """The operation-mix, interleaved, one-launch, placement and replay tests above at shapes drawn from a seeded
    generator: fanout, capacity (ragged, powers of two and their neighbours), tree count, batch and row layout."""
    r = np.random.default_rng(sweep_seed)
    layouts = [(), (5,), (12,), (128,), FIELDS, (68, 24, 4, 68, 1), (5, 68), (3, 8)]
    for case in range(24):
        K = int(r.choice([2, 4, 8, 16, 32, 64]))
        T = int(r.integers(1, 4))
        fb = layouts[int(r.integers(0, len(layouts)))]
        which = case % 6
        if which == 0:
            N = max(1, (1 << int(r.integers(1, 18))) + int(r.integers(-1, 2)))
            test_random_operation_mix(K, N, T)
        elif which == 1:
            test_buffer_wide_weights_through_an_operation_mix(K, int(r.integers(1, 200000)), T)
        elif which == 2:
            test_interleaved_operations(K, int(r.integers(1100, 300000)), T, int(r.integers(0, 1 << 30)))
        elif which == 3:
            N = int(r.integers(1100, 30000))
            if PrioritizedReplay(K, N, T, fb, 1.0).run_steps_fits():
                test_run_steps_equals_the_separate_calls(K, N, T, int(r.integers(1, 1025)), int(r.choice([0, 1, 4, 40])),
                                                         fb, bool(r.integers(0, 2)), bool(r.integers(0, 2)))
                test_run_requests_equals_the_separate_calls(K, N, T, fb, int(r.integers(0, 1 << 30)))
        elif which == 4:
            N = int(r.integers(5000, 300000))
            test_fused_step_wherever_the_update_batch_lies(K, N, min(N, int(r.integers(64, 20000))), fb)
        else:
            N = int(r.integers(4096, 300000))
            test_captured_step_replays(K, N, min(N, int(r.integers(64, 20000))))


@pytest.mark.parametrize("beta", [0.0, 0.01, 0.4, 1.0, 2.5, 3.0])
def test_weights_over_a_wide_range_of_ratios_and_exponents(beta):
    """Importance weights (Section II-A) where the ratio to the batch minimum spans twelve decades and beta goes
    beyond 1: the kernels' own fp64 evaluation of the power against the oracle's, within 1e-6 relative, in the
    separate call, in the one-workgroup form (small batch) and relative to the whole buffer."""
    log(f"weights beta={beta}")
    rng = np.random.default_rng(int(beta * 1000) + 5)
    K, N, T = 16, 6000, 2
    m = Mirror(K, N, T, ())
    m.insert(N, prio=(10.0 ** rng.uniform(-6, 6, (T, N))).astype(np.float32))
    for B in (3000, 40):
        m.sample(wl.uniform01(rng, (T, B)), beta=beta)
    m.set_weight_norm("buffer")
    for B in (3000, 40):
        m.sample(wl.uniform01(rng, (T, B)), beta=beta)
    m.compare_status()


@pytest.mark.parametrize("fb,shift", [((36, 100, 32), 4), ((68, 24, 4, 68, 1), 0), ((128,), 4), ((32, 20), 8), ((44,), 12)])
def test_rows_in_16_byte_pieces_on_4_byte_boundaries(fb, shift):
    """Fields whose size or address is a multiple of 4 bytes only are moved in 16-byte pieces, the last piece of
    a row overlapping the one before it.  Dense arrays that start `shift` bytes into their allocation, sizes just
    above and below the threshold, large and small batches (the scatter and gather kernels, the fused calls and
    the one-workgroup insert), every byte compared with the oracle's rows."""
    log(f"wide rows fb={fb} shift={shift}")
    rng = np.random.default_rng(sum(fb) + shift)
    K, N, T = 16, 20000, 2
    gpu = PrioritizedReplay(K, N, T, fb)
    cpu = MultiOracle(T, K, N, fb, 1.0)

    def shifted(shape_bytes):   # a uint8 device array of that many bytes starting `shift` bytes into its allocation
        return torch.empty(shape_bytes + shift, dtype=torch.uint8, device="cuda")[shift:]

    def insert(n):
        rows = [rng.integers(0, 256, (T, n, b), dtype=np.uint8) for b in fb]
        src = []
        for r in rows:
            d = shifted(r.size)
            d.copy_(torch.from_numpy(r.reshape(-1)).cuda())
            src.append(d)
        prio = (rng.random((T, n)) + 0.1).astype(np.float32)
        gpu.insert(n, src, dev(prio))
        cpu.insert(n, rows, prio)

    def check(idx):
        B = idx.shape[1]
        out = [shifted(T * B * b) for b in fb]
        for o in out:
            o.fill_(0xEE)
        gpu.gather(idx_to_dev(idx), out)
        want = cpu.gather(idx)
        for f, b in enumerate(fb):
            assert np.array_equal(out[f].cpu().numpy().reshape(T, B, b), want[f]), f"field {f}"

    insert(9000)                 # the scatter kernel
    insert(7)                    # the one-workgroup insert
    insert(N - 9007 + 300)       # wraps the ring
    check(rng.integers(0, N, (T, 5000)).astype(np.uint32))
    check(rng.integers(0, N, (T, 3)).astype(np.uint32))
    bad = rng.integers(0, N, (T, 70)).astype(np.uint32)
    bad[:, 5] = N + 1            # an index out of range gives a row of zeros
    check(bad)
    # fused sampling + gather into shifted arrays
    B = 3000
    u = wl.uniform01(rng, (T, B))
    out = [shifted(T * B * b) for b in fb]
    gi, _, _ = gpu.sample(dev(u), 0.4, rows_out=out)
    ci, _, _ = cpu.sample(u, 0.4, True)
    assert np.array_equal(idx_to_host(gi), ci)
    want = cpu.gather(ci)
    for f, b in enumerate(fb):
        assert np.array_equal(out[f].cpu().numpy().reshape(T, B, b), want[f]), f"fused field {f}"


@pytest.mark.parametrize("shift", [0, 4, 13])
@pytest.mark.parametrize("fb", [(68, 24, 4, 68, 1), (16, 4, 4, 1), (6, 2, 40, 8), (200, 8, 100, 3)])
def test_rows_gathered_whole(fb, shift):
    """Gathers of several fields that read each sampled row once and write every field's dense rows from a copy
    of the rows in LDS: dense arrays on 16-byte, 4-byte and odd boundaries, batches with a ragged last pass and
    shorter than one pass, a field left out, an index out of range, the stand-alone gather and the fused calls;
    every byte compared with the oracle's rows, and the form with one job per field run beside it."""
    log(f"whole rows fb={fb} shift={shift}")
    rng = np.random.default_rng(sum(fb) * 7 + shift)
    K, N, T = 16, 20000, 3
    gpu = PrioritizedReplay(K, N, T, fb)
    cpu = MultiOracle(T, K, N, fb, 1.0)

    def shifted(n_bytes, b):   # n_bytes of field size b, as far into an allocation as the field's alignment allows
        align = 16
        while b % align:
            align //= 2
        sh = shift - shift % align
        return torch.empty(n_bytes + sh, dtype=torch.uint8, device="cuda")[sh:]

    rows = [rng.integers(0, 256, (T, N, b), dtype=np.uint8) for b in fb]
    prio = (rng.random((T, N)) + 0.1).astype(np.float32)
    gpu.insert(N, [dev(r) for r in rows], dev(prio))
    cpu.insert(N, rows, prio)

    def check(idx, leave_out=None):
        B = idx.shape[1]
        want = cpu.gather(idx)
        for mode in (2, 0):
            gpu.set_tuning("whole_rows", mode)
            out = [None if f == leave_out else shifted(T * B * b, b) for f, b in enumerate(fb)]
            for o in out:
                if o is not None:
                    o.fill_(0xEE)
            gpu.gather(idx_to_dev(idx), out)
            for f, b in enumerate(fb):
                if out[f] is not None:
                    assert np.array_equal(out[f].cpu().numpy().reshape(T, B, b), want[f]), f"mode {mode} field {f}"

    check(rng.integers(0, N, (T, 5000)).astype(np.uint32))
    check(rng.integers(0, N, (T, 1001)).astype(np.uint32), leave_out=0)
    check(rng.integers(0, N, (T, 5)).astype(np.uint32), leave_out=len(fb) - 1)
    bad = rng.integers(0, N, (T, 70)).astype(np.uint32)
    bad[:, 5] = N + 1
    bad[1, 69] = 0xFFFFFFFF
    check(bad)
    assert gpu.status() != 0
    gpu.clear_status()
    gpu.set_tuning("whole_rows", 2)
    # fused: sampling + gather, then a whole step (sampling, gather and the update of the sampled batch)
    B = 3001
    u = wl.uniform01(rng, (T, B))
    out = [shifted(T * B * b, b) for b in fb]
    gi, _, _ = gpu.sample(dev(u), 0.4, rows_out=out)
    ci, _, _ = cpu.sample(u, 0.4, True)
    assert np.array_equal(idx_to_host(gi), ci)
    want = cpu.gather(ci)
    for f, b in enumerate(fb):
        assert np.array_equal(out[f].cpu().numpy().reshape(T, B, b), want[f]), f"fused field {f}"
    u = wl.uniform01(rng, (T, B))
    newp = (rng.random((T, B)) + 0.05).astype(np.float32)
    out = [shifted(T * B * b, b) for b in fb]
    gi, _, _ = gpu.step(dev(u), 0.4, dev(newp), None, rows_out=out)
    ci, _, _ = cpu.sample(u, 0.4, True)
    assert np.array_equal(idx_to_host(gi), ci)
    want = cpu.gather(ci)
    cpu.update(ci, newp)
    for f, b in enumerate(fb):
        assert np.array_equal(out[f].cpu().numpy().reshape(T, B, b), want[f]), f"step field {f}"
    u = wl.uniform01(rng, (T, 64))
    gi, _, _ = gpu.sample(dev(u), 0.4)
    ci, _, _ = cpu.sample(u, 0.4, True)
    assert np.array_equal(idx_to_host(gi), ci)
