"""Pins for the CPU oracle: it is checked against things other than itself.

Each test ties one part of ``oracle/`` to what the paper or the mathematics
fixes: the prefix-sum definition of sampling (Eq. 1) by brute force with exact
rational arithmetic, closed forms, the parent-equals-sum-of-children invariant
(Section V-A), textbook special cases, and a chi-square test of the sampling
distribution Pr(i) = P(i) / sum P (Section II-A).
"""
import os
from fractions import Fraction

import numpy as np
import pytest
from scipy import stats

from oracle.per_oracle import (FLAG_BAD_INDEX, FLAG_BAD_PRIORITY, FLAG_ZERO_TOTAL, Oracle)
from paper_2311_09445_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
KS = [2, 4, 8, 16, 32, 64]


def filled(K, leaves, fields=(), **kw):
    leaves = np.asarray(leaves, dtype=np.float32)
    o = Oracle(K, len(leaves), fields, **kw)
    o.insert(len(leaves), None, leaves)
    return o


def pairwise_f32(x):
    """Balanced pairwise fp32 sum over the last axis (length a power of two)."""
    x = np.asarray(x, dtype=np.float32)
    while x.shape[-1] > 1:
        x = (x[..., 0::2] + x[..., 1::2]).astype(np.float32)
    return x[..., 0]


def check_invariant(o):
    """Every stored node is the pairwise fp32 sum of its K children (zero padded)."""
    K = o.K
    lvl = o.read_level(0)
    for h in range(1, o.H + 1):
        up = o.read_level(h)
        pad = np.zeros(len(up) * K, dtype=np.float32)
        pad[:len(lvl)] = lvl
        want = pairwise_f32(pad.reshape(len(up), K))
        assert up.tobytes() == want.tobytes(), f"height {h}"
        lvl = up
    assert len(lvl) == 1 and lvl[0] == np.float32(o.total)


# ---------------------------------------------------------------- golden example
def _golden():
    d = {}
    with open(os.path.join(GOLDEN, "eq1_worked_example.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, *v = line.split()
            d[k] = [float(x) for x in v]
    return d


@pytest.mark.parametrize("K", [2, 4, 8])
def test_golden_worked_example(K):
    g = _golden()
    o = filled(K, g["leaves"])
    idx, w, v = o.sample(np.array(g["u"], np.float32), beta=g["beta"][0])
    assert idx.tolist() == [int(x) for x in g["idx"]]
    assert v.tolist() == g["prio"]
    np.testing.assert_allclose(w, g["weight"], rtol=1e-7)
    h = 1
    while f"k{K}_h{h}" in g:
        assert o.read_level(h).tolist() == g[f"k{K}_h{h}"]
        h += 1
    assert h - 1 == o.H


# ------------------------------------------------------------- brute force, exact
def brute_force_index(leaves, t):
    """min{i : prefix(i) > t} with exact rationals: the half-open reading of Eq. 1."""
    acc = Fraction(0)
    for i, p in enumerate(leaves):
        acc += Fraction(float(p))
        if acc > t:
            return i
    raise AssertionError("target beyond total")


@pytest.mark.parametrize("K", KS)
@pytest.mark.parametrize("N", [1, 2, 7, 33, 64, 100])
def test_bruteforce_prefix_search_exact(K, N):
    rng = np.random.default_rng(1000 * K + N)
    for trial in range(6):
        # small integers times a dyadic scale: every fp32 sum and difference is exact
        scale = 2.0 ** rng.integers(-3, 3)
        leaves = (rng.integers(0, 8, N) * (rng.random(N) < 0.7)).astype(np.float32) * np.float32(scale)
        if leaves.sum() == 0:
            leaves[rng.integers(N)] = np.float32(scale)
        o = filled(K, leaves)
        total = Fraction(float(leaves.astype(np.float64).sum()))
        assert Fraction(o.total) == total
        for B in (1, 4, 64):
            u = rng.integers(0, 64, B).astype(np.float32) / np.float32(64)
            idx, _, v = o.sample(u, want_weights=False)
            for i in range(B):
                t = (Fraction(i) + Fraction(float(u[i]))) * total / B
                assert idx[i] == brute_force_index(leaves, t), (K, N, B, i)
                assert v[i] == leaves[idx[i]] and v[i] > 0


@pytest.mark.parametrize("K", [2, 16])
@pytest.mark.parametrize("B", [3, 5, 7, 48])
def test_bruteforce_non_power_of_two_batch(K, B):
    """total/B is rounded once; the brute force takes the same fp32 target, then scans exactly."""
    rng = np.random.default_rng(B)
    leaves = rng.integers(0, 8, 50).astype(np.float32)
    leaves[0] = 1
    o = filled(K, leaves)
    u = rng.integers(0, 64, B).astype(np.float32) / np.float32(64)
    seg = np.float32(o.total) / np.float32(B)
    idx, _, _ = o.sample(u, want_weights=False)
    for i in range(B):
        t = (np.float32(i) + u[i]) * seg
        assert isinstance(t, np.float32)
        assert idx[i] == brute_force_index(leaves, Fraction(float(t)))


# ------------------------------------------------------ bracket on arbitrary floats
@pytest.mark.parametrize("K", KS)
@pytest.mark.parametrize("dist", ["uniform_1e-3_1", "lognormal_0_1", "exponential_1", "pareto_1.5"])
def test_bracket_against_fp64_prefix(K, dist):
    rng = np.random.default_rng(7)
    N, B = 5000, 512
    leaves = wl._draw_priorities(dist, rng, (N,))
    leaves[rng.random(N) < 0.05] = 0
    o = filled(K, leaves)
    u = wl.uniform01(rng, (B,))
    idx, _, v = o.sample(u, want_weights=False)
    prefix = np.concatenate([[0.0], np.cumsum(leaves.astype(np.float64))])
    total = np.float32(o.total)
    seg = total / np.float32(B)
    tol = 4 * o.HB * 2.0 ** -24 * float(total)
    for i in range(B):
        t = float((np.float32(i) + u[i]) * seg)
        assert prefix[idx[i]] - tol <= t <= prefix[idx[i] + 1] + tol
        assert v[i] == leaves[idx[i]] and v[i] > 0
    assert np.all(np.diff(idx.astype(np.int64)) >= 0)          # sorted targets -> sorted indices
    assert abs(float(total) - prefix[-1]) <= tol


# ------------------------------------------------------------------- closed forms
@pytest.mark.parametrize("K", KS)
def test_all_ones_closed_form(K):
    N = 4096
    o = filled(K, np.ones(N, np.float32))
    assert o.total == N
    rng = np.random.default_rng(3)
    for B in (64, 4096):
        u = wl.uniform01(rng, (B,))
        idx, w, v = o.sample(u, beta=0.7)
        pos = (np.arange(B, dtype=np.float32) + u).astype(np.float32)
        want = np.floor(pos.astype(np.float64) * (N / B)).astype(np.int64)
        assert np.array_equal(idx, want)
        assert np.all(w == 1.0) and np.all(v == 1.0)
    idx, _, _ = o.sample(np.full(N, 0.5, np.float32))
    assert np.array_equal(idx, np.arange(N))


@pytest.mark.parametrize("K", KS)
@pytest.mark.parametrize("where", [0, 1, 500, 998, 999])
def test_single_nonzero_leaf(K, where):
    leaves = np.zeros(1000, np.float32)
    leaves[where] = 0.37
    o = filled(K, leaves)
    u = wl.uniform01(np.random.default_rng(0), (128,))
    u[0], u[-1] = 0.0, np.float32(1 - 2.0 ** -24)
    idx, w, v = o.sample(u)
    assert np.all(idx == where) and np.all(v == np.float32(0.37)) and np.all(w == 1.0)


def test_zero_leaves_and_unfilled_slots_never_sampled():
    rng = np.random.default_rng(5)
    N = 3000
    o = Oracle(16, N)
    leaves = wl._draw_priorities("pareto_1.5", rng, (2000,))
    leaves[rng.random(2000) < 0.3] = 0
    leaves[-1] = 0.0
    o.insert(2000, None, leaves)
    assert o.size == 2000
    for _ in range(20):
        idx, _, v = o.sample(wl.uniform01(rng, (256,)))
        assert np.all(idx < 2000) and np.all(leaves[idx] > 0) and np.all(v == leaves[idx])


def test_target_inside_its_stratum():
    """Sample i draws from stratum i: with B = number of equal-mass blocks, sample i lands in block i."""
    K, blocks, per = 4, 16, 8
    rng = np.random.default_rng(11)
    leaves = np.zeros(blocks * per, np.float32)
    for b in range(blocks):                       # each block holds mass exactly 8 spread unevenly
        cuts = np.sort(rng.choice(np.arange(1, 8), 3, replace=False))
        parts = np.diff(np.concatenate([[0], cuts, [8]]))
        leaves[b * per + rng.choice(per, 4, replace=False)] = parts
    o = filled(K, leaves)
    for _ in range(10):
        idx, _, _ = o.sample(wl.uniform01(rng, (blocks,)))
        assert np.array_equal(idx // per, np.arange(blocks))


# ------------------------------------------------------------ tree values / update
@pytest.mark.parametrize("K", KS)
@pytest.mark.parametrize("N", [1, 5, 64, 1000, 4097])
def test_invariant_after_insert_and_update(K, N):
    rng = np.random.default_rng(K * 31 + N)
    leaves = wl._draw_priorities("lognormal_0_1", rng, (N,))
    o = filled(K, leaves)
    check_invariant(o)
    assert np.array_equal(o.read_level(0), leaves)
    for _ in range(5):
        B = 97
        idx = rng.integers(0, N, B).astype(np.uint32)
        pr = wl._draw_updates("absnormal1_eps_pow0.6", rng, (B,))
        o.update(idx, pr)
        for j in range(B):                         # plain sequential semantics on a flat array
            leaves[idx[j]] = pr[j]
        check_invariant(o)
        assert np.array_equal(o.read_level(0), leaves)
    # equals a from-scratch build of the final leaves, and an idempotent update changes no bit
    fresh = filled(K, leaves)
    for h in range(o.H + 1):
        assert o.read_level(h).tobytes() == fresh.read_level(h).tobytes()
    before = [o.read_level(h).tobytes() for h in range(o.H + 1)]
    all_idx = np.arange(N, dtype=np.uint32)
    o.update(all_idx, leaves)
    assert before == [o.read_level(h).tobytes() for h in range(o.H + 1)]


def test_root_is_exact_total_for_dyadic_leaves():
    rng = np.random.default_rng(2)
    leaves = (rng.integers(0, 1024, 3000) / 64.0).astype(np.float32)
    for K in KS:
        o = filled(K, leaves)
        assert Fraction(o.total) == sum(Fraction(float(x)) for x in leaves)
        # a K-group's parent is the exact sum of its K children
        lvl1 = o.read_level(1)
        for j in (0, len(lvl1) // 2, len(lvl1) - 1):
            assert Fraction(float(lvl1[j])) == sum(Fraction(float(x)) for x in leaves[j * K:(j + 1) * K])


def test_last_writer_wins_on_duplicates():
    rng = np.random.default_rng(9)
    N = 257
    o = filled(8, np.ones(N, np.float32))
    shadow = np.ones(N, np.float32)
    batches = [
        (np.full(64, 5, np.uint32), rng.random(64).astype(np.float32)),                 # all equal
        (np.tile(np.array([3, 200], np.uint32), 50), rng.random(100).astype(np.float32)),  # alternating
        (rng.integers(0, 16, 300).astype(np.uint32), rng.random(300).astype(np.float32)),
    ]
    for idx, pr in batches:
        o.update(idx, pr)
        last = {}
        for j, i in enumerate(idx):
            last[int(i)] = pr[j]
        for i, v in last.items():
            shadow[i] = v
        assert np.array_equal(o.read_level(0), shadow)
        check_invariant(o)


def test_k_invariance_reduces_every_fanout_to_the_binary_tree():
    """Same leaves, same uniforms: identical indices, and identical sums wherever binary depths coincide."""
    rng = np.random.default_rng(4)
    N = 4096
    leaves = wl._draw_priorities("exponential_1", rng, (N,))
    leaves[rng.random(N) < 0.1] = 0
    u = wl.uniform01(rng, (1024,))
    ref = filled(2, leaves)                         # K = 2 is the textbook binary sum tree
    ridx, rw, rv = ref.sample(u, beta=0.5)
    for K in KS[1:]:
        o = filled(K, leaves)
        idx, w, v = o.sample(u, beta=0.5)
        assert np.array_equal(idx, ridx) and np.array_equal(v, rv) and np.array_equal(w, rw)
        shift = o.HB - ref.HB                      # extra all-zero-right levels above the real root
        assert shift >= 0
        for h in range(o.H + 1):
            d = o.HB - h * (o.K.bit_length() - 1)  # binary depth of K-ary height h
            if d - shift < 0:
                continue
            mine = o.read_level(h)
            theirs = ref.read_binary_depth(d - shift)[:len(mine)]
            assert mine.tobytes() == theirs.tobytes()
        assert o.total == ref.total


def test_denormals_and_negative_zero():
    tiny = np.float32(1e-42)                        # subnormal
    leaves = np.array([0.0, -0.0, tiny, 0.0, tiny, -0.0, tiny, tiny], np.float32)
    for K in (2, 4, 8):
        o = filled(K, leaves)
        assert o.total == np.float32(4) * tiny and o.total > 0
        assert o.status == 0                        # -0.0 is a valid priority
        idx, w, v = o.sample(np.array([0.0, 0.5, 0.5, 0.99], np.float32))
        assert idx.tolist() == [2, 4, 6, 7] and np.all(v == tiny) and np.all(w == 1.0)


# -------------------------------------------------------------------- distribution
def test_sampling_frequency_is_proportional_to_priority():
    rng = np.random.default_rng(12345)
    N, B, steps = 256, 64, 2000
    leaves = td = wl.td_to_priority(rng.standard_normal(N), 1e-6, 0.6)
    o = filled(16, leaves)
    counts = np.zeros(N)
    for _ in range(steps):
        idx, _, _ = o.sample(wl.uniform01(rng, (B,)), want_weights=False)
        np.add.at(counts, idx, 1)
    expect = B * steps * td.astype(np.float64) / td.astype(np.float64).sum()
    x2 = float(((counts - expect) ** 2 / expect).sum())
    assert x2 < stats.chi2.ppf(0.9999, N - 1)
    # and the test has teeth: the same counts are rejected against a uniform law
    flat = np.full(N, B * steps / N)
    assert float(((counts - flat) ** 2 / flat).sum()) > stats.chi2.ppf(0.9999, N - 1)


# ------------------------------------------------------------- importance weights
def test_importance_weights():
    rng = np.random.default_rng(8)
    N = 2000
    leaves = wl._draw_priorities("lognormal_0_1", rng, (N,))
    o = Oracle(16, 3000)
    o.insert(N, None, leaves)
    u = wl.uniform01(rng, (256,))
    for beta in (0.0, 0.4, 1.0):
        idx, w, v = o.sample(u, beta=beta)
        assert w.max() == 1.0 and np.all(w > 0) and np.all(w <= 1)
        if beta == 0.0:
            assert np.all(w == 1.0)
        # definition: w_i = (size * P(i))^-beta / max_j(...), P(i) = v_i / total; size = filled rows
        P = v.astype(np.float64) / float(np.float32(o.total))
        raw = (N * P) ** (-beta)
        np.testing.assert_allclose(w, raw / raw.max(), rtol=2e-7)
        i, j = 3, 200
        np.testing.assert_allclose(w[i] / w[j], (float(v[j]) / float(v[i])) ** beta, rtol=1e-6)
    o2 = filled(4, np.full(64, 0.25, np.float32))
    assert np.all(o2.sample(u[:32], beta=0.9)[1] == 1.0)


def test_importance_weights_relative_to_the_whole_buffer():
    """Closed forms: with beta = 1 the weight of a row is (smallest positive priority of the buffer) / (its own),
    whatever else was sampled; rows with priority 0 and unfilled slots do not count; a batch that happens to
    hold the smallest row gets the batch-relative weights; equal priorities give weights of one."""
    o = Oracle(2, 16)
    o.insert(6, None, np.array([4.0, 0.0, 1.0, 8.0, 2.0, 16.0], np.float32))    # total 31, smallest positive 1
    o.set_weight_norm("buffer")
    B = 31                                                                       # one target per unit of priority
    idx, w, v = o.sample(np.full(B, 0.5, np.float32), beta=1.0)
    assert sorted(set(idx.tolist())) == [0, 2, 3, 4, 5]
    np.testing.assert_allclose(w, 1.0 / v, rtol=2e-7)
    upper = np.array([0.99], np.float32)                                         # a batch of one: the last row only
    idx, w, v = o.sample(upper, beta=1.0)
    assert idx.tolist() == [5] and abs(float(w[0]) - 1.0 / 16.0) < 1e-8
    idx, w, v = o.sample(upper, beta=0.5)
    assert abs(float(w[0]) - 0.25) < 1e-7
    o.set_weight_norm("batch")
    assert o.sample(upper, beta=1.0)[1].tolist() == [1.0]
    # against the definition written out with numpy: every stored row's weight, then the maximum
    rng = np.random.default_rng(18)
    N = 3000
    leaves = wl._draw_priorities("pareto_1.5", rng, (N,))
    leaves[rng.integers(0, N, 30)] = 0.0
    o = Oracle(16, 5000)
    o.insert(N, None, leaves)
    o.set_weight_norm("buffer")
    u = wl.uniform01(rng, (300,))
    for beta in (0.0, 0.4, 1.0):
        idx, w, v = o.sample(u, beta=beta)
        total = float(np.float32(o.total))
        every = (N * leaves[leaves > 0].astype(np.float64) / total) ** (-beta)
        np.testing.assert_allclose(w, (N * v.astype(np.float64) / total) ** (-beta) / every.max(), rtol=2e-7)
        assert np.all(w <= 1.0) and np.all(w > 0)
        o.set_weight_norm("batch")
        wb = o.sample(u, beta=beta)[1]
        o.set_weight_norm("buffer")
        ratio = (float(leaves[leaves > 0].min()) / float(v.min())) ** beta       # buffer-wide = batch-relative * this
        np.testing.assert_allclose(w, wb * ratio, rtol=3e-7)
    # updates move the minimum
    o.update(np.array([int(np.argmin(np.where(leaves > 0, leaves, np.inf)))], np.uint32), np.array([1e-3], np.float32))
    idx, w, v = o.sample(u, beta=1.0)
    np.testing.assert_allclose(w, 1e-3 / v.astype(np.float64), rtol=2e-7)
    o2 = filled(4, np.full(64, 0.25, np.float32))
    o2.set_weight_norm("buffer")
    assert np.all(o2.sample(u[:32], beta=0.9)[1] == 1.0)


# ----------------------------------------------------------- insert / ring / gather
def test_ring_insert_gather_and_max_priority():
    w = wl.WORKLOADS["c1_binary_small"]
    N, fb = 50, w.field_bytes
    o = Oracle(4, N, fb, init_max=1.0)
    counter = 0

    def rows(n):
        nonlocal counter
        c = np.arange(counter, counter + n)
        counter += n
        return [wl.row_bytes(0, c, f, b) for f, b in enumerate(fb)]

    slots = o.insert(30, rows(30))
    assert slots.tolist() == list(range(30)) and o.size == 30 and o.cursor == 30
    assert np.all(o.read_level(0)[:30] == 1.0) and np.all(o.read_level(0)[30:] == 0.0)
    o.update(np.array([3, 4], np.uint32), np.array([2.5, 0.5], np.float32))
    assert o.max_priority == 2.5
    slots = o.insert(30, rows(30))                  # wraps: slots 30..49 then 0..9
    assert slots.tolist() == list(range(30, 50)) + list(range(10))
    assert o.size == N and o.cursor == 10
    lv = o.read_level(0)
    assert np.all(lv[:10] == 2.5) and lv[10] == 1.0 and np.all(lv[30:] == 2.5)
    check_invariant(o)
    # slot s holds the row with the largest insert counter that mapped to it
    holder = {}
    for c in range(60):
        holder[c % N] = c
    idx = np.array([0, 9, 10, 29, 30, 49, 7, 7], np.uint32)
    got = o.gather(idx)
    for f, b in enumerate(fb):
        want = wl.row_bytes(0, [holder[int(i)] for i in idx], f, b)
        assert np.array_equal(got[f], want)
    # explicit priorities raise the running max only after the call; invalid ones are skipped
    o.insert(3, rows(3), np.array([7.0, np.nan, -1.0], np.float32))
    assert o.max_priority == 7.0 and o.status == FLAG_BAD_PRIORITY
    lv = o.read_level(0)
    assert lv[10] == 7.0 and lv[11] == 1.0 and lv[12] == 1.0
    with pytest.raises(ValueError):
        o.insert(N + 1)


def test_status_flags_and_skips():
    o = Oracle(2, 16, (4,))
    idx, w, v = o.sample(np.zeros(4, np.float32))
    assert np.all(idx == 0xFFFFFFFF) and np.all(w == 0) and o.status == FLAG_ZERO_TOTAL
    o.clear_status()
    o.insert(8, None, np.ones(8, np.float32))
    o.update(np.array([1, 8, 2, 3, 4], np.uint32), np.array([2, 2, np.inf, -1, np.nan], np.float32))
    assert o.status == FLAG_BAD_INDEX | FLAG_BAD_PRIORITY
    assert o.read_level(0).tolist() == [1, 2, 1, 1, 1, 1, 1, 1] + [0] * 8
    assert o.max_priority == 2.0
    o.clear_status()
    g = o.gather(np.array([0, 16, 0xFFFFFFFF], np.uint32))
    assert np.all(g[0][1:] == 0) and o.status == FLAG_BAD_INDEX
    assert o.get_priority(np.array([1, 99], np.uint32)).tolist() == [2.0, 0.0]


def test_level_shapes_follow_ceil_division():
    for K, N in [(32, 1 << 14), (16, 1 << 10), (16, 10000), (2, 4096), (32, 33)]:
        o = Oracle(K, N, with_payload=False)
        n, h = N, 0
        while True:
            assert o.level_count(h) == n
            if n == 1 and h >= 1:
                break
            n = -(-n // K)
            h += 1
        assert o.H == h


# ---------------------------------------------------------------------------------------------
# The multi-threaded CPU baseline (oracle/per_workers.c) must be the oracle, bit for bit.
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("K,N,B", [(2, 1000, 257), (16, 70001, 4096), (32, 1 << 16, 20000), (64, 5000, 33)])
def test_worker_threads_reproduce_the_oracle(K, N, B):
    from oracle.per_workers import Workers
    rng = np.random.default_rng(K * 1000 + B)
    fb = (12, 1)
    leaves = rng.pareto(1.5, N).astype(np.float32)
    leaves[rng.random(N) < 0.01] = 0.0
    a, b = Oracle(K, N, fb), Oracle(K, N, fb)
    rows = [rng.integers(0, 256, (N, e), dtype=np.uint8) for e in fb]
    for o in (a, b):
        o.insert(N, rows, leaves)
    wk = Workers(b, threads=5)
    for step in range(4):
        u = (rng.integers(0, 1 << 24, B).astype(np.float32) / np.float32(1 << 24)).astype(np.float32)
        ia, wa, va = a.sample(u, 0.6)
        ib, wb, vb = wk.sample(u, 0.6)
        assert np.array_equal(ia, ib) and va.tobytes() == vb.tobytes() and wa.tobytes() == wb.tobytes()
        for ra, rb in zip(a.gather(ia), wk.gather(ib)):
            assert np.array_equal(ra, rb)
        # update batch: the sampled indices, some slots repeated out of order, some invalid elements
        idx = ia.copy()
        dst = rng.integers(0, B, B // 5)
        idx[dst] = ia[rng.integers(0, B, B // 5)]
        prio = rng.random(B).astype(np.float32)
        if step == 1:
            rng.shuffle(idx)                     # an unsorted batch
        if step == 2:
            prio[::7] = np.float32("nan")
            prio[3::11] = -1.0
            idx[5::13] = N + 3                   # out of range
        a.update(idx, prio)
        wk.update(idx, prio)
        for d in range(a.HB + 1):
            assert a.read_binary_depth(d).tobytes() == b.read_binary_depth(d).tobytes(), (step, d)
        assert a.max_priority == b.max_priority and a.status == b.status


# ---------------------------------------------------------------------------------------------
# Priority update in the paper's own form (Section V-A): add delta to every node from the root down
# to the leaf.  Pinned by exact arithmetic (dyadic values: every fp32 sum is exact, so every node must
# be the exact sum of the leaves below it and the result must coincide with the set form), by the
# additivity of duplicates, by an fp64 bound on arbitrary floats, and by its validity rules.
# ---------------------------------------------------------------------------------------------
def _exact_level(leaves_int, K, N, h):
    """Sums of integer leaves per K-ary node of height h, by plain integer arithmetic."""
    n = N
    for _ in range(h):
        n = -(-n // K)
    span = K ** h
    pad = np.zeros(n * span, dtype=np.int64)
    pad[:N] = leaves_int
    return pad.reshape(n, span).sum(axis=1)


@pytest.mark.parametrize("K,N", [(2, 37), (4, 1000), (16, 4097), (32, 70000), (64, 300)])
def test_delta_update_on_dyadic_values_is_exact_and_equals_the_set_form(K, N):
    rng = np.random.default_rng(K + N)
    scale = np.float32(2.0 ** -6)
    top = max(2, min(1 << 10, (1 << 23) // N))        # every partial sum stays below 2^24 units: exact in fp32
    leaves_int = rng.integers(0, top, N)
    a, b = Oracle(K, N), Oracle(K, N)
    for o in (a, b):
        o.insert(N, None, (leaves_int * scale).astype(np.float32))
    for _ in range(3):
        B = 500
        idx = rng.choice(N, size=min(B, N), replace=False).astype(np.uint32)       # distinct indices
        new_int = rng.integers(0, top, idx.size)
        old = a.get_priority(idx)
        delta = (new_int * scale).astype(np.float32) - old                         # retrieval, then the change
        a.update_delta(idx, delta)
        b.update(idx, (new_int * scale).astype(np.float32))
        leaves_int[idx] = new_int
        for h in range(a.H + 1):
            want = (_exact_level(leaves_int, K, N, h) * float(scale)).astype(np.float32)
            assert a.read_level(h).tobytes() == want.tobytes(), h
            assert a.read_level(h).tobytes() == b.read_level(h).tobytes(), h
    assert a.status == 0


def test_delta_update_duplicates_add_up_and_invalid_elements_are_skipped():
    K, N = 8, 100
    o = Oracle(K, N)
    o.insert(60, None, np.full(60, 2.0, np.float32))          # size 60 of capacity 100
    before = [o.read_level(h).copy() for h in range(o.H + 1)]
    o.update_delta(np.array([5, 5, 5, 70, 7, 8], np.uint32),
                   np.array([0.5, 0.25, -1.0, 1.0, np.nan, np.inf], np.float32))
    assert o.status == FLAG_BAD_INDEX | FLAG_BAD_PRIORITY
    leaf = o.read_level(0)
    assert leaf[5] == np.float32(1.75) and leaf[7] == 2.0 and leaf[8] == 2.0 and leaf[70] == 0.0
    for h in range(1, o.H + 1):                               # only the ancestors of leaf 5 moved, by -0.25
        d = o.read_level(h) - before[h]
        assert d[5 // K ** h] == np.float32(-0.25) and np.count_nonzero(d) == 1, h
    assert o.max_priority == 2.0                              # the running maximum never sees a change


@pytest.mark.parametrize("K,N", [(16, 5000), (2, 777)])
def test_delta_update_stays_within_the_rounding_bound_of_the_true_sums(K, N):
    rng = np.random.default_rng(N)
    o = Oracle(K, N)
    leaves = rng.exponential(1.0, N).astype(np.float32)
    o.insert(N, None, leaves)
    truth = leaves.astype(np.float64)
    steps, B = 20, 300
    for _ in range(steps):
        idx = rng.integers(0, N, B).astype(np.uint32)
        delta = (rng.standard_normal(B) * 0.1).astype(np.float32)
        o.update_delta(idx, delta)
        np.add.at(truth, idx, delta.astype(np.float64))
    for h in range(o.H + 1):
        n = o.level_count(h)
        pad = np.zeros(n * K ** h)
        pad[:N] = truth
        want = pad.reshape(n, K ** h).sum(axis=1)
        mag = np.zeros(n * K ** h)
        mag[:N] = np.abs(leaves.astype(np.float64)) + 0.1 * 4 * steps
        bound = 2.0 ** -23 * (o.HB + steps * B) * mag.reshape(n, K ** h).sum(axis=1)
        assert np.all(np.abs(o.read_level(h).astype(np.float64) - want) <= bound), h


# ---------------------------------------------------------------------------------------------
# Update from temporal-difference errors: value = (|td| + eps)^alpha.  Pinned by closed forms
# (alpha = 1, alpha = 0, exact squares with alpha = 0.5, td = 0) and by an independent evaluation
# of the power (numpy's, in fp64) within one fp32 rounding; the tree below is the set form's.
# ---------------------------------------------------------------------------------------------
def test_td_update_closed_forms_and_validity():
    N = 64
    o = Oracle(4, N)
    o.insert(N, None, np.ones(N, np.float32))
    idx = np.arange(8, dtype=np.uint32)
    td = np.array([-3.0, 0.25, 0.0, 16.0, -9.0, np.nan, np.inf, 2.0], np.float32)
    o.update_td(idx, td, 0.0, 1.0)                       # alpha = 1, eps = 0: |td|
    assert o.read_level(0)[:5].tolist() == [3.0, 0.25, 0.0, 16.0, 9.0]
    assert o.read_level(0)[5] == 1.0 and o.read_level(0)[6] == 1.0 and o.status == FLAG_BAD_PRIORITY
    assert o.max_priority == 16.0
    o.update_td(idx[:5], td[:5], 0.0, 0.5)               # exact squares
    assert o.read_level(0)[[3, 4]].tolist() == [4.0, 3.0]
    o.update_td(idx[:5], td[:5], 0.5, 0.0)               # alpha = 0: 1 everywhere
    assert o.read_level(0)[:5].tolist() == [1.0] * 5
    o.update_td(np.array([2, 70], np.uint32), np.array([0.0, 1.0], np.float32), 1e-6, 0.6)   # td = 0: eps^alpha
    assert abs(float(o.read_level(0)[2]) - (1e-6) ** 0.6) <= 1e-7 * (1e-6) ** 0.6
    assert o.status == FLAG_BAD_PRIORITY | FLAG_BAD_INDEX
    ref = Oracle(4, N)                                   # the tree is the set form's for the same leaf values
    ref.insert(N, None, o.read_level(0).copy())
    for h in range(o.H + 1):
        assert o.read_level(h).tobytes() == ref.read_level(h).tobytes()


def test_td_update_matches_an_independent_power_within_one_rounding():
    rng = np.random.default_rng(11)
    N, B = 5000, 3000
    o = Oracle(16, N)
    o.insert(N, None, np.ones(N, np.float32))
    idx = rng.choice(N, B, replace=False).astype(np.uint32)
    td = (rng.standard_normal(B) * 3).astype(np.float32)
    o.update_td(idx, td, 1e-6, 0.6)
    want = np.power(np.abs(td.astype(np.float64)) + 1e-6, 0.6)
    got = o.read_level(0)[idx].astype(np.float64)
    assert np.all(np.abs(got - want) <= 2.0 ** -23 * want)


# ---------------------------------------------------------------------------------------------
# Counter-based uniforms (Philox4x32-10): pinned by the generator's published known-answer vectors,
# by the [0,1) range and 2^-24 grid of the uniforms, and by a chi-square test of their distribution.
# ---------------------------------------------------------------------------------------------
def test_philox_known_answers():
    from oracle.per_oracle import philox4x32_10
    path = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        w = [int(x, 16) for x in r]
        assert philox4x32_10(w[0:4], w[4:6]).tolist() == w[6:10]


def test_counter_based_uniforms():
    from oracle.per_oracle import philox4x32_10, uniforms
    u = uniforms(seed=0x123456789ABCDEF0, call=(7 << 32) | 5, tree=3, B=50000)
    assert u.dtype == np.float32 and u.min() >= 0.0 and u.max() < 1.0
    assert np.all(u * 16777216.0 == np.floor(u * 16777216.0))                 # on the 2^-24 grid
    x = philox4x32_10([12345, 5, 7, 3], [0x9ABCDEF0, 0x12345678])             # counter (i, call lo, call hi, tree)
    assert u[12345] == np.float32(x[0] >> 8) * np.float32(2.0 ** -24)
    counts = np.bincount((u * 64).astype(int), minlength=64)
    assert float(((counts - 50000 / 64) ** 2 / (50000 / 64)).sum()) < stats.chi2.ppf(0.9999, 63)
    assert not np.array_equal(u, uniforms(0x123456789ABCDEF0, (7 << 32) | 6, 3, 50000))   # next call: new stream
    assert not np.array_equal(u, uniforms(0x123456789ABCDEF0, (7 << 32) | 5, 4, 50000))   # other tree


# ---------------------------------------------------------------------------------------------
# Collision-free insertion (Section IV-B): slots named by the protected batch keep their rows and
# priorities; the rows aimed at them are reported as deferred; everything else as a plain insert.
# Pinned against a dictionary model of the ring.
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("K,N", [(4, 50), (16, 1000)])
def test_protected_insert_against_a_ring_model(K, N):
    rng = np.random.default_rng(N)
    fb = (3,)
    o = Oracle(K, N, fb)
    model_rows, model_prio = {}, {}
    cursor, size, counter, maxv = 0, 0, 0, 1.0
    for it in range(12):
        n = int(rng.integers(1, N // 2))
        protect = rng.integers(0, N + 3, int(rng.integers(0, 20))).astype(np.uint32) if it % 3 else None
        rows = rng.integers(0, 256, (n, 3), dtype=np.uint8)
        prio = (rng.random(n) * 5).astype(np.float32) if it % 2 else None
        out = o.insert(n, [rows], prio, protect)
        entry_max = maxv
        for j in range(n):
            slot = (cursor + j) % N
            if protect is not None and slot in set(protect.tolist()):
                assert out[j] == 0xFFFFFFFF
                continue
            assert out[j] == slot
            model_rows[slot] = rows[j].copy()
            model_prio[slot] = float(prio[j]) if prio is not None else entry_max
            if prio is not None:
                maxv = max(maxv, float(prio[j]))
        cursor, size = (cursor + n) % N, min(N, size + n)
        assert o.cursor == cursor and o.size == size and o.max_priority == np.float32(maxv)
        leaves = o.read_level(0)
        for slot in range(N):
            assert leaves[slot] == np.float32(model_prio.get(slot, 0.0)), (it, slot)
        got = o.gather(np.arange(N, dtype=np.uint32))[0]
        for slot, r in model_rows.items():
            assert np.array_equal(got[slot], r)
        ref = Oracle(K, N)                       # ancestors: the set form of the same leaves
        ref.insert(N, None, leaves.copy())
        for h in range(o.H + 1):
            assert o.read_level(h).tobytes() == ref.read_level(h).tobytes()
