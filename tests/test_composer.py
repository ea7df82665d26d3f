"""The System Composer calculator (Section VI: Eq. 4-7, Algorithm 1) against values worked out by hand,
brute force over all assignments, and limiting cases."""
import itertools
import json

import pytest

from paper_2311_09445_amd.composer import (DeviceRow, Link, Platform, Workload, fpga_learner, fpga_rm_sampling,
                                           fpga_rm_update_or_insert, rm_latencies_from_bench)

US = 1e-6


def platform(shared=None):
    rows = {"cpu": DeviceRow(100 * US, 80 * US, 50 * US, learner=1000 * US, rm_power=100.0, learner_power=150.0),
            "gpu": DeviceRow(20 * US, 15 * US, 10 * US, learner=200 * US, rm_power=300.0, learner_power=400.0,
                             shared=shared or {})}
    links = {("cpu", "gpu"): Link(10 * US, 1e9), ("cpu", "cpu"): Link(0.0, 1e10), ("gpu", "gpu"): Link(0.0, 1e12)}
    return Platform(rows, links)


W = Workload(BS=256, E=10, n_actor=64)


def test_fpga_pipeline_models():
    # Eq. 4: 2 F (BS + D) cycles; Eq. 5: 2 (BS + D); Eq. 6: T_stage (BS + 3 (layers - 1))
    assert fpga_rm_sampling(F=4, BS=32, D=5, clock_hz=250e6) == pytest.approx(296 / 250e6)
    assert fpga_rm_sampling(4, 32, 5, 250e6, t_comm=3e-6) == pytest.approx(296 / 250e6 + 3e-6)
    assert fpga_rm_update_or_insert(BS=32, D=5, clock_hz=250e6) == pytest.approx(74 / 250e6)
    assert fpga_learner(t_stage=2e-6, BS=64, n_layers=3) == pytest.approx(2e-6 * 70)
    # sampling costs F times an update at equal communication
    assert fpga_rm_sampling(16, 100, 7, 1e8) == pytest.approx(16 * fpga_rm_update_or_insert(100, 7, 1e8))


def test_iteration_time_by_hand():
    p = platform()
    idx = 256 * 4
    # RM and Learner on the GPU: indices and priorities stay in device memory, insertions come over the link
    t = 20 * US + idx / 1e12 + max(10 * US + (10 * US + 64 * 4 / 1e9), 15 * US + idx / 1e12 + 200 * US)
    assert p.iteration_time("gpu", "gpu", W) == pytest.approx(t, rel=1e-12)
    # RM on the CPU, Learner on the GPU: indices and priorities cross the link, insertions do not
    t = 100 * US + (10 * US + idx / 1e9) + max(50 * US + 64 * 4 / 1e10, 80 * US + (10 * US + idx / 1e9) + 200 * US)
    assert p.iteration_time("cpu", "gpu", W) == pytest.approx(t, rel=1e-12)
    # the insertion branch of the max decides when the Learner is fast
    p.rows["gpu"].learner = 1 * US
    p.rows["gpu"].rm_insert = 500 * US
    t = 20 * US + idx / 1e12 + (500 * US + 10 * US + 256 / 1e9)
    assert p.iteration_time("gpu", "gpu", W) == pytest.approx(t, rel=1e-12)
    # a device without a Learner entry is not a candidate
    p.rows["cpu"].learner = None
    assert p.iteration_time("gpu", "cpu", W) is None


def test_shared_device_column():
    p = platform(shared={"learner": 260 * US, "rm_sampling": 25 * US})
    alone = platform()
    assert p.iteration_time("gpu", "gpu", W) - alone.iteration_time("gpu", "gpu", W) == pytest.approx(65 * US)
    assert p.iteration_time("cpu", "gpu", W) == pytest.approx(alone.iteration_time("cpu", "gpu", W))


def test_step_1_is_the_argmax_over_all_pairs():
    p = platform()
    best, score, scores = p.place_primitives(W)
    brute = {(i, j): W.BS / p.iteration_time(i, j, W) for i, j in itertools.product(("cpu", "gpu"), repeat=2)}
    assert scores == pytest.approx(brute)
    assert best == max(brute, key=brute.get) == ("gpu", "gpu")
    assert score == pytest.approx(W.BS / p.iteration_time("gpu", "gpu", W))
    # power efficiency divides by the power of the two primitives on their devices
    best_p, score_p, scores_p = p.place_primitives(W, "power")
    for (i, j), s in scores_p.items():
        assert s == pytest.approx(brute[(i, j)] / (p.rows[i].rm_power + p.rows[j].learner_power))
    assert best_p == max(scores_p, key=scores_p.get)
    # free links: the choice reduces to the fastest device for each side of the critical path
    free = {k: Link(0.0, 1e30) for k in p.links}
    q = Platform(p.rows, free)
    assert q.place_primitives(W)[0] == ("gpu", "gpu")
    q.rows["gpu"].learner = 5000 * US
    assert q.place_primitives(W)[0] == ("gpu", "cpu")
    # a slow link keeps both primitives on one side
    slow = dict(p.links)
    slow[("cpu", "gpu")] = Link(1.0, 1e3)
    r = Platform(platform().rows, slow)
    (i, j), _, _ = r.place_primitives(W)
    assert i == j == "cpu"       # the GPU pair would still wait for the insertions over the link


def test_step_2_data_storage_by_hand():
    p = platform()
    # RM and Learner on the GPU, Actors on the host: words per iteration 256*11, 64*10, 256
    best, t, totals = p.place_data_storage(W, "gpu", "gpu")
    on_gpu = 4 * (2816 / 1e12 + 640 / 1e9 + 256 / 1e12)
    on_cpu = 4 * (2816 / 1e9 + 640 / 1e10 + 256 / 1e9)
    assert totals == pytest.approx({"gpu": on_gpu, "cpu": on_cpu})
    assert best == "gpu" and t == pytest.approx(on_gpu)
    # many actors and a tiny batch pull the storage to the host
    w = Workload(BS=2, E=10, n_actor=100000)
    assert p.place_data_storage(w, "gpu", "gpu")[0] == "cpu"
    # everything on one device: one candidate
    assert p.place_data_storage(W, "cpu", "cpu")[2].keys() == {"cpu"}


def test_gpu_row_from_a_bench_line():
    line = json.loads('{"kernels_us": {"k_sample": 10.0, "k_tree_finish": 12.0, "k_insert_small": 8.0}, '
                      '"config": {"B": 64, "T": 1}}')
    row = rm_latencies_from_bench(line)
    assert (row.rm_sampling, row.rm_update, row.rm_insert) == pytest.approx((10e-6, 12e-6, 8e-6))
    del line["kernels_us"]["k_insert_small"]
    assert rm_latencies_from_bench(line).rm_insert == pytest.approx(12e-6)
