#!/usr/bin/env python3
"""Throughput of the prioritized-replay hot path on one MI355X.

One step = priority sampling (with importance weights) -> row gather -> priority
update over one batch of synthetic input, on the workload the headline metric is
quoted on (N = 2^24 leaves, K = 32, B = 65536, 128-byte rows, 10 % duplicated
update indices).  Prints ONE JSON line: transitions/s, the roofline figure of the
dominant kernel (HIP-event timed inside this run) and the CPU oracle's rate on a
bounded sample of the same steps.

All inputs are resident in HBM before the timed region.  The headline form is the
loop of Listing 2 as it is: the update of step s targets the indices sampled in
step s, taken through the workload's duplicate position map inside the step
(`per_step`), so the sample -> update dependency is inside the timed region.
Beside it the line reports the relaxed form in which the update batch is a
separate array that exists before the step starts ("earlier_batch_form": the
priorities of an earlier batch; the array is filled from a first pass).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published peak


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c4_stress")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="time budget of the oracle leg (0: skip)")
    ap.add_argument("--no-graph", action="store_true", help="enqueue the timed steps eagerly instead of as one HIP graph")
    ap.add_argument("--separate-gather", action="store_true",
                    help="call per_sample and per_gather separately instead of the fused per_sample_gather")
    ap.add_argument("--separate-update", action="store_true",
                    help="call per_update by itself instead of per_sample_gather_update")
    ap.add_argument("--separate-insert", action="store_true",
                    help="call per_insert and per_step instead of per_insert_step (workloads with a per-step insert)")
    ap.add_argument("--overlap", action="store_true",
                    help="with --separate-gather: run the row gather on a second stream beside the update")
    ap.add_argument("--no-delta-form", action="store_true",
                    help="skip the extra timing of the step with the paper's delta-propagation update")
    ap.add_argument("--tune", action="append", default=[], help="name=value passed to per_set_tuning")
    ap.add_argument("--only-headline", action="store_true",
                    help="time only the headline form (for profiler runs: every kernel launch then belongs to it)")
    ap.add_argument("--weight-norm", choices=["batch", "buffer"], default="batch",
                    help="importance weights relative to the sampled batch (the metric's form) or to the whole buffer")
    return ap.parse_args()


def algorithmic_bytes(w, idx, upd_idx, K, H, h_lds, weights):
    """Bytes the method itself must move in one step, per part of the step, each distinct K-group counted
    once per phase (what a perfect cache would move).  idx / upd_idx: [T, B] uint32 of one step.
    h_lds: lowest height taken to be on chip; only the child groups below it count as memory traffic.
      sample : 4B (u) + sum_{h < h_lds} 4K G_h + 4B (idx) + 4B (weight) + 4B (sampled priority, requested here)
      gather : 4B (idx) + E R (distinct rows) + E B (dense rows)
      update : 8B (idx, prio) + 4U (leaf writes) + sum_{h=1..H} (4K Q_h + 4 Q_h)
    Values that only pass between two kernels of the step (the sampled value on its way to becoming a weight)
    are not counted."""
    logK = K.bit_length() - 1
    T, B = idx.shape
    E = w.row_bytes
    out = {"k_sample": 0, "k_weights": 0, "k_rows_gather": 0, "k_update_claim": 0, "k_update_tree": 0}
    for t in range(T):
        i64 = idx[t].astype(np.int64)
        groups = sum(len(np.unique(i64 >> ((h + 1) * logK))) * 4 * K for h in range(0, min(h_lds, H)))
        out["k_sample"] += 4 * B + groups + 4 * B + 4 * B                                 # u, groups, idx, sampled priority
        out["k_weights"] += 4 * B if weights else 0                                       # weight out
        out["k_rows_gather"] += 4 * B + E * len(np.unique(i64)) + E * B                   # idx, distinct rows, dense rows
        u64 = upd_idx[t].astype(np.int64)
        out["k_update_claim"] += 8 * B                                                    # idx, prio
        out["k_update_tree"] += 4 * len(np.unique(u64))                                   # leaf writes
        for h in range(1, H + 1):
            q = len(np.unique(u64 >> (h * logK)))
            out["k_update_tree"] += 4 * K * q + 4 * q                                     # child groups in, node out
    return out


def per_launched_kernel(parts, launched):
    """Algorithmic bytes of the kernels that were launched, from the parts of the step each one carries."""
    alg = dict(parts)
    if "k_step" in launched:            # sampling and the update of the sampled batch in one kernel; rows and weights in its epilogue
        alg["k_step"] = parts["k_sample"] + parts["k_update_claim"] + parts["k_update_tree"]
        alg["k_step_epilogue"] = parts["k_rows_gather"] + parts["k_weights"]
    elif "k_tree_finish" in launched:   # two-kernel step: claim in the sampling kernel, tree pass beside rows and weights
        alg["k_sample"] = parts["k_sample"] + parts["k_update_claim"]
        alg["k_tree_finish"] = parts["k_update_tree"] + parts["k_rows_gather"] + parts["k_weights"]
    elif "k_finish" in launched:        # second kernel: rows and weights, plus the claim when no claim kernel ran
        alg["k_finish"] = parts["k_rows_gather"] + parts["k_weights"] + \
            (0 if "k_update_claim" in launched else parts["k_update_claim"])
    return alg


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the rocprofv3 counter runs summarised under profiles/
    (FETCH_SIZE + WRITE_SIZE, scaled by a copy kernel of known size); None if no summary exists."""
    path = os.path.join(ROOT, "profiles", f"{workload}_hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        parts = line.split()
        if len(parts) >= 2 and parts[0] == kernel:
            try:
                return int(float(parts[1]))
            except ValueError:
                return None
    return None


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2311_09445_amd import workloads as wl
    from paper_2311_09445_amd.per import PrioritizedReplay

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    w = wl.WORKLOADS[args.workload]
    K, N, T, B = w.K, w.N, w.T, w.B
    steps, warmup = args.steps, args.warmup
    total_steps = steps + warmup
    t_setup = time.time()

    # ---------------------------------------------------------------- state
    buf = PrioritizedReplay(K, N, T, w.field_bytes)
    for kv in args.tune:
        k, v = kv.split("=")
        buf.set_tuning(k, int(v))
    buf.set_weight_norm(args.weight_norm)
    prio0 = wl.initial_priorities(w, args.seed)
    chunk = 1 << 20
    for lo in range(0, N, chunk):
        m = min(chunk, N - lo)
        cnt = torch.arange(lo, lo + m, device="cuda")
        rows = [torch.stack([wl.row_bytes_torch(t, cnt, f, b) for t in range(T)]) for f, b in enumerate(w.field_bytes)]
        buf.insert(m, rows, torch.from_numpy(np.ascontiguousarray(prio0[:, lo:lo + m])).cuda())
    del rows
    counter = N

    # ---------------------------------------------------------------- inputs, resident on the device
    inputs = [wl.step_inputs(w, s, args.seed) for s in range(total_steps)]
    d_u = torch.from_numpy(np.stack([i["u"] for i in inputs])).cuda()
    d_prio = torch.from_numpy(np.stack([i["upd_prio"] for i in inputs])).cuda()
    d_idx = torch.empty((total_steps, T, B), dtype=torch.int32, device="cuda")
    d_upd_idx = torch.empty((total_steps, T, B), dtype=torch.int32, device="cuda")
    d_w = torch.empty((T, B), dtype=torch.float32, device="cuda")
    d_v = torch.empty((T, B), dtype=torch.float32, device="cuda")
    d_rows = [torch.empty((T, B, b), dtype=torch.uint8, device="cuda") for b in w.field_bytes]
    ins_rows = None
    if w.n_insert:
        ins_rows = []
        for s in range(total_steps):
            cnt = torch.arange(counter + s * w.n_insert, counter + (s + 1) * w.n_insert, device="cuda")
            ins_rows.append([torch.stack([wl.row_bytes_torch(t, cnt, f, b) for t in range(T)])
                             for f, b in enumerate(w.field_bytes)])
    has_dup = "dup_dst" in inputs[0]
    d_pos = None
    if has_dup:   # the duplicate map as a position map: update element j targets the index sampled at position pos[j]
        d_pos = torch.from_numpy(np.stack([wl.dup_positions(i, T, B) for i in inputs]).view(np.int32)).cuda()

    side = torch.cuda.Stream()
    gather_done = [None]
    fused = not args.separate_gather
    fused_step = fused and not args.separate_update

    def step_in(s):
        """The loop of Listing 2 as it is: insert -> sample -> gather -> update of the batch just sampled (through the
        duplicate position map where the workload has one), one per_step call."""
        ins = None
        if w.n_insert and args.separate_insert:
            buf.insert(w.n_insert, ins_rows[s])
        elif w.n_insert:
            ins = (w.n_insert, ins_rows[s], None, None)      # per_insert_step: the insertion inside the step call
        buf.step(d_u[s], inputs[s]["beta"], d_prio[s], None if d_pos is None else d_pos[s], want_weights=w.weights,
                 want_prio=True, out_idx=d_idx[s], out_weight=d_w, out_prio=d_v, rows_out=d_rows, insert=ins)

    def step(s, overlap=False):
        """The relaxed form: the update batch of step s is a separate array that exists before the step starts.
        With overlap the row gather (which only reads the sampled indices and the payload) runs on a second
        stream beside the update, as the paper's runtime overlaps data movement with the replay operations."""
        main = torch.cuda.current_stream()
        if w.n_insert:
            if overlap and gather_done[0] is not None:
                main.wait_event(gather_done[0])      # an insert may overwrite a row the last gather reads
            buf.insert(w.n_insert, ins_rows[s])
        buf.sample(d_u[s], inputs[s]["beta"], want_weights=w.weights, want_prio=True,
                   out_idx=d_idx[s], out_weight=d_w, out_prio=d_v, rows_out=d_rows if fused else None,
                   update=(d_upd_idx[s], d_prio[s]) if fused_step else None)
        if fused_step:
            return
        if fused:
            pass
        elif overlap:
            sampled = torch.cuda.Event()
            sampled.record(main)
            with torch.cuda.stream(side):
                side.wait_event(sampled)
                buf.gather(d_idx[s], d_rows)
                gather_done[0] = torch.cuda.Event()
                gather_done[0].record(side)
        else:
            buf.gather(d_idx[s], d_rows)
        buf.update(d_upd_idx[s], d_prio[s])

    torch.cuda.synchronize()
    snapshot = buf.arena.clone()
    cursor0 = (buf.cursor, buf.size)

    def restore():
        buf.arena.copy_(snapshot)
        buf.set_ring(*cursor0)
        torch.cuda.synchronize()

    stream = torch.cuda.current_stream()

    def time_form(one_step, overlap=False):
        """Per-kernel durations with HIP events attached to each launch (a pass of its own: the events add gaps
        between kernels), then the timed run: warm-up steps eagerly, the timed steps as one HIP graph."""
        restore()
        for s in range(warmup):
            one_step(s)
        buf.profile(True)
        for s in range(warmup, total_steps):
            one_step(s)
        torch.cuda.synchronize()
        kern = buf.profile_read()
        buf.profile(False)
        idx_seen = d_idx.cpu().numpy().view(np.uint32).copy()
        root_seen = buf.total().cpu().numpy().copy()
        status_seen = buf.status()
        restore()
        gather_done[0] = None
        for s in range(warmup):
            one_step(s)
        torch.cuda.synchronize()
        graph = None
        if not args.no_graph:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for s in range(warmup, total_steps):
                    one_step(s, overlap=overlap) if overlap else one_step(s)
                if overlap:
                    torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        ev0.record(stream)
        if graph is not None:
            graph.replay()
        else:
            for s in range(warmup, total_steps):
                one_step(s, overlap=overlap) if overlap else one_step(s)
            if overlap:
                stream.wait_stream(side)
        ev1.record(stream)
        torch.cuda.synchronize()
        ms = ev0.elapsed_time(ev1) / steps
        buf.note_replay()
        # the timed run must have reproduced the trajectory of the pass before it
        assert np.array_equal(d_idx.cpu().numpy().view(np.uint32)[warmup:], idx_seen[warmup:]), "timed run diverged"
        assert buf.total().cpu().numpy().tobytes() == root_seen.tobytes(), "timed run ended in a different state"
        return ms, kern, idx_seen, root_seen, status_seen, graph is not None

    # ---------------------------------------------------------------- headline: the update targets this step's sample
    ms_per_step, kernels, rec_idx, final_root, status_record, graphed = time_form(step_in)
    rec_upd = np.stack([wl.apply_dup_map(rec_idx[s], inputs[s]) for s in range(total_steps)])

    # ---------------------------------------------------------------- beside it: the update batch known before the step
    # (same trajectory: the array holds what the headline form derives inside the step)
    d_upd_idx.copy_(torch.from_numpy(rec_upd.view(np.int32)).cuda())
    overlap = args.overlap and not fused
    if args.only_headline:
        ms_early, kernels_early = ms_per_step, kernels
    else:
        ms_early, kernels_early, idx_early, root_early, _, _ = time_form(step, overlap=overlap)
        assert np.array_equal(idx_early, rec_idx) and root_early.tobytes() == final_root.tobytes(), "the two forms disagree"
    restore_ok = True

    # ---------------------------------------------------------------- algorithmic bytes and roofline
    H = buf.H
    lvl_n = [buf.level_count(h) for h in range(H + 1)]
    # h_lds: the lowest height such that it and everything above it fit the LDS of one compute unit beside the
    # sampling kernel's staging rows (c4: height 2, 64 KiB + 2.2 KiB); child groups below it count as traffic
    h_lds, acc = H, 0
    for l in range(H - 1, -1, -1):
        add = lvl_n[l + 1] * K * 4
        if acc + add > 96 * 1024:
            break
        acc += add
        h_lds = l
    sel = list(range(warmup, total_steps, max(1, steps // 16)))
    per_step = [algorithmic_bytes(w, rec_idx[s], rec_upd[s], K, H, h_lds, w.weights) for s in sel]
    parts = {k: float(np.mean([p[k] for p in per_step])) for k in per_step[0]}
    a_sample = parts["k_sample"]
    a_gather = parts["k_rows_gather"] + parts["k_weights"]
    a_update = parts["k_update_claim"] + parts["k_update_tree"]
    a_step = a_sample + a_gather + a_update

    def kernel_view(kern):
        alg = per_launched_kernel(parts, set(kern))
        kern_ms = {k: v[0] / max(1, v[1]) for k, v in kern.items()}
        per = {k: v[1] / steps for k, v in kern.items()}
        return alg, kern_ms, per, [k for k in kern if k in alg]

    alg, kern_ms, kern_per_step, step_kernels = kernel_view(kernels)
    dominant = max(step_kernels, key=lambda k: kernels[k][0])
    dom_bytes = alg[dominant] / max(1e-9, kern_per_step[dominant])
    dom_gbs = dom_bytes / (kern_ms[dominant] * 1e-3) / 1e9
    roofline = {
        "kernel": dominant, "bound": "hbm", "achieved": round(dom_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": round(dom_gbs / HBM_PEAK_GBS, 4), "traffic": measured_traffic(w.name, dominant),
        "traffic_source": f"profiles/{w.name}_hbm_traffic.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command)",
        "algorithmic_bytes_per_launch": int(dom_bytes), "avg_launch_us": round(kern_ms[dominant] * 1e3, 2),
    }
    step_gbs = a_step / (ms_per_step * 1e-3) / 1e9
    alg_e, kern_ms_e, kern_per_e, step_kernels_e = kernel_view(kernels_early)
    early_form = {
        "update_indices": "a separate array filled before the step (the priorities of an earlier batch); here it holds "
                          "what the headline form derives in-step, so both forms walk the same trajectory",
        "calls_per_step": "per_sample_gather_update" if fused_step else
                          ("per_sample_gather, per_update" if fused else "per_sample, per_gather, per_update"),
        "ms_per_step": round(ms_early, 5), "value": round(T * B / (ms_early * 1e-3), 1), "unit": "transitions/s",
        "step_hbm_frac": round(a_step / (ms_early * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "streams": 2 if overlap else 1,
        "kernels_us": {k: round(v * 1e3, 2) for k, v in sorted(kern_ms_e.items())},
        "kernel_algorithmic_bytes": {k: int(alg_e[k]) for k in sorted(step_kernels_e)},
    }

    # ---------------------------------------------------------------- the paper's own update form, for comparison
    # Same step with the update done as the paper does it (Section V-A): retrieve the old priorities, form
    # delta = new - old, add delta along every path (per_get_priority, one subtraction, per_update_delta).
    # Changes meet in no fixed order there, so this run is timed but not compared with a recorded trajectory.
    delta_form = None
    if fused and not args.no_delta_form:
        d_old = torch.empty((T, B), dtype=torch.float32, device="cuda")
        d_delta = torch.empty((T, B), dtype=torch.float32, device="cuda")

        def delta_step(s):
            if w.n_insert:
                buf.insert(w.n_insert, ins_rows[s])
            buf.sample(d_u[s], inputs[s]["beta"], want_weights=w.weights, want_prio=True,
                       out_idx=d_idx[s], out_weight=d_w, out_prio=d_v, rows_out=d_rows)
            buf.get_priority(d_upd_idx[s], out=d_old)
            torch.sub(d_prio[s], d_old, out=d_delta)
            buf.update_delta(d_upd_idx[s], d_delta)

        restore()
        for s in range(warmup):
            delta_step(s)
        buf.profile(True)
        for s in range(warmup, total_steps):
            delta_step(s)
        torch.cuda.synchronize()
        dk = buf.profile_read()
        buf.profile(False)
        restore()
        for s in range(warmup):
            delta_step(s)
        torch.cuda.synchronize()
        g2 = None
        if not args.no_graph:
            g2 = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g2):
                for s in range(warmup, total_steps):
                    delta_step(s)
            torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        if g2 is not None:
            g2.replay()
        else:
            for s in range(warmup, total_steps):
                delta_step(s)
        e1.record(stream)
        torch.cuda.synchronize()
        ms_delta = e0.elapsed_time(e1) / steps
        delta_form = {"ms_per_step": round(ms_delta, 5), "value": round(T * B / (ms_delta * 1e-3), 1),
                      "unit": "transitions/s", "status_flags": buf.status(),
                      "calls_per_step": "per_sample_gather, per_get_priority, (new - old), per_update_delta",
                      "kernels_us": {k: round(v[0] / max(1, v[1]) * 1e3, 2) for k, v in sorted(dk.items())},
                      "update_algorithmic_bytes": int(T * (8 * B + 4 * B + 8 * B * (H + 1)))}
        del g2
    # ---------------------------------------------------------------- the same steps as one launch (small buffers)
    # When a whole tree fits the LDS of a compute unit, per_run_steps runs the list of steps in one kernel,
    # one workgroup per tree (the paper's on-chip tree and request stream, Section V-A "RM on FPGA").
    step_stream = None
    if fused_step and buf.run_steps_fits() and B <= 1024 and w.n_insert <= 1024:
        restore()
        o_idx = torch.empty((total_steps, T, B), dtype=torch.int32, device="cuda")
        o_w = torch.empty((total_steps, T, B), dtype=torch.float32, device="cuda") if w.weights else None
        o_v = torch.empty((total_steps, T, B), dtype=torch.float32, device="cuda")
        o_rows = [torch.empty((total_steps, T, B, b), dtype=torch.uint8, device="cuda") for b in w.field_bytes]
        d_beta = torch.tensor([inputs[s]["beta"] for s in range(total_steps)], dtype=torch.float32, device="cuda")
        i_rows = None
        if w.n_insert:
            i_rows = [torch.stack([ins_rows[s][f] for s in range(total_steps)]) for f in range(len(w.field_bytes))]

        def run(lo, hi):
            buf.run_steps(d_u[lo:hi], d_beta[lo:hi], o_idx[lo:hi], None if o_w is None else o_w[lo:hi], o_v[lo:hi],
                          [r[lo:hi] for r in o_rows], upd_prio=d_prio[lo:hi], upd_idx=d_upd_idx[lo:hi],
                          n_insert=w.n_insert, ins_rows=None if i_rows is None else [r[lo:hi] for r in i_rows])

        run(0, warmup)
        torch.cuda.synchronize()
        s0, s1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s0.record(stream)
        run(warmup, total_steps)
        s1.record(stream)
        torch.cuda.synchronize()
        ms_stream = s0.elapsed_time(s1) / steps
        assert np.array_equal(o_idx.cpu().numpy().view(np.uint32), rec_idx), "step kernel diverged from the separate calls"
        assert buf.total().cpu().numpy().tobytes() == final_root.tobytes(), "step kernel ended in a different state"
        step_stream = {"ms_per_step": round(ms_stream, 5), "value": round(T * B / (ms_stream * 1e-3), 1),
                       "unit": "transitions/s", "launches": 1, "steps_per_launch": steps,
                       "call": "per_run_steps (tree, or its heights above the leaves, held in LDS; one workgroup per tree)"}

        # the same steps once more as a queue of op-coded requests (insert, sample, update per step)
        from paper_2311_09445_amd.per import OP_INSERT, OP_SAMPLE, OP_UPDATE

        def queue(lo, hi):
            q = []
            for s in range(lo, hi):
                if w.n_insert:
                    q.append({"op": OP_INSERT, "n": w.n_insert, "rows": None if i_rows is None else [r[s] for r in i_rows]})
                q.append({"op": OP_SAMPLE, "u": d_u[s], "beta": float(inputs[s]["beta"]), "idx": o_idx[s],
                          "out_weight": None if o_w is None else o_w[s], "out_prio": o_v[s], "rows": [r[s] for r in o_rows]})
                q.append({"op": OP_UPDATE, "idx": d_upd_idx[s], "prio": d_prio[s]})
            return q

        restore()
        o_idx.zero_()
        keep = [buf.run_requests(queue(0, warmup))]
        timed_queue = buf.prepare_requests(queue(warmup, total_steps))   # encoded and copied to the device beforehand
        torch.cuda.synchronize()
        s0.record(stream)
        keep.append(buf.run_requests(timed_queue))
        s1.record(stream)
        torch.cuda.synchronize()
        ms_queue = s0.elapsed_time(s1) / steps
        assert np.array_equal(o_idx.cpu().numpy().view(np.uint32), rec_idx), "request queue diverged from the separate calls"
        assert buf.total().cpu().numpy().tobytes() == final_root.tobytes(), "request queue ended in a different state"
        step_stream["request_queue"] = {
            "ms_per_step": round(ms_queue, 5), "requests": timed_queue[0],
            "call": "per_run_requests (the same steps as a queue of op-coded requests, one launch)"}
        del o_idx, o_w, o_v, o_rows, keep

    # what a plain streaming device copy reaches on this GPU in this run (read + written bytes per second)
    src = torch.empty(1 << 28, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record()
    for _ in range(10):
        dst.copy_(src)
    c1.record()
    torch.cuda.synchronize()
    copy_gbs = 10 * 2 * src.numel() / (c0.elapsed_time(c1) * 1e-3) / 1e9
    del src, dst
    roofline["measured_copy_GBps"] = round(copy_gbs, 1)
    roofline["frac_of_measured_copy"] = round(dom_gbs / copy_gbs, 4)

    # ---------------------------------------------------------------- CPU oracle on a bounded sample
    cpu = None
    cpu_workers = None
    if args.cpu_seconds > 0:
        from oracle.per_oracle import MultiOracle
        orc = MultiOracle(T, K, N, w.field_bytes, with_payload=True)
        orc.set_weight_norm(args.weight_norm)
        for lo in range(0, N, chunk):
            m = min(chunk, N - lo)
            cnt = np.arange(lo, lo + m)
            rows = [np.stack([wl.row_bytes(t, cnt, f, b) for t in range(T)]) for f, b in enumerate(w.field_bytes)]
            orc.insert(m, rows, prio0[:, lo:lo + m])
        done, t_cpu = 0, 0.0

        def cpu_inputs(s):   # the recorded steps first, then further steps of the same generator
            return inputs[s] if s < total_steps else wl.step_inputs(w, s, args.seed)

        while t_cpu < args.cpu_seconds or done < 3:
            inp = cpu_inputs(done)
            ins = None
            if w.n_insert:
                cnt = np.arange(counter + done * w.n_insert, counter + (done + 1) * w.n_insert)
                ins = [np.stack([wl.row_bytes(t, cnt, f, b) for t in range(T)]) for f, b in enumerate(w.field_bytes)]
            t0 = time.perf_counter()
            if w.n_insert:
                orc.insert(w.n_insert, ins)
            ci, cw, cv = orc.sample(inp["u"], inp["beta"], w.weights)
            orc.gather(ci)
            upd = wl.apply_dup_map(ci, inp)
            orc.update(upd, inp["upd_prio"])
            t_cpu += time.perf_counter() - t0
            if done < total_steps and (restore_ok or done == 0):
                assert np.array_equal(ci, rec_idx[done]), f"oracle and GPU disagree on step {done}"
            done += 1
        model = "unknown CPU"
        try:
            for line in open("/proc/cpuinfo"):
                if line.startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
        except OSError:
            pass
        affinity = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else os.cpu_count()
        cpu = {"value": round(T * B * done / t_cpu, 1), "unit": "transitions/s", "cores": 1, "kind": "oracle",
               "sample": f"first {done} steps of the same workload and inputs, {t_cpu:.1f} s of CPU time, "
                         f"single thread; host: {model}, {os.cpu_count()} cores visible, {affinity} in the affinity mask"}

        # Second CPU baseline: the same arithmetic on worker threads (Section V-A's CPU kernel splits
        # the batch of requests over workers), continuing on the oracle's state with the next steps.
        from oracle.per_workers import Workers
        wks = [Workers(o) for o in orc.trees]
        s_w, done_w, t_w = done, 0, 0.0
        while t_w < args.cpu_seconds / 2 or done_w < 3:
            inp = cpu_inputs(s_w)
            ins = None
            if w.n_insert:
                cnt = np.arange(counter + s_w * w.n_insert, counter + (s_w + 1) * w.n_insert)
                ins = [np.stack([wl.row_bytes(t, cnt, f, b) for t in range(T)]) for f, b in enumerate(w.field_bytes)]
            t0 = time.perf_counter()
            if w.n_insert:
                orc.insert(w.n_insert, ins)
            ci = np.empty((T, B), dtype=np.uint32)
            for t in range(T):
                ci[t], _, _ = wks[t].sample(inp["u"][t], inp["beta"], w.weights)
                wks[t].gather(ci[t])
            upd = wl.apply_dup_map(ci, inp)
            for t in range(T):
                wks[t].update(upd[t], inp["upd_prio"][t])
            t_w += time.perf_counter() - t0
            if s_w < total_steps and restore_ok:
                assert np.array_equal(ci, rec_idx[s_w]), f"worker baseline and GPU disagree on step {s_w}"
            s_w += 1
            done_w += 1
        if done_w:
            cpu_workers = {"value": round(T * B * done_w / t_w, 1), "unit": "transitions/s", "cores": wks[0].threads,
                           "kind": "oracle arithmetic on worker threads (OpenMP), bit-identical to the oracle",
                           "sample": f"steps {done}..{s_w - 1} of the same workload and inputs, {t_w:.1f} s"}
        del wks

    out = {
        "metric": "sampled+updated transitions/s per step; % of HBM peak at N=2^24, B=65536",
        "value": round(T * B / (ms_per_step * 1e-3), 1), "unit": "transitions/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "K": K, "N": N, "T": T, "B": B, "row_bytes": w.row_bytes,
                   "insert_per_step": w.n_insert, "launch": "hip_graph" if graphed else "eager",
                   "streams": 1, "weight_norm": args.weight_norm,
                   "calls_per_step": "per_insert_step" if w.n_insert and not args.separate_insert else
                                     "per_insert, per_step" if w.n_insert else "per_step",
                   "update_indices": "this step's sampled indices" +
                                     (" through the duplicate position map, applied inside the step" if has_dup else "")},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "cpu_workers_baseline": cpu_workers,
        "earlier_batch_form": None if args.only_headline else early_form,
        "paper_update_form": delta_form,
        "step_stream": step_stream,
        "step_algorithmic_bytes": int(a_step),
        "h_lds": h_lds,
        "step_hbm_frac": round(step_gbs / HBM_PEAK_GBS, 4),
        "phase_algorithmic_bytes": {"sample": int(a_sample), "gather_and_weights": int(a_gather), "update": int(a_update)},
        "kernel_algorithmic_bytes": {k: int(alg[k]) for k in sorted(step_kernels)},
        "kernels_us": {k: round(v * 1e3, 2) for k, v in sorted(kern_ms.items())},
        "kernels_per_step": {k: round(v, 2) for k, v in sorted(kern_per_step.items())},
        "device_status_flags": status_record,
        "setup_s": round(time.time() - t_setup, 1),
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
