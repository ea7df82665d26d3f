"""System Composer cost model as a calculator (Section VI of the paper): where should the Replay
Manager (RM), the Learner and the Data Storage live, given per-device latencies and the links
between devices?  Pure host arithmetic; no kernel, no GPU needed.

What it evaluates, in the paper's notation:

* communication between primitives, ``T_comm = lat + data size / bandwidth`` (Section VI-A);
* the FPGA pipeline models of Eq. 4-6: ``T_RM^sampling = 2 F (BS + D) + T_comm``,
  ``T_RM^{update or insert} = 2 (BS + D) + T_comm``, ``T_Learner = T_stage (BS + 3 (#layers - 1))``
  (cycle counts, turned into seconds by the clock period), for filling FPGA rows of the table;
* the iteration time of Eq. 7 for RM on device i and Learner on device j,
  ``T_itr = T_RM^sampling(i) + comm(i->j) + max(T_RM^insert(i) + comm(cpu->i),
  T_RM^update(i) + comm(j->i) + T_Learner(j))``;
* Algorithm 1, step 1: the (i, j) that maximises ``BS / T_itr`` (throughput) or
  ``BS / (T_itr * sum of power)`` (power efficiency);
* Algorithm 1, step 2: the device for the Data Storage, among those of Learner, Actors and RM, with
  the smallest total ``sum_i' C_i' / bandwidth(D[i], D[i'])``, where per iteration
  ``C_Learner = BS (E + 1)``, ``C_Actor = N_actor E``, ``C_RM = BS`` words.

The rows of the "Primitive Device Assignment Matrix" (Table 2) are plain numbers supplied by the
caller: measured, like the MI355X row that `rm_latencies_from_bench` takes from a bench line of this
repository, or modelled (the FPGA functions below).  When RM and Learner share a device the third
column of the table applies (latencies measured with both resident); it defaults to the separate ones.
"""
from __future__ import annotations

import argparse
import itertools
import json
from dataclasses import dataclass, field
from typing import Dict, Optional, Tuple


@dataclass(frozen=True)
class Link:
    """A path between two devices (or inside one): fixed latency in seconds, bandwidth in bytes/s."""
    lat: float
    bandwidth: float

    def time(self, nbytes: float) -> float:
        return self.lat + nbytes / self.bandwidth


@dataclass
class DeviceRow:
    """One row of the Primitive Device Assignment Matrix: seconds per iteration of each primitive on
    this device (None: the primitive cannot run there), and the power drawn while running it."""
    rm_sampling: Optional[float] = None
    rm_update: Optional[float] = None
    rm_insert: Optional[float] = None
    learner: Optional[float] = None
    rm_power: float = 0.0
    learner_power: float = 0.0
    # third column of the table: both primitives resident on this device (defaults to the separate entries)
    shared: Dict[str, float] = field(default_factory=dict)

    def latency(self, what: str, together: bool) -> Optional[float]:
        if together and what in self.shared:
            return self.shared[what]
        return getattr(self, what)


# ------------------------------------------------------------------ Eq. 4-6 (FPGA pipeline models)
def fpga_rm_sampling(F: int, BS: int, D: int, clock_hz: float, t_comm: float = 0.0) -> float:
    """Eq. 4: 2 F (BS + D) cycles, D = sum tree depth (pipeline fill and drain), plus T_comm."""
    return 2 * F * (BS + D) / clock_hz + t_comm


def fpga_rm_update_or_insert(BS: int, D: int, clock_hz: float, t_comm: float = 0.0) -> float:
    """Eq. 5: 2 (BS + D) cycles plus T_comm."""
    return 2 * (BS + D) / clock_hz + t_comm


def fpga_learner(t_stage: float, BS: int, n_layers: int) -> float:
    """Eq. 6: T_stage (BS + 3 (#layers - 1)); t_stage in seconds."""
    return t_stage * (BS + 3 * (n_layers - 1))


# ------------------------------------------------------------------ Eq. 7 and Algorithm 1
@dataclass
class Workload:
    BS: int                 # batch size of an iteration
    E: int                  # words per experience
    n_actor: int            # experiences inserted per iteration
    word_bytes: int = 4


class Platform:
    def __init__(self, rows: Dict[str, DeviceRow], links: Dict[Tuple[str, str], Link], host: str = "cpu"):
        """links[(a, b)] describes a -> b; (a, a) the device's own memory.  A missing (b, a) falls back to (a, b)."""
        self.rows, self.links, self.host = rows, links, host

    def link(self, a: str, b: str) -> Link:
        if (a, b) in self.links:
            return self.links[(a, b)]
        if (b, a) in self.links:
            return self.links[(b, a)]
        raise KeyError(f"no link between {a} and {b}")

    def iteration_time(self, i: str, j: str, w: Workload) -> Optional[float]:
        """Eq. 7 for RM on i and Learner on j; None if a primitive cannot run on its device."""
        together = i == j
        ri, rj = self.rows[i], self.rows[j]
        sampling, update = ri.latency("rm_sampling", together), ri.latency("rm_update", together)
        insert, learner = ri.latency("rm_insert", together), rj.latency("learner", together)
        if None in (sampling, update, insert, learner):
            return None
        wb = w.word_bytes
        idx_out = self.link(i, j).time(w.BS * wb)                  # sampled indices to the Learner's device
        prio_back = self.link(j, i).time(w.BS * wb)                # new priorities back to the RM
        ins_in = self.link(self.host, i).time(w.n_actor * wb)      # insertion requests from the Actors (host)
        return sampling + idx_out + max(insert + ins_in, update + prio_back + learner)

    def place_primitives(self, w: Workload, objective: str = "throughput"):
        """Algorithm 1, step 1.  Returns ((D_RM, D_Learner), score, table of all scores)."""
        if objective not in ("throughput", "power"):
            raise ValueError(objective)
        scores = {}
        for i, j in itertools.product(self.rows, self.rows):
            t = self.iteration_time(i, j, w)
            if t is None:
                continue
            s = w.BS / t
            if objective == "power":
                s /= self.rows[i].rm_power + self.rows[j].learner_power
            scores[(i, j)] = s
        if not scores:
            raise ValueError("no feasible assignment")
        best = max(scores, key=lambda k: (scores[k], k))   # ties: a fixed order
        return best, scores[best], scores

    def place_data_storage(self, w: Workload, d_rm: str, d_learner: str, d_actors: Optional[str] = None):
        """Algorithm 1, step 2.  Returns (device, traffic time, {candidate: traffic time})."""
        d_actors = self.host if d_actors is None else d_actors
        where = {"Learner": d_learner, "Actors": d_actors, "RM": d_rm}
        cost = {"Learner": w.BS * (w.E + 1), "Actors": w.n_actor * w.E, "RM": w.BS}   # words per iteration
        totals = {}
        for cand in ("Learner", "Actors", "RM"):        # the paper's order; the first minimum wins
            dev = where[cand]
            if dev in totals:
                continue
            totals[dev] = sum(cost[k] * w.word_bytes / self.link(dev, where[k]).bandwidth for k in cost)
        best = min(totals, key=totals.get)
        return best, totals[best], totals


# ------------------------------------------------------------------ the MI355X row from a bench line
def rm_latencies_from_bench(line: dict) -> DeviceRow:
    """RM entries of a device row from one JSON line of this repository's bench.py: the fused step's two
    kernels split as sampling (+ gather and weights) and update; insertion from k_insert_small when the
    workload inserts, else the update's time (Eq. 5 gives both the same form)."""
    k = line["kernels_us"]
    sampling = k.get("k_sample", 0.0) * 1e-6
    update = (k.get("k_tree_finish", 0.0) + k.get("k_update_claim", 0.0) + k.get("k_update_tree", 0.0)) * 1e-6
    insert = k.get("k_insert_small", 0.0) * 1e-6 or update
    return DeviceRow(rm_sampling=sampling, rm_update=update, rm_insert=insert)


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--bench-json", required=True, help="file holding a JSON line printed by bench.py (RM on the GPU)")
    ap.add_argument("--learner-gpu-us", type=float, required=True, help="one SGD step of the Learner on the GPU")
    ap.add_argument("--learner-cpu-us", type=float, required=True)
    ap.add_argument("--rm-cpu-us", type=float, nargs=3, metavar=("SAMPLING", "UPDATE", "INSERT"), required=True)
    ap.add_argument("--pcie-gbps", type=float, default=64.0)
    ap.add_argument("--pcie-lat-us", type=float, default=5.0)
    ap.add_argument("--hbm-gbps", type=float, default=8000.0)
    ap.add_argument("--ddr-gbps", type=float, default=300.0)
    ap.add_argument("--E", type=int, default=32, help="words per experience")
    ap.add_argument("--n-actor", type=int, default=64)
    args = ap.parse_args(argv)
    with open(args.bench_json) as f:
        line = json.loads([x for x in f if x.startswith("{")][-1])
    gpu = rm_latencies_from_bench(line)
    gpu.learner = args.learner_gpu_us * 1e-6
    cpu = DeviceRow(*(x * 1e-6 for x in args.rm_cpu_us), learner=args.learner_cpu_us * 1e-6)
    pcie = Link(args.pcie_lat_us * 1e-6, args.pcie_gbps * 1e9)
    plat = Platform({"cpu": cpu, "gpu": gpu},
                    {("cpu", "gpu"): pcie, ("cpu", "cpu"): Link(0.0, args.ddr_gbps * 1e9),
                     ("gpu", "gpu"): Link(0.0, args.hbm_gbps * 1e9)})
    w = Workload(BS=line["config"]["B"] * line["config"]["T"], E=args.E, n_actor=args.n_actor)
    (d_rm, d_learner), score, scores = plat.place_primitives(w)
    storage, _, totals = plat.place_data_storage(w, d_rm, d_learner)
    print(json.dumps({"D[RM]": d_rm, "D[Learner]": d_learner, "D[Data Storage]": storage,
                      "throughput_per_s": score, "all": {f"{i}/{j}": s for (i, j), s in scores.items()},
                      "storage_traffic_s": totals}))


if __name__ == "__main__":
    main()
