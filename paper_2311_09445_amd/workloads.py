"""Seeded synthetic inputs for the prioritized-replay workloads.

This module only *draws inputs*: priorities, uniforms, update values, duplicate
maps and row payload bytes.  It holds none of the sum-tree arithmetic, so both
the CPU oracle's tests and the HIP path's tests/bench may use it without
sharing any part of the method.

The five workloads stand in for the paper's Gym benchmarks (Table 3: DQN
CartPole / DDPG MountainCar / DQN Pong), whose simulators are not available;
only buffer shapes, batch sizes and priority distributions matter to the
replay path.  Every value is drawn in fp64 and rounded once to fp32; uniforms
are (uint32 >> 8) * 2^-24, i.e. exactly representable and in [0, 1).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Tuple

import numpy as np

__all__ = [
    "Workload", "WORKLOADS", "uniform01", "initial_priorities", "step_inputs",
    "row_bytes", "row_bytes_torch", "td_to_priority", "apply_dup_map",
]


@dataclass(frozen=True)
class Workload:
    name: str
    K: int                     # fanout
    N: int                     # capacity (leaves) per tree
    T: int                     # independent trees
    B: int                     # sample / update batch per tree
    n_insert: int              # rows inserted per tree per step (0: none)
    fields: Tuple[Tuple[str, int], ...]   # (name, bytes per row), stored SoA
    steps: int
    prio_dist: str             # initial leaf-value distribution
    upd_dist: str              # distribution of the update values
    beta0: float = 0.4
    beta1: float = 0.4         # beta annealed linearly beta0 -> beta1 over the run
    dup_frac: float = 0.0      # fraction of update slots overwritten by another slot's index
    zero_frac: float = 0.0     # fraction of initial leaves forced to 0
    weights: bool = True

    @property
    def field_bytes(self) -> Tuple[int, ...]:
        return tuple(b for _, b in self.fields)

    @property
    def row_bytes(self) -> int:
        return sum(self.field_bytes)

    def beta(self, step: int) -> float:
        if self.steps <= 1 or self.beta0 == self.beta1:
            return float(self.beta0)
        return float(self.beta0 + (self.beta1 - self.beta0) * step / (self.steps - 1))


_MLP_ROW = (("s", 68), ("a", 24), ("r", 4), ("s2", 68), ("done", 1))

WORKLOADS: Dict[str, Workload] = {
    # Binary tree, classic-control sized rows.
    "c1_binary_small": Workload(
        "c1_binary_small", K=2, N=4096, T=1, B=64, n_insert=4,
        fields=(("s", 16), ("a", 4), ("r", 4), ("s2", 16), ("done", 1)),
        steps=100, prio_dist="uniform_1e-3_1", upd_dist="absnormal1_eps_pow0.6"),
    # DQN-shaped: frame-index rows, small batch, beta annealed.
    "c2_dqn": Workload(
        "c2_dqn", K=16, N=1 << 20, T=1, B=32, n_insert=4,
        fields=(("frames", 16), ("a", 4), ("r", 4), ("done", 1)),
        steps=10_000, prio_dist="lognormal_0_1", upd_dist="absnormal2_eps_pow0.6",
        beta0=0.4, beta1=1.0),
    # DDPG-shaped: 17-float states, 6-float actions, large batch.
    "c3_ddpg": Workload(
        "c3_ddpg", K=16, N=1 << 20, T=1, B=4096, n_insert=1,
        fields=_MLP_ROW, steps=2_000, prio_dist="exponential_1",
        upd_dist="absnormal1_eps_pow0.6"),
    # Large-scale stress: the configuration the headline metric is quoted on.
    "c4_stress": Workload(
        "c4_stress", K=32, N=1 << 24, T=1, B=65536, n_insert=0,
        fields=(("row", 128),), steps=500, prio_dist="pareto_1.5",
        upd_dist="absnormal1_eps_pow0.6", dup_frac=0.10, zero_frac=0.01),
    # Many independent buffers (parallel actor-learner setting).
    "c5_multi": Workload(
        "c5_multi", K=16, N=1 << 18, T=64, B=1024, n_insert=16,
        fields=_MLP_ROW, steps=1_000, prio_dist="uniform_1e-2_1",
        upd_dist="absnormal1_pow0.6"),
}


def _rng(seed: int, *stream: int) -> np.random.Generator:
    return np.random.default_rng([int(seed), *[int(s) for s in stream]])


def uniform01(rng: np.random.Generator, shape) -> np.ndarray:
    """fp32 uniforms in [0, 1): (uint32 >> 8) * 2^-24, exact in fp32."""
    bits = rng.integers(0, 1 << 32, size=shape, dtype=np.uint32)
    return ((bits >> np.uint32(8)).astype(np.float32) * np.float32(2.0 ** -24)).astype(np.float32)


def td_to_priority(delta: np.ndarray, eps: float, alpha: float) -> np.ndarray:
    """(|delta| + eps)^alpha evaluated in fp64 and rounded once to fp32.

    The tree stores p^alpha as handed in; doing the transform here means the
    oracle and the HIP path consume the very same fp32 values.
    """
    d = np.abs(np.asarray(delta, dtype=np.float64)) + float(eps)
    return np.power(d, float(alpha)).astype(np.float32)


def _draw_priorities(dist: str, rng: np.random.Generator, shape) -> np.ndarray:
    if dist == "uniform_1e-3_1":          # (1e-3, 1]
        x = 1.0 - rng.random(shape) * (1.0 - 1e-3)
    elif dist == "uniform_1e-2_1":        # (1e-2, 1]
        x = 1.0 - rng.random(shape) * (1.0 - 1e-2)
    elif dist == "lognormal_0_1":
        x = rng.lognormal(0.0, 1.0, shape)
    elif dist == "exponential_1":
        x = rng.exponential(1.0, shape)
    elif dist == "pareto_1.5":            # x_m = 1, shape 1.5
        x = (1.0 - rng.random(shape)) ** (-1.0 / 1.5)
    else:
        raise ValueError(dist)
    return np.asarray(x, dtype=np.float64).astype(np.float32)


def _draw_updates(dist: str, rng: np.random.Generator, shape) -> np.ndarray:
    if dist == "absnormal1_eps_pow0.6":
        return td_to_priority(rng.standard_normal(shape), 1e-6, 0.6)
    if dist == "absnormal2_eps_pow0.6":
        return td_to_priority(2.0 * rng.standard_normal(shape), 1e-6, 0.6)
    if dist == "absnormal1_pow0.6":       # no epsilon: exact zeros are possible in principle
        return td_to_priority(rng.standard_normal(shape), 0.0, 0.6)
    raise ValueError(dist)


def initial_priorities(w: Workload, seed: int = 0, n: int | None = None) -> np.ndarray:
    """[T, n] fp32 leaf values of the initial fill (n defaults to the capacity)."""
    n = w.N if n is None else int(n)
    rng = _rng(seed, 1)
    v = _draw_priorities(w.prio_dist, rng, (w.T, n))
    if w.zero_frac > 0.0:
        z = _rng(seed, 2).random((w.T, n)) < w.zero_frac
        v[z] = np.float32(0.0)
    return v


def step_inputs(w: Workload, step: int, seed: int = 0, B: int | None = None) -> dict:
    """Inputs of one step: uniforms, update values, duplicate map, beta.

    ``dup_dst`` / ``dup_src`` are positions in the batch: the update indices are
    the sampled indices with ``idx[dup_dst] = idx[dup_src]`` applied (all sources
    read before any destination is written).
    """
    B = w.B if B is None else int(B)
    rng = _rng(seed, 3, step)
    out = {
        "u": uniform01(rng, (w.T, B)),
        "upd_prio": _draw_updates(w.upd_dist, rng, (w.T, B)),
        "beta": w.beta(step),
    }
    n_dup = int(w.dup_frac * B)
    if n_dup > 0:
        out["dup_dst"] = np.stack([rng.choice(B, size=n_dup, replace=False) for _ in range(w.T)]).astype(np.int64)
        out["dup_src"] = rng.integers(0, B, size=(w.T, n_dup), dtype=np.int64)
    return out


def apply_dup_map(idx: np.ndarray, inp: dict) -> np.ndarray:
    """Update indices = sampled indices with the step's duplicate map applied ([T, B])."""
    out = np.array(idx, copy=True)
    if "dup_dst" in inp:
        for t in range(out.shape[0]):
            out[t, inp["dup_dst"][t]] = idx[t, inp["dup_src"][t]]
    return out


def dup_positions(inp: dict, T: int, B: int) -> np.ndarray | None:
    """The step's duplicate map as a position map [T, B]: update element j targets the index sampled at position
    pos[j] (pos[j] = j except pos[dup_dst] = dup_src); None when the step has no duplicate map."""
    if "dup_dst" not in inp:
        return None
    pos = np.tile(np.arange(B, dtype=np.uint32), (T, 1))
    for t in range(T):
        pos[t, inp["dup_dst"][t]] = inp["dup_src"][t].astype(np.uint32)
    return pos


# ----------------------------------------------------------------------------
# Row payloads: every byte is a hash of (tree, insert counter, field, offset),
# so a misplaced or stale byte anywhere in storage shows up in a comparison.
# ----------------------------------------------------------------------------
_M1, _M2, _M3, _M4 = 0x9E3779B1, 0x85EBCA6B, 0xC2B2AE35, 0x27D4EB2F
_F1, _F2 = 0x2C1B3C6D, 0x297A2D39


def _row_words_np(tree: int, counters: np.ndarray, fld: int, nwords: int) -> np.ndarray:
    c = np.asarray(counters, dtype=np.uint64).astype(np.uint32)[:, None]
    wi = np.arange(nwords, dtype=np.uint32)[None, :]
    const = np.uint32((tree * _M4 + fld * _M2) & 0xFFFFFFFF)
    x = c * np.uint32(_M1) + wi * np.uint32(_M3) + const
    x ^= x >> np.uint32(15)
    x *= np.uint32(_F1)
    x ^= x >> np.uint32(12)
    x *= np.uint32(_F2)
    x ^= x >> np.uint32(15)
    return x


def row_bytes(tree: int, counters, fld: int, nbytes: int) -> np.ndarray:
    """[len(counters), nbytes] uint8 payload of field ``fld`` for the given insert counters."""
    nwords = (nbytes + 3) // 4
    words = _row_words_np(tree, np.asarray(counters), fld, nwords)
    b = words.astype("<u4").view(np.uint8).reshape(len(words), nwords * 4)
    return np.ascontiguousarray(b[:, :nbytes])


def row_bytes_torch(tree: int, counters, fld: int, nbytes: int):
    """Same bytes as :func:`row_bytes`, computed with torch ops on ``counters.device``.

    Integer torch ops only (int64 arithmetic masked to 32 bits); used to fill
    multi-GiB payloads on the device without a host round trip.
    """
    import torch
    mask = 0xFFFFFFFF
    nwords = (nbytes + 3) // 4
    c = (counters.to(torch.int64) & mask)[:, None]
    wi = torch.arange(nwords, dtype=torch.int64, device=counters.device)[None, :]
    const = (tree * _M4 + fld * _M2) & mask
    x = (c * _M1 + wi * _M3 + const) & mask
    x = x ^ (x >> 15)
    x = (x * _F1) & mask
    x = x ^ (x >> 12)
    x = (x * _F2) & mask
    x = x ^ (x >> 15)
    sh = torch.tensor([0, 8, 16, 24], dtype=torch.int64, device=counters.device)
    b = ((x[:, :, None] >> sh) & 0xFF).to(torch.uint8).reshape(x.shape[0], nwords * 4)
    return b[:, :nbytes].contiguous()
