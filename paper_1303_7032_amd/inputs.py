"""Seeded synthetic workloads for the clustered associative memory (GBNN).

This module only *draws inputs*: random messages, which stored message each probe is
made from, which clusters of it are erased, and the one-hot-per-cluster byte image of a
probe (the data format of Section II-A: neuron i = c*L + l, one active neuron per known
cluster).  It contains none of the method's arithmetic (no storing, no scoring, no
selection) and is the only code shared by the CPU oracle's tests and the GPU path's
tests / benchmark.

The paper's experiments (Section VII) use i.i.d. uniform random messages, store M of
them and probe with partially erased copies of stored ones; that is what is drawn here.
Randomness is a 64-bit counter-based mixer (the splitmix64 finaliser) so that every
value is a pure function of (seed, stream, index) and can be regenerated anywhere.

Symbols are 0-based: a message is C integers in [0, L).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Tuple

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _mix64(z: np.ndarray) -> np.ndarray:
    """splitmix64 output function on an array of uint64 (wrap-around arithmetic)."""
    z = np.asarray(z, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def rnd(seed: int, stream: int, index) -> np.ndarray:
    """Counter-based uniform 64-bit integers: a pure function of (seed, stream, index)."""
    idx = np.asarray(index, dtype=np.uint64)
    with np.errstate(over="ignore"):
        key = _mix64(np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + _GOLDEN * np.uint64(stream + 1))
        return _mix64(key + _GOLDEN * (idx + np.uint64(1)))


def make_messages(C: int, L: int, M: int, seed: int) -> np.ndarray:
    """M messages of C symbols, each symbol i.i.d. uniform in [0, L) -> int32[M][C].

    `rnd % L` is exactly uniform when L is a power of two (every benchmark shape) and
    has a bias below L / 2**64 otherwise.  Duplicate messages are allowed.
    """
    idx = np.arange(M * C, dtype=np.uint64)
    return (rnd(seed, 0, idx) % np.uint64(L)).astype(np.int32).reshape(M, C)


def make_probe_plan(C: int, M: int, K: int, e: int, seed: int) -> Tuple[np.ndarray, np.ndarray]:
    """Which stored message each probe comes from and which clusters are erased.

    Returns (q, erased): q int64[K], drawn uniformly *with replacement* from [0, M);
    erased bool[K][C] with exactly e True per row, a uniformly random e-subset (the
    first e entries of a Fisher-Yates shuffle of 0..C-1).
    """
    if not (0 <= e <= C):
        raise ValueError("need 0 <= e <= C")
    k = np.arange(K, dtype=np.uint64)
    q = (rnd(seed, 1, k) % np.uint64(max(M, 1))).astype(np.int64)
    perm = np.tile(np.arange(C, dtype=np.int64), (K, 1))
    rows = np.arange(K)
    for t in range(e):
        r = t + (rnd(seed, 2, k * np.uint64(C) + np.uint64(t)) % np.uint64(C - t)).astype(np.int64)
        a = perm[rows, t].copy()
        perm[rows, t] = perm[rows, r]
        perm[rows, r] = a
    erased = np.zeros((K, C), dtype=bool)
    for t in range(e):
        erased[rows, perm[:, t]] = True
    return q, erased


def active_neurons(msgs: np.ndarray, L: int) -> np.ndarray:
    """Flat neuron index c*L + m_c of every symbol: int64[...][C]."""
    msgs = np.asarray(msgs)
    C = msgs.shape[-1]
    return np.arange(C, dtype=np.int64) * L + msgs.astype(np.int64)


def one_hot(msgs: np.ndarray, L: int, erased: np.ndarray | None = None) -> np.ndarray:
    """Byte image of messages: uint8[K][C*L], 1 at c*L + m_c for every non-erased cluster."""
    msgs = np.atleast_2d(np.asarray(msgs))
    K, C = msgs.shape
    V = np.zeros((K, C * L), dtype=np.uint8)
    idx = active_neurons(msgs, L)
    if erased is None:
        V[np.arange(K)[:, None], idx] = 1
    else:
        kk, cc = np.nonzero(~np.asarray(erased, dtype=bool))
        V[kk, idx[kk, cc]] = 1
    return V


@dataclass(frozen=True)
class Workload:
    """One benchmark / parity configuration (shapes of the paper's Scenarios 1 and 2)."""
    name: str
    C: int
    L: int
    M: int
    K: int
    e: int
    rules: Tuple[str, ...]
    gamma: int
    max_iters: int
    seed: int
    note: str = ""

    @property
    def n(self) -> int:
        return self.C * self.L

    def density(self) -> float:
        """Expected inter-cluster edge density 1 - (1 - 1/L^2)^M of M uniform messages."""
        return 1.0 - (1.0 - 1.0 / (self.L * self.L)) ** self.M

    def messages(self) -> np.ndarray:
        return make_messages(self.C, self.L, self.M, self.seed)

    def probe_plan(self, K: int | None = None) -> Tuple[np.ndarray, np.ndarray]:
        """(q, erased) for the first K probes (the plan of probe k does not depend on K)."""
        return make_probe_plan(self.C, self.M, self.K if K is None else K, self.e, self.seed)

    def probes(self, msgs: np.ndarray, K: int | None = None):
        """(q, erased, V0 uint8[K][n]) on the host."""
        q, erased = self.probe_plan(K)
        return q, erased, one_hot(msgs[q], self.L, erased)


_BASE_SEED = 0x13037032

WORKLOADS: Dict[str, Workload] = {w.name: w for w in [
    Workload("cfg1", 4, 16, 50, 200, 2, ("sum_of_sum", "sum_of_max", "hybrid"), 1, 4, _BASE_SEED + 1,
             "tiny; correctness only"),
    Workload("cfg2", 8, 128, 5_000, 65_536, 4, ("sum_of_sum",), 1, 4, _BASE_SEED + 2,
             "Scenario-1 shape, sum-of-sum with memory effect 1"),
    Workload("cfg3", 8, 256, 20_000, 65_536, 4, ("sum_of_max", "hybrid"), 1, 20, _BASE_SEED + 3,
             "headline shape: c=8, l=256"),
    Workload("cfg4_m10k", 8, 256, 10_000, 262_144, 4, ("hybrid", "sum_of_max"), 1, 20, _BASE_SEED + 4),
    Workload("cfg4_m30k", 8, 256, 30_000, 262_144, 4, ("hybrid", "sum_of_max"), 1, 20, _BASE_SEED + 5),
    Workload("cfg4_m50k", 8, 256, 50_000, 262_144, 4, ("hybrid", "sum_of_max"), 1, 20, _BASE_SEED + 6),
    Workload("cfg5", 16, 512, 100_000, 131_072, 8, ("sum_of_max", "hybrid"), 1, 20, _BASE_SEED + 7,
             "Scenario-2 shape; W is 8 MiB bit-packed"),
]}
