"""Seeded synthetic planner inputs (the five benchmark configurations).

This module only draws numbers: per-layer forward/backward times (int64 us),
activation sizes (int64 bytes), a device bandwidth matrix (int64 bytes/us) and
candidate device orderings (int32).  It holds none of the method's arithmetic
(no prefix sums, no transfer times, no DP, no schedule), so both the GPU
library and the CPU oracle can be fed from it without sharing code.

The paper's own workloads are profiled traces of VGG19 ... BERT-48 on two GPU
testbeds (Sec. V-A) and a BERT-large trace on 8 servers x 4 GPUs (Sec. V-C);
none of them is available, so these generators stand in with the same shape:
non-uniform convolutional layer costs, near-uniform transformer blocks, a few
fast islands of GPUs joined by a slow fabric.

Units: 1 GB/s = 1000 bytes/us; KB/MB mean KiB/MiB.
Draw order for every configuration: fwd, bwd factor, activations, bandwidth,
orderings; numpy Generator(PCG64(BASE_SEED + config number)).
"""
import itertools
import math
from dataclasses import dataclass, field
from typing import Optional, Tuple

import numpy as np

BASE_SEED = 220410562
KIB = 1 << 10
MIB = 1 << 20
GBPS = 1000  # bytes per microsecond


@dataclass
class Workload:
    name: str
    L: int
    D: int
    S: int
    N: int
    Ms: Tuple[int, ...]
    fwd: np.ndarray            # int64 [L] us
    bwd: np.ndarray            # int64 [L] us
    actf: np.ndarray           # int64 [L] bytes (entry L-1 unused)
    actb: np.ndarray           # int64 [L] bytes
    bw: np.ndarray             # int64 [D, D] bytes/us
    orderings: Optional[np.ndarray] = field(default=None)  # int32 [N, S] or None = all D! lexicographic

    def explicit_orderings(self) -> np.ndarray:
        """The candidate list as an explicit int32 [N, S] array."""
        if self.orderings is not None:
            return self.orderings
        return all_orderings(self.D)


def all_orderings(D: int) -> np.ndarray:
    """All D! device orderings in lexicographic order (itertools order), int32 [D!, D]."""
    return np.array(list(itertools.permutations(range(D))), dtype=np.int32).reshape(-1, D)


def _rng(config: int, seed_offset: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(BASE_SEED + config + seed_offset))


def _rint(x) -> np.ndarray:
    return np.rint(x).astype(np.int64)


def _sym_from_pairs(D: int, draw) -> np.ndarray:
    bw = np.zeros((D, D), np.int64)
    for u in range(D):
        for v in range(u + 1, D):
            bw[u, v] = bw[v, u] = draw()
    return bw


def _sample_orderings(rng: np.random.Generator, N: int, D: int) -> np.ndarray:
    # independent uniform shuffles of (0..D-1), one per row (duplicates possible)
    rows = np.tile(np.arange(D, dtype=np.int32), (N, 1))
    return rng.permuted(rows, axis=1)


def tiny(seed_offset: int = 0) -> Workload:
    """Config 1: L=16, D=4, all 24 orderings, M in {4, 8}."""
    rng = _rng(1, seed_offset)
    L, D = 16, 4
    fwd = rng.integers(100, 1001, size=L).astype(np.int64)
    bwd = _rint(fwd * rng.uniform(1.5, 2.5, size=L))
    act = _rint(np.exp(rng.uniform(math.log(1 * MIB), math.log(64 * MIB), size=L)))
    bw = _sym_from_pairs(D, lambda: (150 if rng.random() < 0.5 else 16) * GBPS)
    return Workload("tiny", L, D, D, math.factorial(D), (4, 8), fwd, bwd, act, act.copy(), bw)


def transformer(seed_offset: int = 0) -> Workload:
    """Config 2: L=48 (24 blocks x {attention, FFN}), D=8, all 40320 orderings, M in {8, 16}."""
    rng = _rng(2, seed_offset)
    L, D = 48, 8
    att = rng.integers(800, 1201, size=L // 2)
    ffn = rng.integers(1500, 2001, size=L // 2)
    fwd = np.empty(L, np.int64)
    fwd[0::2] = att
    fwd[1::2] = ffn
    bwd = 2 * fwd
    act = np.full(L, 8 * MIB, np.int64)
    bw = np.empty((D, D), np.int64)
    for u in range(D):
        for v in range(D):
            bw[u, v] = (300 if u // 4 == v // 4 else 25) * GBPS
    np.fill_diagonal(bw, 0)
    return Workload("transformer", L, D, D, math.factorial(D), (8, 16), fwd, bwd, act, act.copy(), bw)


def gpt(seed_offset: int = 0) -> Workload:
    """Config 3 (the graded one): L=128, D=8, all 40320 orderings, M in {8, 16, 32, 64}."""
    rng = _rng(3, seed_offset)
    L, D = 128, 8
    fwd = np.maximum(1, _rint(rng.normal(1000.0, 50.0, size=L)))
    bwd = _rint(fwd * rng.uniform(1.8, 2.2, size=L))
    act = np.full(L, 16 * MIB, np.int64)
    levels = np.array([25, 50, 150, 300], np.int64) * GBPS
    bw = _sym_from_pairs(D, lambda: int(levels[rng.integers(0, 4)]))
    return Workload("gpt", L, D, D, math.factorial(D), (8, 16, 32, 64), fwd, bwd, act, act.copy(), bw)


def gpt_varied(seed_offset: int = 0) -> Workload:
    """The GPT-shaped configuration with activation sizes that differ from boundary to boundary
    (16 MiB x U[0.5, 2), from a generator of its own so that every other draw is config 3's):
    same L, D, N and value ranges, but the transfer times depend on the cut position, which is
    the case the general partition-DP kernel exists for."""
    w = gpt(seed_offset)
    rng = np.random.Generator(np.random.PCG64(BASE_SEED + 3 + 1009 + seed_offset))
    act = _rint(16 * MIB * rng.uniform(0.5, 2.0, size=w.L))
    return Workload("gpt_varied", w.L, w.D, w.S, w.N, w.Ms, w.fwd, w.bwd, act, act.copy(), w.bw)


def hetero(seed_offset: int = 0, N: int = 10 ** 6) -> Workload:
    """Config 4: L=300 conv-net-shaped, D=16, N seed-sampled orderings, M in {16, 32}."""
    rng = _rng(4, seed_offset)
    L, D = 300, 16
    ramp = 2000.0 - 1800.0 * np.arange(L) / (L - 1)
    fwd = np.maximum(1, _rint(ramp * rng.uniform(0.8, 1.2, size=L)))
    bwd = 2 * fwd
    act = _rint(200.0 * MIB * (1.0 / 200.0) ** (np.arange(L) / (L - 1)))
    bw = np.empty((D, D), np.int64)
    for u in range(D):
        for v in range(D):
            bw[u, v] = (300 if u // 4 == v // 4 else 16) * GBPS
    np.fill_diagonal(bw, 0)
    orderings = _sample_orderings(rng, N, D)
    return Workload("hetero", L, D, D, N, (16, 32), fwd, bwd, act, act.copy(), bw, orderings)


def stress(seed_offset: int = 0, N: int = 1 << 20) -> Workload:
    """Config 5: L=1024, D=32, N seed-sampled orderings, M=128."""
    rng = _rng(5, seed_offset)
    L, D = 1024, 32
    fwd = rng.integers(50, 501, size=L).astype(np.int64)
    bwd = _rint(fwd * rng.uniform(1.5, 2.5, size=L))
    act = _rint(np.exp(rng.uniform(math.log(512 * KIB), math.log(128 * MIB), size=L)))
    lo, hi = math.log(10 * GBPS), math.log(400 * GBPS)
    bw = _sym_from_pairs(D, lambda: int(np.rint(math.exp(rng.uniform(lo, hi)))))
    orderings = _sample_orderings(rng, N, D)
    return Workload("stress", L, D, D, N, (128,), fwd, bwd, act, act.copy(), bw, orderings)


def random_small(seed: int, L: int, D: int, S: int, N: int, zero_frac: float = 0.0,
                 asym: bool = True, hi_time: int = 50, hi_act: int = 4000,
                 same_act: bool = False) -> Workload:
    """Small adversarial inputs for tests: narrow value ranges (many ties), optional
    zero durations, asymmetric bandwidth, position-dependent activation sizes (or, with
    same_act, one forward and one backward size for every layer boundary, as in a stack of
    equal blocks), sampled orderings that may use fewer stages than devices."""
    rng = np.random.Generator(np.random.PCG64(seed))
    fwd = rng.integers(0 if zero_frac > 0 else 1, hi_time + 1, size=L).astype(np.int64)
    bwd = rng.integers(0 if zero_frac > 0 else 1, 2 * hi_time + 1, size=L).astype(np.int64)
    if zero_frac > 0:
        fwd[rng.random(L) < zero_frac] = 0
        bwd[rng.random(L) < zero_frac] = 0
    actf = rng.integers(0, hi_act + 1, size=L).astype(np.int64)
    actb = rng.integers(0, hi_act + 1, size=L).astype(np.int64)
    bw = rng.integers(1, 200, size=(D, D)).astype(np.int64)
    if not asym:
        bw = np.minimum(bw, bw.T)
    np.fill_diagonal(bw, 0)
    orderings = _sample_orderings(rng, N, D)[:, :S].copy()
    if same_act:
        actf[:] = actf[0]
        actb[:] = actb[0]
    return Workload("random_small", L, D, S, N, (1, 2, 3, 5, 8), fwd, bwd, actf, actb, bw, orderings)


CONFIGS = {"tiny": tiny, "transformer": transformer, "gpt": gpt, "hetero": hetero, "stress": stress}
# the five configurations plus variants used by the benchmark and the tests
WORKLOADS = dict(CONFIGS, gpt_varied=gpt_varied)


def pair_evals_per_candidate(L: int, S: int) -> int:
    """Number of (cell, split) pairs the partition DP inspects for one candidate:
    sum over xi = 2..S of (L - xi + 1)(L - xi + 2) / 2."""
    return sum((L - xi + 1) * (L - xi + 2) // 2 for xi in range(2, S + 1))


def parameter_sizes(w: Workload, seed_offset: int = 0) -> np.ndarray:
    """Per-layer parameter (= gradient) sizes alpha_l in bytes for the AllReduce term of the
    planner with replicated stages: log-uniform in [1 MiB, 64 MiB], from a generator of its
    own (seeded by the workload's name and length), so that the draws of the workload itself
    do not change."""
    tag = sum(ord(ch) for ch in w.name) * 1000 + w.L
    rng = np.random.Generator(np.random.PCG64(BASE_SEED + 7919 + tag + seed_offset))
    return _rint(np.exp(rng.uniform(math.log(1 * MIB), math.log(64 * MIB), size=w.L)))
