"""Seeded synthetic inputs shared by the CPU oracle's tests and the GPU tests/bench.

This module only *draws inputs*: hierarchical point-to-point cost matrices shaped like the
pairwise-RTT probe of a rented VM cluster (paper Fig. 2 / Section 3: latencies spread from a few
microseconds inside a rack to hundreds across racks; Section 2.1: rack/host hierarchy; Section 1:
the provider hands the VM list over in random order).  It contains none of the method's arithmetic
(no cost model, no move scoring, no shuffle used by the search) and imports neither the oracle nor
the GPU library.

Units: int32, RTT in 0.1 microsecond steps (or inverse-bandwidth units for the directed workload).
"""
from __future__ import annotations

import dataclasses
from typing import Optional, Tuple

import numpy as np

COST_MAX = (1 << 21) - 1          # largest matrix entry the library accepts
MATRIX_SEED_BASE = 20210528       # + workload id
SEARCH_SEED_BASE = 0xC0FFEE00     # + workload id


@dataclasses.dataclass(frozen=True)
class Workload:
    """One named workload: matrix shape + the amount of search/evaluation work done on it."""
    wid: int
    name: str
    n: int
    group_sizes: Tuple[int, ...]          # innermost first: (vms per host, hosts per rack) or (rack size,)
    level_ranges: Tuple[Tuple[int, int], ...]   # U[lo,hi] per hierarchy level, innermost first
    sigma: float                          # lognormal(0, sigma) multiplicative tenant noise; 0 = none
    symmetric: bool
    objective: str                        # "sum", "max", "sum_directed", "max_directed"
    restarts: int                         # 2-opt restarts (0 = none)
    batch: int                            # permutations scored by a batch call (0 = none)

    @property
    def matrix_seed(self) -> int:
        return MATRIX_SEED_BASE + self.wid

    @property
    def search_seed(self) -> int:
        return SEARCH_SEED_BASE + self.wid


# The five workloads (wid 1..5) and the batch-evaluation headline case (wid 6 reuses matrix 2).
WORKLOADS = {
    1: Workload(1, "C1_n8_two_racks", 8, (4,), ((200, 400), (800, 2000)), 0.0, True, "sum", 0, 4096),
    2: Workload(2, "C2_n64_sum", 64, (8,), ((200, 400), (800, 2000)), 0.25, True, "sum", 1024, 1 << 20),
    3: Workload(3, "C3_n64_max_directed", 64, (8,), ((500, 1250), (4000, 10000)), 0.25, False,
                "max_directed", 1024, 1 << 20),
    4: Workload(4, "C4_n256_sum", 256, (4, 8), ((50, 100), (200, 400), (800, 2000)), 0.3, True, "sum", 4096, 0),
    5: Workload(5, "C5_n1024_rd_and_sum", 1024, (4, 8), ((50, 100), (200, 400), (800, 2000)), 0.3, True,
                "sum", 256, 65536),
}


def hierarchy_levels(n: int, group_sizes: Tuple[int, ...]) -> np.ndarray:
    """level[a, b] = index of the innermost group that holds both a and b (0 = same innermost group,
    len(group_sizes) = only the whole cluster in common).  Nodes are numbered hierarchy-contiguously."""
    idx = np.arange(n)
    level = np.full((n, n), len(group_sizes), dtype=np.int64)
    span = 1
    spans = []
    for g in group_sizes:
        span *= g
        spans.append(span)
    for lv in range(len(group_sizes) - 1, -1, -1):
        grp = idx // spans[lv]
        level[grp[:, None] == grp[None, :]] = lv
    return level


def _finish(real: np.ndarray, rng: np.random.Generator, relabel: bool) -> np.ndarray:
    c = np.rint(real)
    c = np.maximum(c, 1.0)
    np.fill_diagonal(c, 0.0)
    if c.max() > COST_MAX:
        raise ValueError("generated cost exceeds COST_MAX")
    c = c.astype(np.int32)
    if relabel:
        p = rng.permutation(c.shape[0])
        c = np.ascontiguousarray(c[np.ix_(p, p)])
    return c


def hierarchical_matrix(n: int, group_sizes: Tuple[int, ...], level_ranges, sigma: float, symmetric: bool,
                        seed: int, relabel: bool = True, directed_ratio: Optional[int] = None) -> np.ndarray:
    """Draw an n x n int32 cost matrix.

    One base value per *unordered* pair from U[lo, hi] of the pair's hierarchy level.  Symmetric:
    the pair's base times one lognormal(0, sigma) factor, mirrored.  Asymmetric: each direction gets
    its own lognormal factor.  `directed_ratio` (used by the inverse-bandwidth workload): the base is
    drawn from the outermost range for every pair and divided by the ratio for pairs inside a rack.
    Then round, clamp to >= 1, zero the diagonal, and (relabel) shuffle node ids so rack membership is
    not visible in the numbering.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    level = hierarchy_levels(n, group_sizes)
    iu = np.triu_indices(n, 1)
    lv = level[iu]
    if directed_ratio is None:
        lo = np.array([r[0] for r in level_ranges], dtype=np.float64)[lv]
        hi = np.array([r[1] for r in level_ranges], dtype=np.float64)[lv]
        base_u = rng.uniform(lo, hi)
    else:
        lo, hi = level_ranges[-1]
        base_u = rng.uniform(lo, hi, size=lv.shape[0])
        base_u = np.where(lv < len(group_sizes), base_u / directed_ratio, base_u)
    real = np.zeros((n, n), dtype=np.float64)
    if symmetric:
        if sigma > 0:
            base_u = base_u * rng.lognormal(0.0, sigma, size=base_u.shape[0])
        real[iu] = base_u
        real = real + real.T
    else:
        f_up = rng.lognormal(0.0, sigma, size=base_u.shape[0]) if sigma > 0 else 1.0
        f_dn = rng.lognormal(0.0, sigma, size=base_u.shape[0]) if sigma > 0 else 1.0
        real[iu] = base_u * f_up
        real.T[iu] = base_u * f_dn
    return _finish(real, rng, relabel)


def make_matrix(wid: int) -> np.ndarray:
    """Cost matrix of workload `wid` (1..5)."""
    w = WORKLOADS[wid]
    if wid == 3:
        return hierarchical_matrix(w.n, w.group_sizes, w.level_ranges, w.sigma, False, w.matrix_seed,
                                   directed_ratio=8)
    return hierarchical_matrix(w.n, w.group_sizes, w.level_ranges, w.sigma, w.symmetric, w.matrix_seed)


def clean_hierarchy(n: int, rack: int, intra: int, cross: int) -> np.ndarray:
    """Noise-free two-level matrix, nodes numbered rack-contiguously: `intra` inside a rack,
    `cross` between racks, zero diagonal.  Used by closed-form checks."""
    level = hierarchy_levels(n, (rack,))
    c = np.where(level == 0, intra, cross).astype(np.int32)
    np.fill_diagonal(c, 0)
    return c


def random_matrix(n: int, seed: int, symmetric: bool, lo: int = 1, hi: int = 5000) -> np.ndarray:
    """Unstructured uniform integer matrix (zero diagonal) for property tests."""
    rng = np.random.Generator(np.random.PCG64(seed))
    c = rng.integers(lo, hi + 1, size=(n, n), dtype=np.int64)
    if symmetric:
        c = np.triu(c, 1)
        c = c + c.T
    np.fill_diagonal(c, 0)
    return c.astype(np.int32)


def random_perms(n: int, count: int, seed: int) -> np.ndarray:
    """`count` uniformly random permutations of range(n), int32 [count, n] (numpy's own shuffle;
    unrelated to the search's restart generator)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    base = np.tile(np.arange(n, dtype=np.int32), (count, 1))
    return rng.permuted(base, axis=1)


def probe_samples(base: np.ndarray, k: int, seed: int, interference: float = 0.2) -> np.ndarray:
    """Synthetic latency probes (stand-in for the echo-tool traces of Section 4.2): int32 [N, N, k], sample s of
    the ordered pair a -> b.  Each direction jitters a few percent above the pair's base RTT; a fraction
    `interference` of the samples is inflated by a heavy lognormal tail (queueing, noisy neighbours)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    n = base.shape[0]
    jitter = rng.gamma(2.0, 0.01, size=(n, n, k))
    hit = rng.random(size=(n, n, k)) < interference
    tail = rng.lognormal(0.5, 1.0, size=(n, n, k))
    direction = 1.0 + 0.02 * rng.random(size=(n, n, 1))
    real = base[:, :, None].astype(np.float64) * direction * (1.0 + jitter + hit * tail)
    out = np.minimum(np.rint(real), COST_MAX).astype(np.int32)
    out[np.arange(n), np.arange(n), :] = 0
    return out
