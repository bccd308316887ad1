"""ctypes access to the CPU oracle (oracle/cc_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the benchmark's CPU-baseline leg.
The GPU library never imports this package and this package never imports the GPU library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cc_oracle.c")
_LIB = os.path.join(_HERE, "libcc_oracle.so")

SUM, MAX, SUM_DIRECTED, MAX_DIRECTED = 0, 1, 2, 3
OBJECTIVES = {"sum": SUM, "max": MAX, "sum_directed": SUM_DIRECTED, "max_directed": MAX_DIRECTED}


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 (plain C, no intrinsics)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-Wall", "-Wextra", "-fPIC", "-shared", _SRC, "-o", _LIB])
    return _LIB


_lib = None


def _declare(path: str) -> ctypes.CDLL:
    """Loads an oracle library and declares its prototypes (also used by the mutation tests on altered builds)."""
    lib = ctypes.CDLL(path)
    i32, i64, u64, u32 = ctypes.c_int32, ctypes.c_int64, ctypes.c_uint64, ctypes.c_uint32
    p = ctypes.c_void_p
    lib.cco_splitmix64_at.restype = u64
    lib.cco_splitmix64_at.argtypes = [u64, u64]
    lib.cco_init_tour.restype = None
    lib.cco_init_tour.argtypes = [u64, u32, i32, p]
    lib.cco_init_tours.restype = None
    lib.cco_init_tours.argtypes = [u64, i32, i64, i64, p]
    lib.cco_ring_cost.restype = i64
    lib.cco_ring_cost.argtypes = [p, i32, p, i32]
    lib.cco_rd_cost.restype = i64
    lib.cco_rd_cost.argtypes = [p, i32, p]
    lib.cco_ring_cost_batch.restype = ctypes.c_int
    lib.cco_ring_cost_batch.argtypes = [p, i32, i32, p, i64, p]
    lib.cco_rd_cost_batch.restype = ctypes.c_int
    lib.cco_rd_cost_batch.argtypes = [p, i32, p, i64, p]
    lib.cco_apply_move.restype = None
    lib.cco_apply_move.argtypes = [p, i32, i32, i32, i32]
    lib.cco_move_id.restype = i64
    lib.cco_move_id.argtypes = [i32, i32, i32, i32, i32]
    lib.cco_move_value_by_definition.restype = i64
    lib.cco_move_value_by_definition.argtypes = [p, i32, i32, p, i32, i32, i32]
    lib.cco_neighbourhood_size.restype = i64
    lib.cco_neighbourhood_size.argtypes = [i32, i32]
    lib.cco_all_move_values.restype = ctypes.c_int
    lib.cco_all_move_values.argtypes = [p, i32, i32, p, p]
    lib.cco_2opt_descend.restype = ctypes.c_int
    lib.cco_2opt_descend.argtypes = [p, i32, i32, p, p, p, i32, p, i32]
    lib.cco_2opt_restarts.restype = ctypes.c_int
    lib.cco_2opt_restarts.argtypes = [p, i32, i32, u64, i64, i64, p, p, p, p]
    lib.cco_2opt_search.restype = ctypes.c_int
    lib.cco_2opt_search.argtypes = [p, i32, i32, i32, u64, p, p, p, p, p, p, p]
    lib.cco_exhaustive_rings.restype = ctypes.c_int
    lib.cco_exhaustive_rings.argtypes = [p, i32, i32, i32, p, p, p, p, p, i64]
    lib.cco_apply_swap.restype = None
    lib.cco_apply_swap.argtypes = [p, i32, i32]
    lib.cco_rd_swap_value_by_definition.restype = i64
    lib.cco_rd_swap_value_by_definition.argtypes = [p, i32, p, i32, i32]
    lib.cco_rd_swap_neighbourhood_size.restype = i64
    lib.cco_rd_swap_neighbourhood_size.argtypes = [i32]
    lib.cco_rd_swap_all_values.restype = ctypes.c_int
    lib.cco_rd_swap_all_values.argtypes = [p, i32, p, p]
    lib.cco_rd_swap_descend.restype = ctypes.c_int
    lib.cco_rd_swap_descend.argtypes = [p, i32, p, p, p, i32, p, i32]
    lib.cco_rd_swap_restarts.restype = ctypes.c_int
    lib.cco_rd_swap_restarts.argtypes = [p, i32, u64, i64, i64, p, p, p, p]
    lib.cco_bcube_cost.restype = i64
    lib.cco_bcube_cost.argtypes = [p, i32, i32, p]
    lib.cco_bcube_cost_batch.restype = ctypes.c_int
    lib.cco_bcube_cost_batch.argtypes = [p, i32, i32, p, i64, p]
    lib.cco_sa_proposal.restype = None
    lib.cco_sa_proposal.argtypes = [u64, ctypes.c_uint32, ctypes.c_uint32, i32, p, p, p]
    lib.cco_sa_log2_fix.restype = i32
    lib.cco_sa_log2_fix.argtypes = [i32]
    lib.cco_sa_accepts.restype = ctypes.c_int
    lib.cco_sa_accepts.argtypes = [i64, i64, i64, i32]
    lib.cco_sa_chain.restype = ctypes.c_int
    lib.cco_sa_chain.argtypes = [p, i32, p, i64, i32, i32, u64, ctypes.c_uint32, i32, p, p, p, p, p]
    lib.cco_sa_chains.restype = ctypes.c_int
    lib.cco_sa_chains.argtypes = [p, i32, i64, i32, i32, u64, i64, i64, p, p, p, p]
    lib.cco_dbt_tree_cost.restype = i64
    lib.cco_dbt_tree_cost.argtypes = [p, i32, p, i32]
    lib.cco_dbt_cost.restype = i64
    lib.cco_dbt_cost.argtypes = [p, i32, p]
    lib.cco_dbt_cost_batch.restype = ctypes.c_int
    lib.cco_dbt_cost_batch.argtypes = [p, i32, p, i64, p]
    lib.cco_bcube_cost_weighted_batch.restype = ctypes.c_int
    lib.cco_bcube_cost_weighted_batch.argtypes = [p, i32, i32, p, p, i64, p]
    lib.cco_sa_rd_proposal.restype = None
    lib.cco_sa_rd_proposal.argtypes = [u64, ctypes.c_uint32, ctypes.c_uint32, i32, p, p, p]
    lib.cco_sa_rd_chain.restype = ctypes.c_int
    lib.cco_sa_rd_chain.argtypes = [p, i32, p, i64, i32, i32, u64, ctypes.c_uint32, p, p, p, p, p]
    lib.cco_sa_rd_chains.restype = ctypes.c_int
    lib.cco_sa_rd_chains.argtypes = [p, i32, i64, i32, i32, u64, i64, i64, p, p, p, p]
    lib.cco_cost_matrix_from_probes.restype = ctypes.c_int
    lib.cco_cost_matrix_from_probes.argtypes = [p, i32, i32, i32, i32, p]
    lib.cco_oropt_is_move.restype = ctypes.c_int
    lib.cco_oropt_is_move.argtypes = [i32, i32, i32, i32, i32]
    lib.cco_oropt_move_id.restype = i64
    lib.cco_oropt_move_id.argtypes = [i32, i32, i32, i32, i32]
    lib.cco_oropt_apply.restype = None
    lib.cco_oropt_apply.argtypes = [p, i32, i32, i32, i32, i32]
    lib.cco_oropt_value_by_definition.restype = i64
    lib.cco_oropt_value_by_definition.argtypes = [p, i32, p, i32, i32, i32, i32]
    lib.cco_oropt_neighbourhood_size.restype = i64
    lib.cco_oropt_neighbourhood_size.argtypes = [i32]
    lib.cco_oropt_all_values.restype = ctypes.c_int
    lib.cco_oropt_all_values.argtypes = [p, i32, p, p]
    lib.cco_local_classes_ok.restype = ctypes.c_int
    lib.cco_local_classes_ok.argtypes = [i32, i32]
    lib.cco_local_descend.restype = ctypes.c_int
    lib.cco_local_descend.argtypes = [p, i32, i32, i32, p, p, p, i32, p, i32]
    lib.cco_local_restarts.restype = ctypes.c_int
    lib.cco_local_restarts.argtypes = [p, i32, i32, i32, u64, i64, i64, p, p, p, p]
    return lib


def _L():
    """The oracle library: built from cc_oracle.c on first use, or, when CC_ORACLE_LIB names a file, that build of
    the same source (the sanitizer test points it at an instrumented one)."""
    global _lib
    if _lib is None:
        _lib = _declare(os.environ.get("CC_ORACLE_LIB") or build())
    return _lib


def _mat(c) -> np.ndarray:
    c = np.ascontiguousarray(c, dtype=np.int32)
    assert c.ndim == 2 and c.shape[0] == c.shape[1]
    return c


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check(rc: int):
    if rc != 0:
        raise RuntimeError({-1: "oracle: invalid argument", -2: "oracle: matrix not symmetric",
                            -3: "oracle: out of memory"}.get(rc, f"oracle error {rc}"))


def splitmix64_at(seed: int, n: int) -> int:
    return int(_L().cco_splitmix64_at(seed & (2**64 - 1), n & (2**64 - 1)))


def init_tours(seed: int, n: int, count: int, first: int = 0) -> np.ndarray:
    out = np.empty((count, n), dtype=np.int32)
    _L().cco_init_tours(seed, n, first, count, _ptr(out))
    return out


def ring_cost(c, perm, objective: int = SUM) -> int:
    c = _mat(c)
    perm = np.ascontiguousarray(perm, dtype=np.int32)
    return int(_L().cco_ring_cost(_ptr(c), c.shape[0], _ptr(perm), objective))


def rd_cost(c, perm) -> int:
    c = _mat(c)
    perm = np.ascontiguousarray(perm, dtype=np.int32)
    return int(_L().cco_rd_cost(_ptr(c), c.shape[0], _ptr(perm)))


def ring_cost_batch(c, perms, objective: int = SUM) -> np.ndarray:
    c = _mat(c)
    perms = np.ascontiguousarray(perms, dtype=np.int32).reshape(-1, c.shape[0])
    out = np.empty(perms.shape[0], dtype=np.int64)
    _check(_L().cco_ring_cost_batch(_ptr(c), c.shape[0], objective, _ptr(perms), perms.shape[0], _ptr(out)))
    return out


def rd_cost_batch(c, perms) -> np.ndarray:
    c = _mat(c)
    perms = np.ascontiguousarray(perms, dtype=np.int32).reshape(-1, c.shape[0])
    out = np.empty(perms.shape[0], dtype=np.int64)
    _check(_L().cco_rd_cost_batch(_ptr(c), c.shape[0], _ptr(perms), perms.shape[0], _ptr(out)))
    return out


def apply_move(t, i: int, j: int, o: int = 0) -> np.ndarray:
    u = np.array(t, dtype=np.int32, copy=True)
    _L().cco_apply_move(_ptr(u), u.shape[0], i, j, o)
    return u


def move_id(n: int, objective: int, i: int, j: int, o: int = 0) -> int:
    return int(_L().cco_move_id(n, objective, i, j, o))


def move_value_by_definition(c, objective: int, t, i: int, j: int, o: int = 0) -> int:
    c = _mat(c)
    t = np.ascontiguousarray(t, dtype=np.int32)
    return int(_L().cco_move_value_by_definition(_ptr(c), c.shape[0], objective, _ptr(t), i, j, o))


def neighbourhood_size(n: int, objective: int) -> int:
    return int(_L().cco_neighbourhood_size(n, objective))


def moves_in_id_order(n: int, objective: int):
    """(i, j, o) of every move, in increasing id order."""
    directed = bool(objective & 2)
    out = []
    for i in range(1, n - 1):
        for j in range(i + 1, n):
            if (i, j) == (1, n - 1):
                continue
            for o in range(2 if directed else 1):
                out.append((i, j, o))
    return out


def all_move_values(c, objective: int, t) -> np.ndarray:
    c = _mat(c)
    t = np.ascontiguousarray(t, dtype=np.int32)
    out = np.empty(neighbourhood_size(c.shape[0], objective), dtype=np.int64)
    _check(_L().cco_all_move_values(_ptr(c), c.shape[0], objective, _ptr(t), _ptr(out)))
    return out


def descend(c, objective: int, t, use_definition: bool = False, trace_cap: int = 0):
    """One 2-opt descent from tour t. Returns (final tour, cost, applied moves, trace of move ids)."""
    c = _mat(c)
    u = np.array(t, dtype=np.int32, copy=True)
    cost = ctypes.c_int64(0)
    moves = ctypes.c_int32(0)
    trace = np.zeros(max(trace_cap, 1), dtype=np.int64)
    _check(_L().cco_2opt_descend(_ptr(c), c.shape[0], objective, _ptr(u), ctypes.byref(cost), ctypes.byref(moves),
                                 1 if use_definition else 0, _ptr(trace), trace_cap))
    return u, int(cost.value), int(moves.value), trace[:min(trace_cap, moves.value)]


def restarts(c, objective: int, seed: int, r0: int, r1: int, init: Optional[np.ndarray] = None):
    """Restarts [r0, r1): returns (costs int64[r1-r0], tours int32[r1-r0, N], moves int32[r1-r0])."""
    c = _mat(c)
    n = c.shape[0]
    k = r1 - r0
    costs = np.empty(k, dtype=np.int64)
    tours = np.empty((k, n), dtype=np.int32)
    moves = np.empty(k, dtype=np.int32)
    if init is not None:
        init = np.ascontiguousarray(init, dtype=np.int32)
    _check(_L().cco_2opt_restarts(_ptr(c), n, objective, seed, r0, r1, _ptr(init), _ptr(costs), _ptr(tours),
                                  _ptr(moves)))
    return costs, tours, moves


def restarts_parallel(c, objective: int, seed: int, r0: int, r1: int, threads: int,
                      init: Optional[np.ndarray] = None):
    """The same single-threaded routine over disjoint restart ranges on `threads` host threads
    (ctypes releases the GIL).  Results are identical to restarts()."""
    threads = max(1, min(threads, r1 - r0))
    edges = np.linspace(r0, r1, threads * 4 + 1).astype(np.int64)
    spans = [(int(a), int(b)) for a, b in zip(edges[:-1], edges[1:]) if b > a]
    with ThreadPoolExecutor(max_workers=threads) as ex:
        parts = list(ex.map(lambda s: restarts(c, objective, seed, s[0], s[1], init), spans))
    return (np.concatenate([p[0] for p in parts]), np.concatenate([p[1] for p in parts]),
            np.concatenate([p[2] for p in parts]))


def search(c, objective: int, n_restarts: int, seed: int, init: Optional[np.ndarray] = None):
    """Whole multi-start search. Returns dict(best_perm, best_cost, best_restart, costs, tours, moves)."""
    c = _mat(c)
    n = c.shape[0]
    best = np.empty(n, dtype=np.int32)
    bc = ctypes.c_int64(0)
    br = ctypes.c_int32(0)
    costs = np.empty(n_restarts, dtype=np.int64)
    tours = np.empty((n_restarts, n), dtype=np.int32)
    moves = np.empty(n_restarts, dtype=np.int32)
    if init is not None:
        init = np.ascontiguousarray(init, dtype=np.int32)
    _check(_L().cco_2opt_search(_ptr(c), n, objective, n_restarts, seed, _ptr(init), _ptr(best), ctypes.byref(bc),
                                ctypes.byref(br), _ptr(costs), _ptr(tours), _ptr(moves)))
    return dict(best_perm=best, best_cost=int(bc.value), best_restart=int(br.value), costs=costs, tours=tours,
                moves=moves)


def exhaustive_rings(c, objective: int = SUM, half_only: bool = True, keep_all: bool = False):
    """All rings with t[0]=0 (N <= 12). Returns dict(count, best_cost, best_ring[, rings, costs])."""
    c = _mat(c)
    n = c.shape[0]
    count = ctypes.c_int64(0)
    bc = ctypes.c_int64(0)
    best = np.empty(n, dtype=np.int32)
    rings = costs = None
    cap = 0
    if keep_all:
        import math
        cap = math.factorial(n - 1) // (2 if (half_only and n > 2) else 1)
        rings = np.empty((cap, n), dtype=np.int32)
        costs = np.empty(cap, dtype=np.int64)
    _check(_L().cco_exhaustive_rings(_ptr(c), n, objective, 1 if half_only else 0, ctypes.byref(count),
                                     ctypes.byref(bc), _ptr(best), _ptr(rings), _ptr(costs), cap))
    out = dict(count=int(count.value), best_cost=int(bc.value), best_ring=best)
    if keep_all:
        out["rings"], out["costs"] = rings, costs
    return out


# ------------------------------------------------------------------ pair-swap search, halving-doubling model
def rd_swap_value_by_definition(c, t, p: int, q: int) -> int:
    c = _mat(c)
    t = np.ascontiguousarray(t, dtype=np.int32)
    return int(_L().cco_rd_swap_value_by_definition(_ptr(c), c.shape[0], _ptr(t), p, q))


def rd_swap_all_values(c, t) -> np.ndarray:
    """Value of every swap (p, q), p < q, in increasing id order (delta tier)."""
    c = _mat(c)
    t = np.ascontiguousarray(t, dtype=np.int32)
    n = c.shape[0]
    out = np.empty(n * (n - 1) // 2, dtype=np.int64)
    _check(_L().cco_rd_swap_all_values(_ptr(c), n, _ptr(t), _ptr(out)))
    return out


def rd_swap_descend(c, t, use_definition: bool = False, trace_cap: int = 0):
    c = _mat(c)
    u = np.array(t, dtype=np.int32, copy=True)
    cost = ctypes.c_int64(0)
    moves = ctypes.c_int32(0)
    trace = np.zeros(max(trace_cap, 1), dtype=np.int64)
    _check(_L().cco_rd_swap_descend(_ptr(c), c.shape[0], _ptr(u), ctypes.byref(cost), ctypes.byref(moves),
                                    1 if use_definition else 0, _ptr(trace), trace_cap))
    return u, int(cost.value), int(moves.value), trace[:min(trace_cap, moves.value)]


def rd_swap_restarts(c, seed: int, r0: int, r1: int, init: Optional[np.ndarray] = None):
    c = _mat(c)
    n = c.shape[0]
    k = r1 - r0
    costs = np.empty(k, dtype=np.int64)
    tours = np.empty((k, n), dtype=np.int32)
    moves = np.empty(k, dtype=np.int32)
    if init is not None:
        init = np.ascontiguousarray(init, dtype=np.int32)
    _check(_L().cco_rd_swap_restarts(_ptr(c), n, seed, r0, r1, _ptr(init), _ptr(costs), _ptr(tours), _ptr(moves)))
    return costs, tours, moves


def rd_swap_search(c, n_restarts: int, seed: int, init: Optional[np.ndarray] = None):
    costs, tours, moves = rd_swap_restarts(c, seed, 0, n_restarts, init)
    k = int(np.argmin(costs))
    return dict(best_perm=tours[k].copy(), best_cost=int(costs[k]), best_restart=k, costs=costs, tours=tours,
                moves=moves)


# ------------------------------------------------------------------------------------------ BCube cost model
def bcube_cost(c, base: int, perm) -> int:
    c = _mat(c)
    perm = np.ascontiguousarray(perm, dtype=np.int32)
    return int(_L().cco_bcube_cost(_ptr(c), c.shape[0], base, _ptr(perm)))


def bcube_cost_batch(c, base: int, perms) -> np.ndarray:
    c = _mat(c)
    perms = np.ascontiguousarray(perms, dtype=np.int32).reshape(-1, c.shape[0])
    out = np.empty(perms.shape[0], dtype=np.int64)
    _check(_L().cco_bcube_cost_batch(_ptr(c), c.shape[0], base, _ptr(perms), perms.shape[0], _ptr(out)))
    return out


# ------------------------------------------------------------------------------------------ simulated annealing
SA_MAX_STEPS = 1 << 24


def sa_proposal(seed: int, r: int, s: int, n: int):
    """(a, b, u): the two ring edges and the acceptance draw of step s of chain r."""
    a, b, u = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    _L().cco_sa_proposal(seed, r, s, n, ctypes.byref(a), ctypes.byref(b), ctypes.byref(u))
    return a.value, b.value, u.value


def sa_log2_fix(u: int) -> int:
    return int(_L().cco_sa_log2_fix(u))


def sa_accepts(delta: int, steps: int, num: int, u: int) -> bool:
    return bool(_L().cco_sa_accepts(delta, steps, num, u))


def sa_chain(c, t, steps: int, t_start: int, t_end: int, seed: int, r: int, use_definition: bool = False,
             trace: bool = False):
    c = _mat(c)
    n = c.shape[0]
    t = np.array(t, dtype=np.int32, copy=True)
    best_tour = np.empty(n, dtype=np.int32)
    best, final = ctypes.c_int64(), ctypes.c_int64()
    acc = ctypes.c_int32()
    tr = np.empty(steps, dtype=np.int64) if trace else None
    _check(_L().cco_sa_chain(_ptr(c), n, _ptr(t), steps, t_start, t_end, seed, r, int(use_definition), _ptr(best_tour),
                             ctypes.byref(best), ctypes.byref(final), ctypes.byref(acc), _ptr(tr)))
    return dict(final_tour=t, final_cost=final.value, best_tour=best_tour, best_cost=best.value, accepted=acc.value,
                trace=tr)


def sa_chains(c, steps: int, t_start: int, t_end: int, seed: int, r0: int, r1: int, init: Optional[np.ndarray] = None):
    c = _mat(c)
    n = c.shape[0]
    k = r1 - r0
    costs = np.empty(k, dtype=np.int64)
    tours = np.empty((k, n), dtype=np.int32)
    accepted = np.empty(k, dtype=np.int32)
    if init is not None:
        init = np.ascontiguousarray(init, dtype=np.int32)
    _check(_L().cco_sa_chains(_ptr(c), n, steps, t_start, t_end, seed, r0, r1, _ptr(init), _ptr(costs), _ptr(tours),
                              _ptr(accepted)))
    return costs, tours, accepted


def sa_search(c, chains: int, steps: int, t_start: int, t_end: int, seed: int, init: Optional[np.ndarray] = None):
    costs, tours, accepted = sa_chains(c, steps, t_start, t_end, seed, 0, chains, init)
    k = int(np.argmin(costs))
    return dict(best_perm=tours[k].copy(), best_cost=int(costs[k]), best_chain=k, costs=costs, tours=tours,
                accepted=accepted)


# ------------------------------------------------------------------------------------------ double binary tree
def dbt_tree_cost(c, perm, shift: int = 0) -> int:
    c = _mat(c)
    perm = np.ascontiguousarray(perm, dtype=np.int32)
    return int(_L().cco_dbt_tree_cost(_ptr(c), c.shape[0], _ptr(perm), shift))


def dbt_cost(c, perm) -> int:
    c = _mat(c)
    perm = np.ascontiguousarray(perm, dtype=np.int32)
    return int(_L().cco_dbt_cost(_ptr(c), c.shape[0], _ptr(perm)))


def dbt_cost_batch(c, perms) -> np.ndarray:
    c = _mat(c)
    perms = np.ascontiguousarray(perms, dtype=np.int32).reshape(-1, c.shape[0])
    out = np.empty(perms.shape[0], dtype=np.int64)
    _check(_L().cco_dbt_cost_batch(_ptr(c), c.shape[0], _ptr(perms), perms.shape[0], _ptr(out)))
    return out


def bcube_cost_weighted_batch(c, base: int, weights, perms) -> np.ndarray:
    """Size-weighted rounds; base 2 is halving-doubling."""
    c = _mat(c)
    weights = np.ascontiguousarray(weights, dtype=np.int32)
    perms = np.ascontiguousarray(perms, dtype=np.int32).reshape(-1, c.shape[0])
    out = np.empty(perms.shape[0], dtype=np.int64)
    _check(_L().cco_bcube_cost_weighted_batch(_ptr(c), c.shape[0], base, _ptr(weights), _ptr(perms), perms.shape[0],
                                              _ptr(out)))
    return out


# ------------------------------------------------------------------------------------------ cost matrix from probes
def cost_matrix_from_probes(samples, percentile: int = 10, symmetrize: bool = True) -> np.ndarray:
    samples = np.ascontiguousarray(samples, dtype=np.int32)
    assert samples.ndim == 3 and samples.shape[0] == samples.shape[1]
    n, k = samples.shape[0], samples.shape[2]
    out = np.empty((n, n), dtype=np.int32)
    _check(_L().cco_cost_matrix_from_probes(_ptr(samples), n, k, percentile, int(symmetrize), _ptr(out)))
    return out


# ------------------------------------------------------------------------------------------ annealing, halving-doubling
def sa_rd_proposal(seed: int, r: int, s: int, n: int):
    """(p, q, u): the two ranks to exchange and the acceptance draw of step s of chain r."""
    a, b, u = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    _L().cco_sa_rd_proposal(seed, r, s, n, ctypes.byref(a), ctypes.byref(b), ctypes.byref(u))
    return a.value, b.value, u.value


def sa_rd_chain(c, t, steps: int, t_start: int, t_end: int, seed: int, r: int, trace: bool = False):
    c = _mat(c)
    n = c.shape[0]
    t = np.array(t, dtype=np.int32, copy=True)
    best_tour = np.empty(n, dtype=np.int32)
    best, final = ctypes.c_int64(), ctypes.c_int64()
    acc = ctypes.c_int32()
    tr = np.empty(steps, dtype=np.int64) if trace else None
    _check(_L().cco_sa_rd_chain(_ptr(c), n, _ptr(t), steps, t_start, t_end, seed, r, _ptr(best_tour), ctypes.byref(best),
                                ctypes.byref(final), ctypes.byref(acc), _ptr(tr)))
    return dict(final_tour=t, final_cost=final.value, best_tour=best_tour, best_cost=best.value, accepted=acc.value,
                trace=tr)


def sa_rd_chains(c, steps: int, t_start: int, t_end: int, seed: int, r0: int, r1: int,
                 init: Optional[np.ndarray] = None):
    c = _mat(c)
    n = c.shape[0]
    k = r1 - r0
    costs = np.empty(k, dtype=np.int64)
    tours = np.empty((k, n), dtype=np.int32)
    accepted = np.empty(k, dtype=np.int32)
    if init is not None:
        init = np.ascontiguousarray(init, dtype=np.int32)
    _check(_L().cco_sa_rd_chains(_ptr(c), n, steps, t_start, t_end, seed, r0, r1, _ptr(init), _ptr(costs), _ptr(tours),
                                 _ptr(accepted)))
    return costs, tours, accepted


def sa_rd_search(c, chains: int, steps: int, t_start: int, t_end: int, seed: int, init: Optional[np.ndarray] = None):
    costs, tours, accepted = sa_rd_chains(c, steps, t_start, t_end, seed, 0, chains, init)
    k = int(np.argmin(costs))
    return dict(best_perm=tours[k].copy(), best_cost=int(costs[k]), best_chain=k, costs=costs, tours=tours,
                accepted=accepted)


# ---- wider ring neighbourhoods: segment insertion (Or-opt) and the orientation flip
MOVES_2OPT, MOVES_OROPT, MOVES_FLIP = 1, 2, 4


def oropt_is_move(n: int, s: int, length: int, g: int, o: int = 0) -> bool:
    return bool(_L().cco_oropt_is_move(n, s, length, g, o))


def oropt_move_id(n: int, s: int, length: int, g: int, o: int = 0) -> int:
    return int(_L().cco_oropt_move_id(n, s, length, g, o))


def oropt_apply(t, s: int, length: int, g: int, o: int = 0) -> np.ndarray:
    u = np.array(t, dtype=np.int32, copy=True)
    assert oropt_is_move(u.shape[0], s, length, g, o)
    _L().cco_oropt_apply(_ptr(u), u.shape[0], s, length, g, o)
    return u


def oropt_value_by_definition(c, t, s: int, length: int, g: int, o: int = 0) -> int:
    c = _mat(c)
    t = np.ascontiguousarray(t, dtype=np.int32)
    assert oropt_is_move(c.shape[0], s, length, g, o)
    return int(_L().cco_oropt_value_by_definition(_ptr(c), c.shape[0], _ptr(t), s, length, g, o))


def oropt_neighbourhood_size(n: int) -> int:
    return int(_L().cco_oropt_neighbourhood_size(n))


def oropt_moves_in_id_order(n: int):
    """(s, length, g, o) of every segment insertion, in increasing id order."""
    out = []
    for length, o in ((1, 0), (2, 0), (2, 1), (3, 0), (3, 1)):
        for s in range(1, n):
            for g in range(n):
                if oropt_is_move(n, s, length, g, o):
                    out.append((s, length, g, o))
    return out


def oropt_all_values(c, t) -> np.ndarray:
    c = _mat(c)
    t = np.ascontiguousarray(t, dtype=np.int32)
    out = np.empty(oropt_neighbourhood_size(c.shape[0]), dtype=np.int64)
    _check(_L().cco_oropt_all_values(_ptr(c), c.shape[0], _ptr(t), _ptr(out)))
    return out


def local_classes_ok(objective: int, classes: int) -> bool:
    return bool(_L().cco_local_classes_ok(objective, classes))


def local_descend(c, objective: int, classes: int, t, use_definition: bool = False, trace_cap: int = 0):
    """One descent over the enabled move classes. Returns (final tour, cost, applied moves, trace of move ids)."""
    c = _mat(c)
    u = np.array(t, dtype=np.int32, copy=True)
    cost = ctypes.c_int64(0)
    moves = ctypes.c_int32(0)
    trace = np.zeros(max(trace_cap, 1), dtype=np.int64)
    _check(_L().cco_local_descend(_ptr(c), c.shape[0], objective, classes, _ptr(u), ctypes.byref(cost),
                                  ctypes.byref(moves), 1 if use_definition else 0, _ptr(trace), trace_cap))
    return u, int(cost.value), int(moves.value), trace[:min(trace_cap, moves.value)]


def local_restarts(c, objective: int, classes: int, seed: int, r0: int, r1: int, init: Optional[np.ndarray] = None):
    """Restarts [r0, r1): returns (costs int64[r1-r0], tours int32[r1-r0, N], moves int32[r1-r0])."""
    c = _mat(c)
    n = c.shape[0]
    k = r1 - r0
    costs = np.empty(k, dtype=np.int64)
    tours = np.empty((k, n), dtype=np.int32)
    moves = np.empty(k, dtype=np.int32)
    if init is not None:
        init = np.ascontiguousarray(init, dtype=np.int32)
    _check(_L().cco_local_restarts(_ptr(c), n, objective, classes, seed, r0, r1, _ptr(init), _ptr(costs), _ptr(tours),
                                   _ptr(moves)))
    return costs, tours, moves


def local_search(c, objective: int, classes: int, n_restarts: int, seed: int, init: Optional[np.ndarray] = None):
    """Whole multi-start search: all restarts, then the lexicographic minimum of (final cost, restart)."""
    costs, tours, moves = local_restarts(c, objective, classes, seed, 0, n_restarts, init)
    arg = int(np.lexsort((np.arange(n_restarts), costs))[0])
    return dict(best_perm=tours[arg].copy(), best_cost=int(costs[arg]), best_restart=arg, costs=costs, tours=tours,
                moves=moves)
