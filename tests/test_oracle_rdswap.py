"""Pins for the oracle's pair-swap local search under the halving-doubling model (Section 4.3's
"permuting random pairs" neighbour, exhaustive and deterministic): fast swap values against
swap-and-recompute, certificates of local optimality, brute force over all orders at N = 8."""
import itertools

import numpy as np
import pytest

import oracle
from gen import clean_hierarchy, make_matrix, random_matrix, random_perms


def _swaps(n):
    return [(p, q) for p in range(n - 1) for q in range(p + 1, n)]


@pytest.mark.parametrize("n", [2, 4, 8, 16, 64])
@pytest.mark.parametrize("symmetric", [True, False])
def test_fast_swap_values_equal_swap_and_recompute(n, symmetric):
    for hi in (3, 5000):                      # many ties / few ties
        c = random_matrix(n, 60 + n + hi, symmetric=symmetric, lo=0, hi=hi)
        for t in random_perms(n, 2 if n == 64 else 5, seed=n + hi):
            fast = oracle.rd_swap_all_values(c, t)
            sw = _swaps(n)
            assert len(fast) == len(sw) == n * (n - 1) // 2
            for v, (p, q) in zip(fast, sw):
                u = t.copy()
                u[p], u[q] = u[q], u[p]
                assert v == oracle.rd_cost(c, u) == oracle.rd_swap_value_by_definition(c, t, p, q), (n, p, q)


@pytest.mark.parametrize("n", [4, 8, 16])
def test_descent_trajectory_and_certificate(n):
    c = random_matrix(n, 300 + n, symmetric=False, lo=1, hi=2000)
    sw = _swaps(n)
    for t0 in random_perms(n, 4, seed=n * 3):
        a = oracle.rd_swap_descend(c, t0, use_definition=False, trace_cap=512)
        b = oracle.rd_swap_descend(c, t0, use_definition=True, trace_cap=512)
        assert np.array_equal(a[0], b[0]) and a[1] == b[1] and a[2] == b[2] and np.array_equal(a[3], b[3])
        t, cost, moves, trace = a
        assert sorted(t) == list(range(n)) and oracle.rd_cost(c, t) == cost and len(trace) == moves
        # replay: each applied swap is the lowest-id best swap and strictly improves
        u = t0.copy()
        cur = oracle.rd_cost(c, u)
        for mid in trace:
            vals = []
            for (p, q) in sw:
                w = u.copy()
                w[p], w[q] = w[q], w[p]
                vals.append(oracle.rd_cost(c, w))
            k = int(np.argmin(vals))
            assert sw[k][0] * n + sw[k][1] == mid and vals[k] < cur
            u[sw[k][0]], u[sw[k][1]] = u[sw[k][1]], u[sw[k][0]]
            cur = vals[k]
        assert np.array_equal(u, t) and cur == cost
        # local optimum: no swap improves
        assert oracle.rd_swap_all_values(c, t).min() >= cost


def test_against_all_orders_n8():
    c = random_matrix(8, 77, symmetric=True, lo=1, hi=1000)
    perms = np.array(list(itertools.permutations(range(8))), dtype=np.int32)
    costs = oracle.rd_cost_batch(c, perms)
    best = perms[int(np.argmin(costs))]
    t, cost, moves, _ = oracle.rd_swap_descend(c, best)
    assert moves == 0 and cost == costs.min()          # a global optimum is a fixed point
    for t0 in random_perms(8, 20, seed=5):
        assert oracle.rd_swap_descend(c, t0)[1] >= costs.min()


def test_clean_hierarchy_fixed_point_and_flat_moves():
    """Rack-contiguous order on a clean hierarchy is optimal (closed form); swaps inside a rack leave the
    cost unchanged (flat landscape), swaps across racks cannot lower it."""
    c = clean_hierarchy(16, 4, 10, 1000)
    ident = np.arange(16, dtype=np.int32)
    assert oracle.rd_cost(c, ident) == 2 * 10 + 2 * 1000
    vals = oracle.rd_swap_all_values(c, ident)
    sw = _swaps(16)
    for v, (p, q) in zip(vals, sw):
        if p // 4 == q // 4:
            assert v == 2020
        else:
            assert v >= 2020
    assert oracle.rd_swap_descend(c, ident)[2] == 0


def test_restarts_chunking_and_search_winner():
    c = make_matrix(2)
    res = oracle.rd_swap_search(c, 12, seed=0xC0FFEE02)
    k = int(np.argmin(res["costs"]))
    assert res["best_restart"] == k and res["best_cost"] == res["costs"][k]
    a = oracle.rd_swap_restarts(c, 0xC0FFEE02, 3, 9)
    assert np.array_equal(a[0], res["costs"][3:9]) and np.array_equal(a[1], res["tours"][3:9])
    init = oracle.init_tours(0xC0FFEE02, 64, 12)
    b = oracle.rd_swap_restarts(c, 1, 0, 12, init)
    assert np.array_equal(b[1], res["tours"]) and np.array_equal(b[2], res["moves"])
    for t, cost in zip(res["tours"][:3], res["costs"][:3]):
        assert oracle.rd_swap_all_values(c, t).min() >= cost == oracle.rd_cost(c, t)
