"""Pins for the oracle's 2-opt neighbourhood, descent and restarts (Section 4.3 neighbour search made
deterministic): fast move values against apply-and-recompute, structure of the move set, local-optimum
certificates, brute-force lower bounds, and the restart generator against published SplitMix64 values."""
import os

import numpy as np
import pytest

import oracle
from gen import clean_hierarchy, make_matrix, random_matrix, random_perms

OBJ = [oracle.SUM, oracle.MAX, oracle.SUM_DIRECTED, oracle.MAX_DIRECTED]


def _matrix_for(n, obj, seed):
    # undirected objectives are defined on symmetric matrices only
    return random_matrix(n, seed, symmetric=not (obj & 2), lo=1, hi=3000)


# ---------------------------------------------------------------------------------------- generator
def test_splitmix64_published_vectors(golden_dir):
    want = [int(l) for l in open(os.path.join(golden_dir, "splitmix64_seed1234567.txt"))
            if l.strip() and not l.startswith("#")]
    got = [oracle.splitmix64_at(1234567, n) for n in range(1, len(want) + 1)]
    assert got == want


def test_splitmix64_jump_equals_sequence():
    # the n-th output computed directly must equal stepping a sequential generator n times
    mask = 2**64 - 1
    state = 0xDEADBEEF
    for n in range(1, 50):
        state = (state + 0x9E3779B97F4A7C15) & mask
        # sequential generator: its output function applied to the advanced state == jump from state 0
        assert oracle.splitmix64_at(state, 0) == oracle.splitmix64_at(0xDEADBEEF, n)


@pytest.mark.parametrize("n", [2, 3, 8, 13, 64, 256, 1024])
def test_init_tours_are_permutations_and_distinct(n):
    tours = oracle.init_tours(0xC0FFEE02, n, 64)
    assert (np.sort(tours, axis=1) == np.arange(n)).all()
    if n >= 8:
        assert len({tuple(t) for t in tours}) == 64
    other = oracle.init_tours(0xC0FFEE03, n, 64)
    if n >= 8:
        assert not np.array_equal(tours, other)
    # restart r depends on (seed, r) only: any chunking gives the same tours
    assert np.array_equal(oracle.init_tours(0xC0FFEE02, n, 10, first=30), tours[30:40])


def test_init_tours_uniform_n4():
    """All 24 orders of 4 ranks must appear about equally often (chi-square, 23 dof; 99.99% quantile ~ 58)."""
    tours = oracle.init_tours(12345, 4, 24000)
    _, counts = np.unique(tours @ np.array([64, 16, 4, 1]), return_counts=True)
    assert len(counts) == 24
    chi2 = ((counts - 1000.0) ** 2 / 1000.0).sum()
    assert chi2 < 58.0


def test_init_tours_position_marginals_n64():
    tours = oracle.init_tours(777, 64, 64 * 400)
    # every node is equally likely at every rank: check rank 0 and rank 63 marginals
    for pos in (0, 31, 63):
        counts = np.bincount(tours[:, pos], minlength=64)
        chi2 = ((counts - 400.0) ** 2 / 400.0).sum()
        assert chi2 < 130.0          # 63 dof, 99.999% quantile ~ 121


def test_init_tours_frozen_vectors(golden_dir):
    """Self-pin (the paper fixes no generator): vectors written by tests/golden/make_golden.py."""
    data = np.loadtxt(os.path.join(golden_dir, "init_tours_seed_c0ffee02_n16.txt"), dtype=np.int64, comments="#")
    assert np.array_equal(oracle.init_tours(0xC0FFEE02, 16, data.shape[0]), data)


# ------------------------------------------------------------------------------------- neighbourhood
@pytest.mark.parametrize("n", [4, 5, 8, 13])
@pytest.mark.parametrize("obj", OBJ)
def test_move_set_structure(n, obj):
    moves = oracle.moves_in_id_order(n, obj)
    assert len(moves) == oracle.neighbourhood_size(n, obj) == (n * (n - 3) * (2 if obj & 2 else 1)) // 2
    ids = [oracle.move_id(n, obj, *m) for m in moves]
    assert ids == sorted(ids) and len(set(ids)) == len(ids)
    # every pair of non-adjacent ring edges is exchanged exactly once per orientation
    pairs = set()
    for (i, j, o) in moves:
        e1, e2 = i, (j + 1) % n          # edge p joins ranks p-1 and p
        assert (e1 - e2) % n not in (0, 1, n - 1)
        pairs.add((min(e1, e2), max(e1, e2), o))
    assert len(pairs) == len(moves)


def test_neighbourhood_empty_below_4():
    for n in (2, 3):
        for obj in OBJ:
            assert oracle.neighbourhood_size(n, obj) == 0
            c = _matrix_for(n, obj, 1)
            t, cost, moves, _ = oracle.descend(c, obj, np.arange(n))
            assert moves == 0 and np.array_equal(t, np.arange(n)) and cost == oracle.ring_cost(c, t, obj)


@pytest.mark.parametrize("n", [5, 8, 13])
def test_apply_move_properties(n):
    rng = np.random.default_rng(n)
    for t in random_perms(n, 5, seed=n):
        for (i, j, o) in oracle.moves_in_id_order(n, oracle.SUM_DIRECTED):
            u = oracle.apply_move(t, i, j, o)
            assert u[0] == t[0] and sorted(u) == list(range(n))
            if o == 0:
                assert np.array_equal(u[i:j + 1], t[i:j + 1][::-1])
                assert np.array_equal(u[:i], t[:i]) and np.array_equal(u[j + 1:], t[j + 1:])
                assert np.array_equal(oracle.apply_move(u, i, j, 0), t)     # an involution
            else:
                # same ring as orientation 0, walked the other way round
                v = oracle.apply_move(t, i, j, 0)
                assert np.array_equal(u, np.concatenate([[v[0]], v[1:][::-1]]))


@pytest.mark.parametrize("n", [4, 5, 8, 13, 64])
@pytest.mark.parametrize("obj", OBJ)
def test_fast_move_values_equal_apply_and_recompute(n, obj):
    c = _matrix_for(n, obj, 40 + n)
    moves = oracle.moves_in_id_order(n, obj)
    for t in random_perms(n, 3 if n == 64 else 6, seed=n + obj):
        fast = oracle.all_move_values(c, obj, t)
        assert len(fast) == len(moves)
        for v, (i, j, o) in zip(fast, moves):
            assert v == oracle.move_value_by_definition(c, obj, t, i, j, o), (n, obj, i, j, o)
            # and the definition itself is the ring cost of the explicitly edited order
            assert v == oracle.ring_cost(c, oracle.apply_move(t, i, j, o), obj)


@pytest.mark.parametrize("obj", [oracle.SUM_DIRECTED, oracle.MAX_DIRECTED])
def test_directed_on_symmetric_matrix_prefers_orientation_0(obj):
    n = 13
    c = random_matrix(n, 5, symmetric=True)
    t = random_perms(n, 1, seed=3)[0]
    vals = oracle.all_move_values(c, obj, t)
    assert np.array_equal(vals[0::2], vals[1::2])
    und = oracle.all_move_values(c, obj & 1, t)
    assert np.array_equal(vals[0::2], und)


# ------------------------------------------------------------------------------------------- descent
def _certify_local_optimum(c, obj, t, cost):
    assert oracle.ring_cost(c, t, obj) == cost
    n = c.shape[0]
    for (i, j, o) in oracle.moves_in_id_order(n, obj):
        assert oracle.ring_cost(c, oracle.apply_move(t, i, j, o), obj) >= cost


@pytest.mark.parametrize("n", [4, 6, 9, 16])
@pytest.mark.parametrize("obj", OBJ)
def test_descent_trajectory_definition_vs_fast_and_certificate(n, obj):
    c = _matrix_for(n, obj, 70 + n)
    for t0 in random_perms(n, 4, seed=n * 7 + obj):
        a = oracle.descend(c, obj, t0, use_definition=False, trace_cap=256)
        b = oracle.descend(c, obj, t0, use_definition=True, trace_cap=256)
        assert np.array_equal(a[0], b[0]) and a[1] == b[1] and a[2] == b[2] and np.array_equal(a[3], b[3])
        t, cost, moves, trace = a
        assert t[0] == t0[0]
        _certify_local_optimum(c, obj, t, cost)
        # replay the trace by hand: strictly decreasing cost, lowest id among the best moves
        u = t0.copy()
        cur = oracle.ring_cost(c, u, obj)
        allm = oracle.moves_in_id_order(n, obj)
        for mid in trace:
            vals = np.array([oracle.ring_cost(c, oracle.apply_move(u, *m), obj) for m in allm])
            k = int(np.argmin(vals))                # numpy argmin returns the first minimum = lowest id
            assert oracle.move_id(n, obj, *allm[k]) == mid and vals[k] < cur
            u = oracle.apply_move(u, *allm[k])
            cur = int(vals[k])
        assert np.array_equal(u, t) and cur == cost and len(trace) == moves


@pytest.mark.parametrize("n", [6, 8, 9])
def test_descent_vs_exhaustive_optimum(n):
    c = random_matrix(n, 90 + n, symmetric=True)
    ex = oracle.exhaustive_rings(c, oracle.SUM, half_only=True)
    # the global optimum is a fixed point of the descent
    t, cost, moves, _ = oracle.descend(c, oracle.SUM, ex["best_ring"])
    assert moves == 0 and cost == ex["best_cost"]
    for t0 in random_perms(n, 10, seed=n):
        _, cost, _, _ = oracle.descend(c, oracle.SUM, t0)
        assert cost >= ex["best_cost"]
    # directed search on an asymmetric matrix against all (n-1)! directed rings
    ca = random_matrix(n, 190 + n, symmetric=False)
    exd = oracle.exhaustive_rings(ca, oracle.SUM, half_only=False)
    t, cost, moves, _ = oracle.descend(ca, oracle.SUM_DIRECTED, exd["best_ring"])
    assert moves == 0 and cost == exd["best_cost"]
    for t0 in random_perms(n, 10, seed=n + 1):
        assert oracle.descend(ca, oracle.SUM_DIRECTED, t0)[1] >= exd["best_cost"]


def test_sum_and_sum_directed_agree_on_symmetric_matrix():
    n = 16
    c = random_matrix(n, 11, symmetric=True)
    for t0 in random_perms(n, 5, seed=2):
        a = oracle.descend(c, oracle.SUM, t0, trace_cap=128)
        b = oracle.descend(c, oracle.SUM_DIRECTED, t0, trace_cap=128)
        assert np.array_equal(a[0], b[0]) and a[1] == b[1] and a[2] == b[2]
        assert np.array_equal(a[3] * 2, b[3])       # same (i, j), orientation 0


def test_clean_hierarchy_descent_reaches_closed_form():
    # two racks of 4: from any start the steepest descent reaches a ring with exactly 2 cross hops
    c = clean_hierarchy(8, 4, 300, 1500)
    relabel = np.random.default_rng(0).permutation(8)
    c = np.ascontiguousarray(c[np.ix_(relabel, relabel)])
    ex = oracle.exhaustive_rings(c, oracle.SUM)
    assert ex["best_cost"] == 6 * 300 + 2 * 1500
    res = oracle.search(c, oracle.SUM, 32, seed=9)
    assert res["best_cost"] == ex["best_cost"]


# ------------------------------------------------------------------------------------------ restarts
def test_search_is_argmin_over_restarts_lowest_id():
    c = make_matrix(2)
    res = oracle.search(c, oracle.SUM, 24, seed=0xC0FFEE02)
    k = int(np.argmin(res["costs"]))
    assert res["best_restart"] == k and res["best_cost"] == res["costs"][k]
    assert np.array_equal(res["best_perm"], res["tours"][k])
    # restarts are independent: chunked and threaded evaluation give identical per-restart results
    a = oracle.restarts(c, oracle.SUM, 0xC0FFEE02, 5, 17)
    assert np.array_equal(a[0], res["costs"][5:17]) and np.array_equal(a[1], res["tours"][5:17])
    assert np.array_equal(a[2], res["moves"][5:17])
    b = oracle.restarts_parallel(c, oracle.SUM, 0xC0FFEE02, 0, 24, threads=4)
    assert np.array_equal(b[0], res["costs"]) and np.array_equal(b[1], res["tours"])
    # explicit initial tours override the seeded shuffle
    init = oracle.init_tours(0xC0FFEE02, 64, 24)
    res2 = oracle.search(c, oracle.SUM, 24, seed=1, init=init)
    assert np.array_equal(res2["tours"], res["tours"])
    # tie between restarts: duplicated initial tours -> the lower restart id wins
    init2 = np.concatenate([init[k:k + 1], init, init[k:k + 1]])
    res3 = oracle.search(c, oracle.SUM, 26, seed=1, init=init2)
    assert res3["best_restart"] == 0


@pytest.mark.parametrize("wid,obj", [(2, oracle.SUM), (3, oracle.MAX_DIRECTED)])
def test_workload_restarts_are_certified_local_optima(wid, obj):
    c = make_matrix(wid)
    costs, tours, moves = oracle.restarts(c, obj, 0xC0FFEE00 + wid, 0, 6)
    for t, cost in zip(tours, costs):
        assert sorted(t) == list(range(64))
        _certify_local_optimum(c, obj, t, int(cost))
    assert (moves > 0).all()


def test_undirected_objective_rejects_asymmetric_matrix():
    c = random_matrix(8, 1, symmetric=False)
    with pytest.raises(RuntimeError):
        oracle.restarts(c, oracle.SUM, 1, 0, 1)
