"""Pins for the oracle's cost models (Section 4.1): closed forms, invariants, a hand-worked example and
brute force on tiny inputs.  None of these retype the oracle's loop; each fixes the result by an
independent fact."""
import itertools
import math
import os

import numpy as np
import pytest

import oracle
from gen import clean_hierarchy, make_matrix, random_matrix, random_perms

NS = [2, 3, 4, 5, 8, 13, 64]


def _read_worked(path):
    rows, vals = [], {}
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, *rest = line.split()
        if k == "c":
            rows.append([int(x) for x in rest])
        elif k == "pi":
            vals["pi"] = [int(x) for x in rest]
        else:
            vals[k] = int(rest[0])
    return np.array(rows, dtype=np.int32), vals


def test_worked_example_n4(golden_dir):
    c, v = _read_worked(os.path.join(golden_dir, "worked_costs_n4.txt"))
    assert oracle.ring_cost(c, v["pi"], oracle.SUM) == v["ring_sum"]
    assert oracle.ring_cost(c, v["pi"], oracle.MAX) == v["ring_max"]
    assert oracle.rd_cost(c, v["pi"]) == v["rd"]


def test_worked_example_n3():
    # N=3, identity order: hops c[0][2], c[1][0], c[2][1]
    c = np.array([[0, 100, 7], [20, 0, 1000], [10000, 300, 0]], dtype=np.int32)
    assert oracle.ring_cost(c, [0, 1, 2], oracle.SUM) == 7 + 20 + 300
    assert oracle.ring_cost(c, [0, 1, 2], oracle.MAX) == 300
    # order (1, 2, 0): hops c[1][0], c[2][1], c[0][2] -> a rotation of the same ring
    assert oracle.ring_cost(c, [1, 2, 0], oracle.SUM) == 327
    # order (0, 2, 1): hops c[0][1], c[2][0], c[1][2]
    assert oracle.ring_cost(c, [0, 2, 1], oracle.SUM) == 100 + 10000 + 1000


@pytest.mark.parametrize("n", NS)
def test_ring_constant_matrix(n):
    k = 37
    c = np.full((n, n), k, dtype=np.int32)
    np.fill_diagonal(c, 0)
    for perm in random_perms(n, 5, seed=n):
        assert oracle.ring_cost(c, perm, oracle.SUM) == n * k
        assert oracle.ring_cost(c, perm, oracle.MAX) == k


@pytest.mark.parametrize("n", NS)
def test_ring_additive_matrix_is_order_independent(n):
    rng = np.random.default_rng(n)
    u = rng.integers(0, 1000, n)
    v = rng.integers(0, 1000, n)
    c = (u[:, None] + v[None, :]).astype(np.int32)
    for perm in random_perms(n, 8, seed=100 + n):
        assert oracle.ring_cost(c, perm, oracle.SUM) == int(u.sum() + v.sum())


@pytest.mark.parametrize("n", [3, 4, 5, 8, 13, 64])
def test_ring_line_metric_identity(n):
    a = np.arange(n)
    c = np.abs(a[:, None] - a[None, :]).astype(np.int32)
    assert oracle.ring_cost(c, a, oracle.SUM) == 2 * (n - 1)
    assert oracle.ring_cost(c, a, oracle.MAX) == n - 1


@pytest.mark.parametrize("n", [3, 4, 8, 13, 64])
def test_ring_hop_direction(n):
    """The ring equation charges rank p for talking to rank p-1: with c[a][b] = 1 iff b == a-1 (mod n)
    the identity order costs n; the opposite convention would give 0."""
    c = np.zeros((n, n), dtype=np.int32)
    for a in range(n):
        c[a, (a - 1) % n] = 1
    ident = np.arange(n)
    assert oracle.ring_cost(c, ident, oracle.SUM) == n
    assert oracle.ring_cost(c, ident[::-1].copy(), oracle.SUM) == 0
    assert oracle.ring_cost(c.T.copy(), ident, oracle.SUM) == 0


@pytest.mark.parametrize("n", [3, 5, 8, 64])
@pytest.mark.parametrize("obj", [oracle.SUM, oracle.MAX])
def test_ring_rotation_reversal_transpose(n, obj):
    cs = random_matrix(n, 7 + n, symmetric=True)
    ca = random_matrix(n, 9 + n, symmetric=False)
    for perm in random_perms(n, 6, seed=n):
        for c in (cs, ca):
            base = oracle.ring_cost(c, perm, obj)
            for s in (1, 2, n - 1):
                assert oracle.ring_cost(c, np.roll(perm, s), obj) == base
            # walking the ring backwards = the same order on the transposed matrix
            assert oracle.ring_cost(c, perm[::-1].copy(), obj) == oracle.ring_cost(c.T.copy(), perm, obj)
        assert oracle.ring_cost(cs, perm[::-1].copy(), obj) == oracle.ring_cost(cs, perm, obj)
    # asymmetric matrices are generally not reversal invariant
    diffs = [oracle.ring_cost(ca, p[::-1].copy(), oracle.SUM) != oracle.ring_cost(ca, p, oracle.SUM)
             for p in random_perms(n, 6, seed=n)]
    assert any(diffs)


@pytest.mark.parametrize("n,rack", [(8, 4), (8, 2), (9, 3), (10, 5)])
def test_ring_clean_hierarchy_closed_form_and_optimum(n, rack):
    a, b = 300, 1500
    c = clean_hierarchy(n, rack, a, b)
    racks = n // rack
    want = (n - racks) * a + racks * b
    assert oracle.ring_cost(c, np.arange(n), oracle.SUM) == want
    ex = oracle.exhaustive_rings(c, oracle.SUM, half_only=True)
    assert ex["best_cost"] == want           # rack-contiguous is globally optimal
    assert oracle.ring_cost(c, np.arange(n), oracle.MAX) == b


@pytest.mark.parametrize("n", [2, 4, 8, 64, 1024])
def test_rd_constant(n):
    k = 11
    c = np.full((n, n), k, dtype=np.int32)
    np.fill_diagonal(c, 0)
    perm = random_perms(n, 1, seed=n)[0]
    assert oracle.rd_cost(c, perm) == k * int(math.log2(n))


def test_rd_n2():
    c = np.array([[0, 5], [9, 0]], dtype=np.int32)
    assert oracle.rd_cost(c, [0, 1]) == 9
    assert oracle.rd_cost(c, [1, 0]) == 9


@pytest.mark.parametrize("n", [4, 8, 16, 64])
def test_rd_hypercube_automorphisms(n):
    """Relabelling ranks p -> p xor m, or permuting the bit positions of p, maps the set of rounds onto
    itself, so the cost cannot change."""
    bits = int(math.log2(n))
    c = random_matrix(n, 21 + n, symmetric=False)
    rng = np.random.default_rng(n)
    for perm in random_perms(n, 4, seed=n):
        base = oracle.rd_cost(c, perm)
        for m in (1, n - 1, n // 2, int(rng.integers(0, n))):
            q = np.empty_like(perm)
            q[np.arange(n) ^ m] = perm            # new rank p^m holds what rank p held
            assert oracle.rd_cost(c, q) == base
        for _ in range(3):
            sigma = rng.permutation(bits)
            idx = np.zeros(n, dtype=np.int64)
            for bpos in range(bits):
                idx |= ((np.arange(n) >> bpos) & 1) << sigma[bpos]
            q = np.empty_like(perm)
            q[idx] = perm
            assert oracle.rd_cost(c, q) == base


@pytest.mark.parametrize("n,rack", [(8, 4), (8, 2), (64, 8), (1024, 32)])
def test_rd_clean_hierarchy_closed_form(n, rack):
    a, b = 250, 1700
    c = clean_hierarchy(n, rack, a, b)
    want = a * int(math.log2(rack)) + b * (int(math.log2(n)) - int(math.log2(rack)))
    assert oracle.rd_cost(c, np.arange(n)) == want


def test_rd_direction_matters_only_via_max_of_both():
    """A single expensive directed entry c[a][b] is charged in the round that pairs a and b, whichever
    of the two ranks it sits on."""
    n = 8
    c = np.ones((n, n), dtype=np.int32)
    np.fill_diagonal(c, 0)
    c[5, 1] = 1000                      # ranks 5 and 1 differ in bit 2 only
    assert oracle.rd_cost(c, np.arange(n)) == 1 + 1 + 1000
    c[5, 1] = 1
    c[5, 2] = 1000                      # ranks 5 and 2 differ in three bits: never paired
    assert oracle.rd_cost(c, np.arange(n)) == 3


def test_rd_brute_force_minimum_n8():
    """On a clean hierarchy with racks of 2 the optimum over all 8! orders must equal the closed form of
    a rack-contiguous order (no order can do better than one intra round + two cross rounds)."""
    c = clean_hierarchy(8, 2, 10, 1000)
    perms = np.array(list(itertools.permutations(range(8))), dtype=np.int32)
    costs = oracle.rd_cost_batch(c, perms)
    assert costs.min() == 10 + 2 * 1000
    assert oracle.rd_cost(c, np.arange(8)) == costs.min()
    # pair-major recount with numpy for every order (different traversal order of the same sets)
    want = np.zeros(len(perms), dtype=np.int64)
    for k in range(3):
        partner = perms[:, np.arange(8) ^ (1 << k)]
        want += c[perms, partner].max(axis=1)
    assert np.array_equal(costs, want)


def test_exhaustive_enumerator_counts_and_coverage():
    for n in (4, 5, 6, 8):
        c = random_matrix(n, 3 + n, symmetric=True)
        ex = oracle.exhaustive_rings(c, oracle.SUM, half_only=True, keep_all=True)
        assert ex["count"] == math.factorial(n - 1) // 2
        full = oracle.exhaustive_rings(c, oracle.SUM, half_only=False)
        assert full["count"] == math.factorial(n - 1)
        assert full["best_cost"] == ex["best_cost"]
        rings = ex["rings"]
        assert (rings[:, 0] == 0).all() and (rings[:, 1] < rings[:, -1]).all()
        assert len({tuple(r) for r in rings}) == ex["count"]
        # lexicographic order of the tail
        keys = [tuple(r) for r in rings]
        assert keys == sorted(keys)
        # the first minimiser in that order is the one reported
        first = int(np.argmin(ex["costs"]))
        assert np.array_equal(rings[first], ex["best_ring"]) and ex["costs"][first] == ex["best_cost"]
        # every random order canonicalises to a listed ring, and costs at least the optimum
        ringset = {tuple(r): k for k, r in enumerate(rings)}
        for perm in random_perms(n, 20, seed=n):
            z = int(np.where(perm == 0)[0][0])
            canon = np.roll(perm, -z)
            if canon[1] > canon[-1]:
                canon = np.concatenate([[0], canon[1:][::-1]])
            k = ringset[tuple(canon)]
            assert ex["costs"][k] == oracle.ring_cost(c, perm, oracle.SUM) >= ex["best_cost"]


def test_workload1_exhaustive_2520():
    c = make_matrix(1)
    ex = oracle.exhaustive_rings(c, oracle.SUM, half_only=True, keep_all=True)
    assert ex["count"] == 2520
    assert ex["best_cost"] == ex["costs"].min()
    # two racks of four: the optimum uses exactly two cross-rack hops
    cross = (c[ex["best_ring"], np.roll(ex["best_ring"], 1)] >= 800).sum()
    assert cross == 2


def test_batch_equals_single():
    c = make_matrix(2)
    perms = random_perms(64, 50, seed=5)
    for obj in (oracle.SUM, oracle.MAX):
        got = oracle.ring_cost_batch(c, perms, obj)
        assert [oracle.ring_cost(c, p, obj) for p in perms] == list(got)
    got = oracle.rd_cost_batch(c, perms)
    assert [oracle.rd_cost(c, p) for p in perms] == list(got)
