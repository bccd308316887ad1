"""Pins for the oracle's wider ring neighbourhoods (segment insertion and the orientation flip; CPU only).

Section 4.3 of the paper searches with sub-array and pair permutations "alongside standard heuristics"; segment
insertion (Or-opt) and the orientation flip are this project's choice of such heuristics, so the pins are those of
the mathematics: an independent pure-Python model of the move, apply-and-recompute against the delta formulas,
closed forms on a circle metric and on a one-way ring, brute-force enumeration of the reachable tours, and
local-optimum certificates.
"""
import numpy as np
import pytest

import oracle
from oracle import MOVES_2OPT, MOVES_FLIP, MOVES_OROPT


def _sym(n, seed, lo=1, hi=1000):
    rng = np.random.default_rng(seed)
    a = rng.integers(lo, hi, size=(n, n))
    a = np.maximum(a, a.T)
    np.fill_diagonal(a, 0)
    return a.astype(np.int32)


def _asym(n, seed, lo=1, hi=1000):
    rng = np.random.default_rng(seed)
    a = rng.integers(lo, hi, size=(n, n))
    np.fill_diagonal(a, 0)
    return a.astype(np.int32)


def _circle(n):
    idx = np.arange(n)
    d = np.abs(idx[:, None] - idx[None, :])
    return np.minimum(d, n - d).astype(np.int32)


def _ring_sum(c, t):
    """Section 4.1, ring model, written out."""
    n = len(t)
    return sum(int(c[t[p]][t[(p - 1) % n]]) for p in range(n))


def _python_insertion(t, s, length, g, o):
    """The move in list operations: cut the segment, put it back behind the node that sat at rank g."""
    t = list(t)
    seg = t[s:s + length]
    anchor_node = t[g]
    rest = t[:s] + t[s + length:]
    if o:
        seg = seg[::-1]
    at = rest.index(anchor_node) + 1
    return rest[:at] + seg + rest[at:]


@pytest.mark.parametrize("n", [4, 5, 6, 9])
def test_move_set_size_ids_and_validity(n):
    moves = oracle.oropt_moves_in_id_order(n)
    assert len(moves) == oracle.oropt_neighbourhood_size(n)
    want = sum((n - L) * (n - L - 1) * (1 if L == 1 else 2) for L in (1, 2, 3) if L <= n - 3)
    assert len(moves) == want
    ids = [oracle.oropt_move_id(n, s, L, g, o) for s, L, g, o in moves]
    assert ids == sorted(ids) and len(set(ids)) == len(ids)
    # above every 2-opt id (undirected ids are i*n + j < n*n)
    assert min(ids) >= n * n
    for s, L, g, o in moves:
        assert 1 <= s and s + L - 1 <= n - 1 and not (s - 1 <= g <= s + L - 1)
    # the rules that bound the set
    assert not oracle.oropt_is_move(n, 0, 1, 2, 0)          # the anchor never moves
    assert not oracle.oropt_is_move(n, 1, 1, 0, 0)          # putting a segment back where it was
    assert not oracle.oropt_is_move(n, 1, 1, 1, 0)
    assert not oracle.oropt_is_move(n, 1, 1, 2, 1) and not oracle.oropt_is_move(n, 1, 4, 0, 0)
    assert not oracle.oropt_is_move(n, n - 1, 2, 0, 0)      # segment may not wrap past the last rank


@pytest.mark.parametrize("n", [4, 6, 7, 10])
def test_apply_equals_python_list_model(n):
    rng = np.random.default_rng(n)
    t = np.concatenate([[0], 1 + rng.permutation(n - 1)]).astype(np.int32)
    for s, L, g, o in oracle.oropt_moves_in_id_order(n):
        got = oracle.oropt_apply(t, s, L, g, o)
        want = _python_insertion(t, s, L, g, o)
        assert got.tolist() == want, (s, L, g, o)
        assert got[0] == t[0] and sorted(got.tolist()) == list(range(n))


@pytest.mark.parametrize("n", [6, 7])
def test_reachable_tours_are_exactly_the_segment_insertions(n):
    """Brute force: a tour is reachable iff it arises from the start by cutting out 1..3 consecutive non-anchor
    ranks and re-inserting them elsewhere, in either direction, with rank 0 fixed."""
    t = list(range(n))
    got = {tuple(oracle.oropt_apply(np.array(t, dtype=np.int32), s, L, g, o).tolist())
           for s, L, g, o in oracle.oropt_moves_in_id_order(n)}
    want = set()
    for L in (1, 2, 3):
        if L > n - 3:
            continue
        for s in range(1, n - L + 1):
            seg, rest = t[s:s + L], t[:s] + t[s + L:]
            for at in range(1, len(rest) + 1):             # behind rest[at - 1]; never in front of the anchor
                for sg in (seg, seg[::-1]):
                    u = rest[:at] + sg + rest[at:]
                    if u != t and not (sg != seg and at == s):   # the reversal in place is a 2-opt move, not an insertion
                        want.add(tuple(u))
    # in-place unreversed re-insertion (u == t) is excluded on both sides
    assert got - {tuple(t)} == want - {tuple(t)}
    assert tuple(t) not in got or n <= 4


@pytest.mark.parametrize("n,seed", [(4, 1), (5, 2), (6, 3), (7, 4), (12, 5), (33, 6)])
def test_fast_values_equal_apply_and_recompute(n, seed):
    c = _sym(n, seed)
    t = oracle.init_tours(seed, n, 1)[0]
    fast = oracle.oropt_all_values(c, t)
    moves = oracle.oropt_moves_in_id_order(n)
    assert len(fast) == len(moves)
    for v, (s, L, g, o) in zip(fast, moves):
        u = _python_insertion(t, s, L, g, o)
        assert int(v) == _ring_sum(c, u) == oracle.oropt_value_by_definition(c, t, s, L, g, o), (s, L, g, o)


@pytest.mark.parametrize("n", [8, 16, 64])
@pytest.mark.parametrize("length,reverse", [(1, False), (2, False), (2, True), (3, False), (3, True)])
def test_circle_metric_displaced_segment_is_repaired_in_one_move(n, length, reverse):
    """On the circle metric the identity order costs exactly n, the optimum (every hop >= 1).  Cut `length` nodes
    out and put them elsewhere (reversed or not): one segment insertion restores cost n, and it is the best move."""
    c = _circle(n)
    ident = list(range(n))
    assert _ring_sum(c, ident) == n
    s = 2
    seg, rest = ident[s:s + length], ident[:s] + ident[s + length:]
    at = len(rest) - 1
    t = np.array(rest[:at] + (seg[::-1] if reverse else seg) + rest[at:], dtype=np.int32)
    start = _ring_sum(c, t)
    assert start > n
    u, cost, moves, trace = oracle.local_descend(c, oracle.SUM, MOVES_OROPT, t, trace_cap=4)
    assert cost == n and moves == 1
    assert oracle.ring_cost(c, u, oracle.SUM) == n
    assert start == oracle.ring_cost(c, t, oracle.SUM)


@pytest.mark.parametrize("classes", [MOVES_OROPT, MOVES_2OPT | MOVES_OROPT])
@pytest.mark.parametrize("n,seed", [(5, 1), (8, 2), (11, 3)])
def test_trajectory_definition_vs_fast_and_python_scan(n, seed, classes):
    """Every step of the descent is the lexicographic minimum of (value, id) over the enabled classes, scanned
    here in Python from the move lists; 2-opt ids lie below insertion ids, so a 2-opt move wins ties."""
    c = _sym(n, seed, 1, 12)                    # few distinct values: many ties
    t0 = oracle.init_tours(seed + 10, n, 1)[0]
    u1, c1, m1, tr1 = oracle.local_descend(c, oracle.SUM, classes, t0, False, 200)
    u2, c2, m2, tr2 = oracle.local_descend(c, oracle.SUM, classes, t0, True, 200)
    assert c1 == c2 and m1 == m2 and u1.tolist() == u2.tolist() and tr1.tolist() == tr2.tolist()
    t = [int(x) for x in t0]
    cur = _ring_sum(c, t)
    for step in range(m1 + 1):
        cands = []
        if classes & MOVES_2OPT:
            for i, j, o in oracle.moves_in_id_order(n, oracle.SUM):
                v = t[:i] + t[i:j + 1][::-1] + t[j + 1:]
                cands.append((_ring_sum(c, v), i * n + j, v))
        for s, L, g, o in oracle.oropt_moves_in_id_order(n):
            v = _python_insertion(t, s, L, g, o)
            cands.append((_ring_sum(c, v), oracle.oropt_move_id(n, s, L, g, o), v))
        best = min(cands, key=lambda x: (x[0], x[1]))
        if step == m1:
            assert best[0] >= cur                  # certificate: nothing improves at the end
            break
        assert best[0] < cur and best[1] == int(tr1[step])
        t, cur = best[2], best[0]
    assert t == u1.tolist() and cur == c1


def test_union_tie_goes_to_the_2opt_move():
    """Moving one node by one gap and reversing the pair it forms with its neighbour give the same ring; with all
    other moves worse the 2-opt id must be the one reported."""
    n = 6
    c = _circle(n)
    t = np.array([0, 2, 1, 3, 4, 5], dtype=np.int32)       # one adjacent transposition away from the optimum
    u, cost, moves, trace = oracle.local_descend(c, oracle.SUM, MOVES_2OPT | MOVES_OROPT, t, trace_cap=4)
    assert cost == n and moves == 1
    assert int(trace[0]) == 1 * n + 2                      # reversal of ranks 1..2
    u, cost, moves, trace = oracle.local_descend(c, oracle.SUM, MOVES_OROPT, t, trace_cap=4)
    assert cost == n and moves == 1 and int(trace[0]) == oracle.oropt_move_id(n, 1, 1, 2, 0)


@pytest.mark.parametrize("objective", [oracle.SUM_DIRECTED, oracle.MAX_DIRECTED])
def test_flip_on_a_one_way_ring(objective):
    """c[a][a-1] = 1 and every other entry 10: walking the ranks upward costs 1 per hop, downward 10.  From the
    downward order the flip alone reaches the optimum in one move, with the id of the pair (1, N-1)."""
    n = 9
    c = np.full((n, n), 10, dtype=np.int32)
    for a in range(n):
        c[a][(a - 1) % n] = 1
    np.fill_diagonal(c, 0)
    down = np.array([0] + list(range(n - 1, 0, -1)), dtype=np.int32)
    want_start = 10 * n if objective == oracle.SUM_DIRECTED else 10
    want_end = n if objective == oracle.SUM_DIRECTED else 1
    assert oracle.ring_cost(c, down, objective & 1) == want_start
    u, cost, moves, trace = oracle.local_descend(c, objective, MOVES_2OPT | MOVES_FLIP, down, trace_cap=4)
    assert cost == want_end and moves == 1 and u.tolist() == list(range(n))
    assert int(trace[0]) == (1 * n + (n - 1)) * 2
    # without the flip the 2-opt set cannot turn the whole ring round in one move
    u, cost, moves, trace = oracle.local_descend(c, objective, MOVES_2OPT, down, trace_cap=4)
    assert not (moves == 1 and cost == want_end)


@pytest.mark.parametrize("objective", [oracle.SUM_DIRECTED, oracle.MAX_DIRECTED])
@pytest.mark.parametrize("n,seed", [(5, 1), (9, 2)])
def test_flip_trajectory_definition_vs_fast(n, seed, objective):
    c = _asym(n, seed, 1, 30)
    t0 = oracle.init_tours(seed, n, 1)[0]
    a = oracle.local_descend(c, objective, MOVES_2OPT | MOVES_FLIP, t0, False, 100)
    b = oracle.local_descend(c, objective, MOVES_2OPT | MOVES_FLIP, t0, True, 100)
    assert a[1] == b[1] and a[2] == b[2] and a[0].tolist() == b[0].tolist() and a[3].tolist() == b[3].tolist()
    # the value of the flip is the ring cost of the same order on the transposed matrix
    flipped = oracle.apply_move(t0, 1, n - 1, 0)
    assert oracle.ring_cost(c, flipped, objective & 1) == oracle.ring_cost(c.T.copy(), t0, objective & 1)
    # certificate including the flip
    u = a[0]
    cur = a[1]
    assert oracle.move_value_by_definition(c, objective, u, 1, n - 1, 0) >= cur
    for i, j, o in oracle.moves_in_id_order(n, objective):
        assert oracle.move_value_by_definition(c, objective, u, i, j, o) >= cur


def test_class_table_and_errors():
    ok = {(obj, cls) for obj in range(4) for cls in range(8) if oracle.local_classes_ok(obj, cls)}
    want = {(obj, MOVES_2OPT) for obj in range(4)}
    want |= {(oracle.SUM, MOVES_OROPT), (oracle.SUM, MOVES_2OPT | MOVES_OROPT)}
    want |= {(oracle.SUM_DIRECTED, MOVES_2OPT | MOVES_FLIP), (oracle.MAX_DIRECTED, MOVES_2OPT | MOVES_FLIP)}
    assert ok == want
    c = _sym(6, 1)
    t = np.arange(6, dtype=np.int32)
    with pytest.raises(RuntimeError):
        oracle.local_descend(c, oracle.MAX, MOVES_OROPT, t)
    with pytest.raises(RuntimeError):
        oracle.local_restarts(_asym(6, 1), oracle.SUM, MOVES_OROPT, 1, 0, 2)     # needs a symmetric matrix


@pytest.mark.parametrize("objective", range(4))
def test_class_2opt_is_the_2opt_search(objective):
    c = _asym(12, 3) if objective & 2 else _sym(12, 3)
    a = oracle.restarts(c, objective, 99, 0, 6)
    b = oracle.local_restarts(c, objective, MOVES_2OPT, 99, 0, 6)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


def test_union_never_ends_above_a_2opt_optimum_it_starts_from_and_search_is_argmin():
    c = _sym(16, 8)
    costs2, tours2, _ = oracle.restarts(c, oracle.SUM, 5, 0, 8)
    # continue each 2-opt optimum with the union: can only go down, and ends in an optimum of both classes
    costs3, tours3, _ = oracle.local_restarts(c, oracle.SUM, MOVES_2OPT | MOVES_OROPT, 5, 0, 8, init=tours2)
    assert (costs3 <= costs2).all()
    for t, cost in zip(tours3, costs3):
        assert oracle.ring_cost(c, t, oracle.SUM) == cost
        assert oracle.all_move_values(c, oracle.SUM, t).min() >= cost
        assert oracle.oropt_all_values(c, t).min() >= cost
    res = oracle.local_search(c, oracle.SUM, MOVES_2OPT | MOVES_OROPT, 8, 5)
    arg = min(range(8), key=lambda r: (res["costs"][r], r))
    assert res["best_restart"] == arg and res["best_cost"] == res["costs"][arg]
    assert res["best_perm"].tolist() == res["tours"][arg].tolist()


def test_exhaustive_optimum_is_a_fixed_point_and_small_instances_reach_it_often():
    """N = 8: the true optimum (all 2520 rings enumerated) admits no improving move of either class; from 64
    seeded starts the union descent ends at the optimum at least as often as 2-opt alone."""
    c = _sym(8, 21)
    ex = oracle.exhaustive_rings(c, oracle.SUM, half_only=True)
    best_cost, best_ring = ex["best_cost"], ex["best_ring"]
    u, cost, moves, _ = oracle.local_descend(c, oracle.SUM, MOVES_2OPT | MOVES_OROPT, best_ring)
    assert moves == 0 and cost == best_cost
    c2, _, _ = oracle.restarts(c, oracle.SUM, 3, 0, 64)
    c3, _, _ = oracle.local_restarts(c, oracle.SUM, MOVES_2OPT | MOVES_OROPT, 3, 0, 64)
    assert (c3 >= best_cost).all() and (c2 >= best_cost).all()
    assert (c3 == best_cost).sum() >= (c2 == best_cost).sum()
