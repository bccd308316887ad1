"""Pins for the oracle's simulated-annealing chain (Section 4.3 names the method; schedule, random numbers and the
integer acceptance rule are this project's definition, stated in oracle/cc_oracle.c).  The pins fix what the
mathematics fixes: the acceptance rule against the Boltzmann factor, the proposal distribution, the cost
bookkeeping against recomputation, the zero-temperature limit, and the stationary distribution of a
constant-temperature chain on a state space small enough to enumerate."""
import math

import numpy as np
import pytest

import oracle
from gen import random_matrix

SEED = 0xC0FFEE77


def test_log2_fix_exact_at_powers_of_two_and_below_true_log():
    for e in range(23):
        assert oracle.sa_log2_fix(1 << e) == e * 4096
    rng = np.random.default_rng(1)
    prev_u, prev_l = 1, 0
    for u in sorted(set(int(x) for x in rng.integers(1, (1 << 22) + 1, size=3000))):
        l = oracle.sa_log2_fix(u)
        true = math.log2(u) * 4096
        assert l <= true + 1e-6                 # chord of a concave function lies below it
        assert true - l <= 0.0861 * 4096 + 1    # largest gap of log2(1+m) - m, plus truncation
        assert l >= prev_l and u > prev_u or u == 1
        prev_u, prev_l = u, l


@pytest.mark.parametrize("delta,temp", [(1, 1), (1, 7), (5, 3), (100, 100), (100, 37), (1000, 150), (12345, 4000),
                                        (3, 100), (2_000_000, 300_000), (40, 2)])
def test_acceptance_probability_tracks_boltzmann_factor(delta, temp):
    """With num = T * steps the rule accepts u <= u*; u*/2^22 must be 2^(-delta/T) up to the chord error of the
    piecewise-linear logarithm (between 1 and 1.0615 times the exact factor) and the 2^-22 grid."""
    steps = 1000
    num = temp * steps
    top = 1 << 22
    assert oracle.sa_accepts(delta, steps, num, 1)         # u = 1 is E = 22: accepts whenever delta/T <= 22
    lo, hi = 1, top + 1                                   # accepts(lo) true, accepts(hi) false (virtual)
    while hi - lo > 1:
        mid = (lo + hi) // 2
        if mid <= top and oracle.sa_accepts(delta, steps, num, mid):
            lo = mid
        else:
            hi = mid
    p_rule = lo / top
    p_true = 2.0 ** (-delta / temp)
    assert p_true * (1 - 1e-3) - 2 / top <= p_rule <= p_true * 1.0625 + 2 / top
    rng = np.random.default_rng(delta)
    for u in rng.integers(1, top + 1, size=200):          # monotone: exactly the u <= u* are accepted
        assert oracle.sa_accepts(delta, steps, num, int(u)) == (int(u) <= lo)


def test_acceptance_special_cases():
    assert oracle.sa_accepts(0, 10, 0, 1 << 22)            # neutral move, zero temperature
    assert oracle.sa_accepts(-5, 10, 0, 1 << 22)
    assert not oracle.sa_accepts(1, 10, 0, 1)              # zero temperature never goes uphill
    assert not oracle.sa_accepts(1, 10, 10 * 1000, 1 << 22)   # u = 2^22 means probability-one events only
    # extremes of the documented limits do not overflow: the largest delta at the largest temperature and step count
    big = 2 * ((1 << 21) - 1)
    steps = 1 << 24
    num = ((1 << 21) - 1) * steps
    assert oracle.sa_accepts(big, steps, num, 1)           # 2^-2 > 2^-22
    assert not oracle.sa_accepts(big, steps, num, 1 << 21)  # 2^-2 < 1/2


@pytest.mark.parametrize("n", [4, 5, 8, 13, 64, 1000])
def test_proposals_are_non_adjacent_edge_pairs_uniformly(n):
    draws = 40000 if n <= 64 else 5000
    a_count = np.zeros(n, dtype=np.int64)
    d_count = np.zeros(n, dtype=np.int64)
    us = []
    for s in range(draws):
        a, b, u = oracle.sa_proposal(SEED, 3, s, n)
        assert 0 <= a < n and 0 <= b < n
        d = (b - a) % n
        assert 2 <= d <= n - 2
        assert 1 <= u <= 1 << 22
        a_count[a] += 1
        d_count[d] += 1
        us.append(u)
    if n <= 64:
        exp_a = draws / n
        assert np.all(np.abs(a_count - exp_a) < 6 * math.sqrt(exp_a))
        exp_d = draws / (n - 3)
        assert np.all(np.abs(d_count[2:n - 1] - exp_d) < 6 * math.sqrt(exp_d))
    assert abs(np.mean(us) / (1 << 21) - 1) < 0.02
    # different chains and steps give different draws
    assert oracle.sa_proposal(SEED, 3, 0, 64) != oracle.sa_proposal(SEED, 4, 0, 64)
    assert oracle.sa_proposal(SEED, 3, 0, 64) != oracle.sa_proposal(SEED + 1, 3, 0, 64)


def test_proposal_uses_the_documented_counter_and_bit_fields():
    """The draw of step s of chain r is output ((r << 32) | (1024 + s)) + 1 of SplitMix64 (itself pinned to the
    published vectors); fields: top 21 bits -> a, next 21 -> distance, low 22 -> u."""
    n = 64
    for r, s in ((0, 0), (5, 17), (1000, 123456)):
        w = oracle.splitmix64_at(SEED, ((r << 32) | (1024 + s)) + 1)
        a = ((w >> 43) * n) >> 21
        d = 2 + ((((w >> 22) & 0x1FFFFF) * (n - 3)) >> 21)
        assert oracle.sa_proposal(SEED, r, s, n) == (a, (a + d) % n, (w & 0x3FFFFF) + 1)


@pytest.mark.parametrize("n,temp", [(6, 0), (9, 50), (16, 400), (64, 300), (64, 0), (100, 2000)])
def test_chain_bookkeeping_against_recomputation(n, temp):
    c = random_matrix(n, 40 + n, symmetric=True, lo=1, hi=3000)
    t0 = oracle.init_tours(SEED, n, 1, first=2)[0]
    steps = 3000
    fast = oracle.sa_chain(c, t0, steps, temp, temp // 4, SEED, 2, trace=True)
    slow = oracle.sa_chain(c, t0, steps, temp, temp // 4, SEED, 2, use_definition=True, trace=True)
    for k in ("final_cost", "best_cost", "accepted"):
        assert fast[k] == slow[k]
    assert np.array_equal(fast["trace"], slow["trace"])
    assert np.array_equal(fast["final_tour"], slow["final_tour"]) and np.array_equal(fast["best_tour"], slow["best_tour"])
    assert sorted(fast["final_tour"]) == list(range(n)) and sorted(fast["best_tour"]) == list(range(n))
    assert fast["final_cost"] == oracle.ring_cost(c, fast["final_tour"]) == fast["trace"][-1]
    assert fast["best_cost"] == oracle.ring_cost(c, fast["best_tour"])
    assert fast["best_cost"] == min(oracle.ring_cost(c, t0), int(fast["trace"].min()))
    assert fast["final_tour"][0] == t0[0]                 # rank 0 is never inside a reversed span
    changes = int(np.count_nonzero(np.diff(np.concatenate([[oracle.ring_cost(c, t0)], fast["trace"]]))))
    assert changes <= fast["accepted"] <= steps
    if temp == 0:
        assert np.all(np.diff(fast["trace"]) <= 0) and fast["final_cost"] == fast["best_cost"]


def test_chain_replayed_move_by_move():
    """Replay with the primitives: proposal -> 2-opt move (i, j) -> value of that move by definition -> acceptance."""
    n, steps, ts, te = 12, 400, 900, 100
    c = random_matrix(n, 5, symmetric=True, lo=1, hi=2500)
    t = oracle.init_tours(SEED, n, 1, first=7)[0].copy()
    res = oracle.sa_chain(c, t, steps, ts, te, SEED, 7, trace=True)
    cur = oracle.ring_cost(c, t)
    best, best_t, acc = cur, t.copy(), 0
    for s in range(steps):
        a, b, u = oracle.sa_proposal(SEED, 7, s, n)
        lo, hi = min(a, b), max(a, b)
        i, j = (lo, hi - 1) if lo else (hi, n - 1)
        new = oracle.move_value_by_definition(c, oracle.SUM, t, i, j)
        if oracle.sa_accepts(new - cur, steps, ts * (steps - s) + te * s, u):
            t = oracle.apply_move(t, i, j)
            cur = new
            acc += 1
            if cur < best:
                best, best_t = cur, t.copy()
        assert res["trace"][s] == cur
    assert (res["best_cost"], res["accepted"]) == (best, acc)
    assert np.array_equal(res["best_tour"], best_t) and np.array_equal(res["final_tour"], t)


def test_constant_temperature_chain_samples_the_boltzmann_distribution():
    """N = 5: 12 undirected rings, each reached by two of the 24 orders with rank 0 fixed; the proposal is
    symmetric, so a chain at constant T visits ring states with probability proportional to 2^(-cost/T), up to
    the 6 % chord error of the acceptance rule."""
    n, temp, steps = 5, 60, 1 << 21
    c = random_matrix(n, 77, symmetric=True, lo=10, hi=200)
    ex = oracle.exhaustive_rings(c, oracle.SUM, half_only=True, keep_all=True)
    ring_costs = np.asarray(ex["costs"], dtype=np.int64)
    assert ring_costs.size == 12
    levels, mult = np.unique(ring_costs, return_counts=True)
    weights = mult * 2.0 ** (-(levels - levels.min()) / temp)
    want = weights / weights.sum()
    t0 = oracle.init_tours(SEED, n, 1)[0]
    res = oracle.sa_chain(c, t0, steps, temp, temp, SEED, 0, trace=True)
    tr = res["trace"][steps // 64:]                        # drop the burn-in
    got = np.array([(tr == lv).mean() for lv in levels])
    assert abs(got.sum() - 1) < 1e-12                      # every visited cost is a ring's cost
    for g, w in zip(got, want):
        if w > 0.01:
            assert abs(g / w - 1) < 0.12, (got, want)
    assert got[0] > got[-1]                                # cheaper rings are visited more often


def test_degenerate_inputs_and_limits():
    c = random_matrix(8, 3, symmetric=True)
    t0 = oracle.init_tours(SEED, 8, 1)[0]
    r = oracle.sa_chain(c, t0, 0, 100, 10, SEED, 0)
    assert np.array_equal(r["best_tour"], t0) and r["accepted"] == 0 and r["best_cost"] == oracle.ring_cost(c, t0)
    c3 = random_matrix(3, 3, symmetric=True)
    t3 = oracle.init_tours(SEED, 3, 1)[0]
    r = oracle.sa_chain(c3, t3, 50, 100, 10, SEED, 0)
    assert np.array_equal(r["best_tour"], t3) and r["accepted"] == 0
    with pytest.raises(RuntimeError):
        oracle.sa_chain(c, t0, (1 << 24) + 1, 1, 1, SEED, 0)
    with pytest.raises(RuntimeError):
        oracle.sa_chain(c, t0, 10, 1 << 21, 1, SEED, 0)
    with pytest.raises(RuntimeError):
        oracle.sa_chains(random_matrix(8, 3, symmetric=False), 10, 1, 1, SEED, 0, 2)


def test_chains_match_single_chain_calls_and_search_picks_lowest():
    n = 16
    c = random_matrix(n, 21, symmetric=True, lo=1, hi=4000)
    costs, tours, accepted = oracle.sa_chains(c, 2000, 500, 0, SEED, 3, 9)
    for k, r in enumerate(range(3, 9)):
        one = oracle.sa_chain(c, oracle.init_tours(SEED, n, 1, first=r)[0], 2000, 500, 0, SEED, r)
        assert one["best_cost"] == costs[k] and np.array_equal(one["best_tour"], tours[k]) and one["accepted"] == accepted[k]
    res = oracle.sa_search(c, 12, 2000, 500, 0, SEED)
    assert res["best_cost"] == res["costs"].min() and res["best_chain"] == int(np.flatnonzero(res["costs"] == res["costs"].min())[0])
    # annealing from a hot start ends no worse than the best it reports, and helps on average against the start
    starts = oracle.ring_cost_batch(c, oracle.init_tours(SEED, n, 12))
    assert res["costs"].mean() < starts.mean()


# ------------------------------------------------------------------------- halving-doubling model, pair neighbour
@pytest.mark.parametrize("n", [2, 4, 8, 64, 1024])
def test_rd_proposals_are_uniform_ordered_pairs(n):
    draws = 30000 if n <= 64 else 3000
    p_count = np.zeros(n, dtype=np.int64)
    d_count = np.zeros(n, dtype=np.int64)
    for s in range(draws):
        p, q, u = oracle.sa_rd_proposal(SEED, 1, s, n)
        assert 0 <= p < n and 0 <= q < n and p != q and 1 <= u <= 1 << 22
        p_count[p] += 1
        d_count[(q - p) % n] += 1
    if n <= 64:
        assert np.all(np.abs(p_count - draws / n) < 6 * math.sqrt(draws / n))
        if n > 2:
            e = draws / (n - 1)
            assert np.all(np.abs(d_count[1:] - e) < 6 * math.sqrt(e))
    # same random word as the ring chain's step: only the use of its first two fields differs
    w = oracle.splitmix64_at(SEED, ((1 << 32) | (1024 + 5)) + 1)
    p = ((w >> 43) * n) >> 21
    d = 1 + ((((w >> 22) & 0x1FFFFF) * (n - 1)) >> 21)
    assert oracle.sa_rd_proposal(SEED, 1, 5, n) == (p, (p + d) % n, (w & 0x3FFFFF) + 1)


@pytest.mark.parametrize("n,temp", [(2, 50), (4, 0), (8, 100), (16, 300), (64, 200), (64, 0)])
def test_rd_chain_replayed_and_bookkept(n, temp):
    c = random_matrix(n, 90 + n, symmetric=False, lo=1, hi=3000)
    t0 = oracle.init_tours(SEED, n, 1, first=4)[0]
    steps, te = 1500, temp // 3
    res = oracle.sa_rd_chain(c, t0, steps, temp, te, SEED, 4, trace=True)
    t = t0.copy()
    cur = oracle.rd_cost(c, t)
    best, best_t, acc = cur, t.copy(), 0
    for s in range(steps):
        p, q, u = oracle.sa_rd_proposal(SEED, 4, s, n)
        new = oracle.rd_swap_value_by_definition(c, t, min(p, q), max(p, q))
        if oracle.sa_accepts(new - cur, steps, temp * (steps - s) + te * s, u):
            t[p], t[q] = t[q], t[p]
            cur = new
            acc += 1
            if cur < best:
                best, best_t = cur, t.copy()
        assert res["trace"][s] == cur
    assert (res["best_cost"], res["accepted"], res["final_cost"]) == (best, acc, cur)
    assert np.array_equal(res["best_tour"], best_t) and np.array_equal(res["final_tour"], t)
    assert res["final_cost"] == oracle.rd_cost(c, res["final_tour"]) and res["best_cost"] == oracle.rd_cost(c, res["best_tour"])
    if temp == 0:
        assert np.all(np.diff(res["trace"]) <= 0)


def test_rd_constant_temperature_chain_samples_the_boltzmann_distribution():
    """N = 4: all 24 orders are states, the swap proposal is symmetric, so at constant T the chain visits a state
    with probability proportional to 2^(-cost/T) (up to the chord error of the acceptance rule)."""
    import itertools
    n, temp, steps = 4, 70, 1 << 21
    c = random_matrix(n, 31, symmetric=False, lo=10, hi=300)
    all_costs = np.array([oracle.rd_cost(c, np.array(pm, dtype=np.int32)) for pm in itertools.permutations(range(n))])
    levels, mult = np.unique(all_costs, return_counts=True)
    weights = mult * 2.0 ** (-(levels - levels.min()) / temp)
    want = weights / weights.sum()
    res = oracle.sa_rd_chain(c, np.arange(n), steps, temp, temp, SEED, 0, trace=True)
    tr = res["trace"][steps // 64:]
    got = np.array([(tr == lv).mean() for lv in levels])
    assert abs(got.sum() - 1) < 1e-12
    for g, w in zip(got, want):
        if w > 0.01:
            assert abs(g / w - 1) < 0.12, (got, want)


def test_rd_chains_and_limits():
    n = 16
    c = random_matrix(n, 12, symmetric=True, lo=1, hi=4000)
    costs, tours, accepted = oracle.sa_rd_chains(c, 1500, 400, 0, SEED, 2, 7)
    for k, r in enumerate(range(2, 7)):
        one = oracle.sa_rd_chain(c, oracle.init_tours(SEED, n, 1, first=r)[0], 1500, 400, 0, SEED, r)
        assert one["best_cost"] == costs[k] and np.array_equal(one["best_tour"], tours[k]) and one["accepted"] == accepted[k]
    res = oracle.sa_rd_search(c, 10, 1500, 400, 0, SEED)
    assert res["best_cost"] == res["costs"].min()
    assert res["costs"].mean() < oracle.rd_cost_batch(c, oracle.init_tours(SEED, n, 10)).mean()
    with pytest.raises(RuntimeError):
        oracle.sa_rd_chain(random_matrix(12, 1, symmetric=True), np.arange(12), 10, 1, 1, SEED, 0)   # not a power of two
    r0 = oracle.sa_rd_chain(c, np.arange(n), 0, 5, 5, SEED, 0)
    assert np.array_equal(r0["best_tour"], np.arange(n)) and r0["accepted"] == 0
